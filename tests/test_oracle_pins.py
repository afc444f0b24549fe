"""Pins of the CPU oracle against things other than itself (CPU only).

P1  Fig. 2 of the paper: emissions implied by the printed alignments, and the
    predictor / joiner call counts of Algorithms 2 and 3.
P2  dense float64 lattice (library matmuls, scipy log-softmax): every oracle
    decision is the lattice argmax, frames / score / termination agree.
P3  Algorithm 1 == Algorithm 3 (== Algorithm 2 for plain Transducers): the
    test-side label-looping and batched frame-looping decoders, built on the
    oracle's row primitives, give the oracle's hypotheses.
P4  predictor switched off: closed form per frame.
P5  TDT with durations {0} is exactly a plain Transducer.
P6  TDT with durations {1}: one decision per frame.
P7  blank bias +-1e4: empty output / len*S labels.
P8  independence of rows, permutation, causality in the length.
P9  structural invariants.
"""
from __future__ import annotations

import numpy as np
import pytest

import chunks
import dense_lattice
import fig2_model
import loops
from paper_2406_06220_amd import synth


def _setup(oracle, cfg, bias=None):
    w = synth.generate_model(cfg, blank_bias_override=bias)
    enc, ln = synth.generate_inputs(cfg)
    return w, enc, ln, oracle.OracleModel(cfg, w)


SMALL = [
    synth.small_config("s_rnnt_stateless1"),
    synth.small_config("s_rnnt_stateless2", pred_layers=2, emb_dim=4, h_pred=8, seed=12),
    synth.small_config("s_rnnt_lstm1", pred_kind="lstm", seed=13, default_blank_bias=0.7),
    synth.small_config("s_rnnt_lstm2", pred_kind="lstm", pred_layers=2, seed=14,
                       default_blank_bias=0.5),
    synth.small_config("s_tdt_stateless", durations=(0, 1, 2, 3, 4), seed=15,
                       default_blank_bias=0.3),
    synth.small_config("s_tdt_lstm2", pred_kind="lstm", pred_layers=2, durations=(0, 1, 2, 3, 4),
                       seed=16, B=5, T=20, len_lo=0, len_hi=20, default_blank_bias=0.2),
    synth.small_config("s_tdt_no01", pred_kind="lstm", durations=(2, 3), seed=17,
                       default_blank_bias=0.0),
    synth.small_config("s_rnnt_lstm3", pred_kind="lstm", pred_layers=3, seed=19,
                       default_blank_bias=0.5),
    synth.small_config("s_tdt_lstm4", pred_kind="lstm", pred_layers=4, durations=(0, 1, 2), seed=20,
                       h_pred=16, emb_dim=8, default_blank_bias=0.3),
    synth.small_config("s_bf16_lstm", dtype="bf16", pred_kind="lstm", seed=18, d_enc=16,
                       h_pred=16, emb_dim=16, h_joint=24, vocab=11, default_blank_bias=0.6),
    # multi-blank Transducers: the durations are big blanks of the label head
    synth.small_config("s_mb_lstm", pred_kind="lstm", durations=(2, 4), multi_blank=True, seed=31,
                       T=24, len_lo=10, len_hi=24, B=4, default_blank_bias=0.6),
    synth.small_config("s_mb_stateless2", pred_layers=2, emb_dim=4, h_pred=8, durations=(2, 3, 5),
                       multi_blank=True, seed=32, T=24, len_lo=0, len_hi=24, B=5,
                       default_blank_bias=0.4),
]
IDS = [c.name for c in SMALL]


# --------------------------------------------------------------------------- P1
def test_fig2_emissions_and_call_counts(oracle_lib):
    ex = fig2_model.build()
    V, vals = ex["V"], ex["vals"]
    lens = [ex["T"]] * ex["B"]
    # the caption's example: CAT / DOG over 4 frames
    names = [[ex["tokens"][k] + "@" + str(t) for k, t in em] for em in ex["expected"]]
    assert names == [["C@0", "A@2", "T@2"], ["D@1", "O@3", "G@3"]]

    ll = loops.label_looping(fig2_model.scripted_fns(ex), lens, 10, 16)
    fl = loops.frame_looping_batched(fig2_model.scripted_fns(ex), lens, 10, 16)
    for b, em in enumerate(ex["expected"]):
        n = len(em)
        assert ll["len"][b] == n and fl["len"][b] == n
        assert list(zip(ll["labels"][b, :n], ll["frames"][b, :n])) == em
        assert list(zip(fl["labels"][b], fl["frames"][b])) == em
    assert ll["n_pred"] == vals["label_looping_predictor_calls"]
    assert ll["n_joint"] == vals["label_looping_joiner_calls"]
    assert fl["n_pred"] == vals["frame_looping_predictor_calls"]
    assert fl["n_joint"] == vals["frame_looping_joiner_calls"]

    # the same example through the oracle proper, on real weights
    cfg, w, enc, ln = fig2_model.real_model(ex)
    m = oracle_lib.OracleModel(cfg, w)
    r = oracle_lib.decode_batch(m, enc, ln, cfg.max_symbols, 16)
    for b, em in enumerate(ex["expected"]):
        n = r["len"][b]
        assert list(zip(r["labels"][b, :n], r["frames"][b, :n])) == em
        # Algorithm 1 makes one joiner call per alignment symbol
        assert r["n_joint"][b] == len(ex["aligns"][b])
        assert r["n_pred"][b] == len(em) + 1
    # label-looping on the oracle's primitives: same hypotheses, same counts
    ll2 = loops.label_looping(loops.oracle_fns(m, enc), ln, cfg.max_symbols, 16)
    assert ll2["n_pred"] == vals["label_looping_predictor_calls"]
    assert ll2["n_joint"] == vals["label_looping_joiner_calls"]
    for b in range(ex["B"]):
        n = r["len"][b]
        assert ll2["len"][b] == n
        assert (ll2["labels"][b, :n] == r["labels"][b, :n]).all()
        assert (ll2["frames"][b, :n] == r["frames"][b, :n]).all()


# --------------------------------------------------------------------------- P2
@pytest.mark.parametrize("cfg", SMALL + [synth.CFG1], ids=IDS + ["cfg1"])
def test_dense_lattice_brute_force(oracle_lib, cfg):
    w, enc, ln, m = _setup(oracle_lib, cfg)
    u_cap = cfg.T * cfg.max_symbols
    n_checked = 0
    for b in range(cfg.B):
        r = oracle_lib.decode_utt(m, enc[b], int(ln[b]), cfg.max_symbols, u_cap, trace=True)
        lat = dense_lattice.lattice(cfg, w, enc[b], r["labels"])
        walk = dense_lattice.greedy_walk(cfg, lat, int(ln[b]), u_cap)
        if walk["min_margin"] < 1e-4:       # a float64/float32 near-tie proves nothing
            continue
        n_checked += 1
        assert walk["labels"] == r["labels"].tolist()
        assert walk["frames"] == r["frames"].tolist()
        assert walk["end_u"] == r["len"] and walk["end_t"] >= ln[b]
        assert walk["n_dec"] == r["n_joint"] == len(r["trace"]["t"])
        assert abs(walk["score"] - r["score"]) < 2e-4 * max(1, r["len"])
        # the trace's nodes are the walk's nodes and the recorded margins are the lattice's
        for i in range(len(r["trace"]["t"])):
            t, u = r["trace"]["t"][i], r["trace"]["u"][i]
            head = cfg.n_out if cfg.multi_blank else cfg.vocab + 1
            lab = np.sort(lat[t, u, :head])
            assert abs((lab[-1] - lab[-2]) - r["trace"]["margin_lab"][i]) < 1e-4
        # the exported single-node routine agrees with the lattice
        for (t, u) in [(0, 0), (int(ln[b]) - 1, r["len"])] if ln[b] > 0 else []:
            lg = m.lattice_logits(enc[b, t], r["labels"], u)
            np.testing.assert_allclose(lg, lat[t, u], atol=2e-5, rtol=1e-5)
    assert n_checked >= max(1, cfg.B - 1)


# --------------------------------------------------------------------------- P3
@pytest.mark.parametrize("cfg", SMALL + [synth.CFG1], ids=IDS + ["cfg1"])
def test_label_looping_equals_frame_looping(oracle_lib, cfg):
    w, enc, ln, m = _setup(oracle_lib, cfg)
    for u_cap in (cfg.T * cfg.max_symbols, 4):
        r = oracle_lib.decode_batch(m, enc, ln, cfg.max_symbols, u_cap)
        ll = loops.label_looping(loops.oracle_fns(m, enc), ln, cfg.max_symbols, u_cap)
        assert (ll["len"] == r["len"]).all()
        for b in range(cfg.B):
            n = r["len"][b]
            assert (ll["labels"][b, :n] == r["labels"][b, :n]).all()
            assert (ll["frames"][b, :n] == r["frames"][b, :n]).all()
        np.testing.assert_allclose(ll["score"], r["score"], atol=1e-4)
        # Sec. 3.2: predictor calls = longest hypothesis (+1 for BOS, unless the longest
        # hypothesis went inactive together with its last label)
        if cfg.B and ln.max() > 0 and u_cap > 4:
            assert ll["n_pred"] in (r["len"].max(), r["len"].max() + 1)
        if not cfg.durations:
            fl = loops.frame_looping_batched(loops.oracle_fns(m, enc), ln, cfg.max_symbols, u_cap)
            assert (fl["len"] == r["len"]).all()
            for b in range(cfg.B):
                n = r["len"][b]
                assert fl["labels"][b] == r["labels"][b, :n].tolist()
                assert fl["frames"][b] == r["frames"][b, :n].tolist()
            # the point of the method: never more predictor calls than the baseline
            assert ll["n_pred"] <= fl["n_pred"]


# --------------------------------------------------------------------------- P4
@pytest.mark.parametrize("durations", [(), (0, 1, 2, 3, 4)], ids=["rnnt", "tdt"])
def test_predictor_off_closed_form(oracle_lib, durations):
    cfg = synth.small_config("p4", pred_kind="lstm", durations=durations, T=30, len_lo=20,
                             len_hi=30, seed=21, default_blank_bias=0.8, max_symbols=3)
    w = synth.generate_model(cfg)
    w["w_pred"][:] = 0.0
    w["b_pred"][:] = 0.0
    enc, ln = synth.generate_inputs(cfg)
    m = oracle_lib.OracleModel(cfg, w)
    r = oracle_lib.decode_batch(m, enc, ln, cfg.max_symbols, cfg.T * cfg.max_symbols)
    V, S = cfg.vocab, cfg.max_symbols
    for b in range(cfg.B):
        hid = np.maximum(enc[b].astype(np.float64) @ w["w_enc"].T.astype(np.float64), 0.0)
        lg = hid @ w["w_out"].T.astype(np.float64) + w["b_out"]
        k = lg[:, : V + 1].argmax(1)
        exp_l, exp_f = [], []
        if not durations:
            for t in range(ln[b]):
                if k[t] != V:
                    exp_l += [k[t]] * S
                    exp_f += [t] * S
        else:
            d = np.asarray(durations)[lg[:, V + 1:].argmax(1)]
            t = sym = 0
            while t < ln[b]:
                if k[t] == V:
                    t += max(d[t], 1)
                    sym = 0
                else:
                    exp_l.append(k[t])
                    exp_f.append(t)
                    sym += 1
                    step = 1 if (d[t] == 0 and sym >= S) else d[t]
                    if step > 0:
                        t += step
                        sym = 0
        n = r["len"][b]
        assert r["labels"][b, :n].tolist() == exp_l
        assert r["frames"][b, :n].tolist() == exp_f


# --------------------------------------------------------------------------- P5
def test_tdt_zero_duration_is_rnnt(oracle_lib):
    cfg_r = synth.small_config("p5", pred_kind="lstm", T=25, len_lo=10, len_hi=25, seed=22,
                               default_blank_bias=0.6)
    cfg_t = synth.small_config("p5", pred_kind="lstm", T=25, len_lo=10, len_hi=25, seed=22,
                               default_blank_bias=0.6, durations=(0,))
    w_t = synth.generate_model(cfg_t)
    w_r = dict(w_t, w_out=w_t["w_out"][: cfg_r.vocab + 1].copy(),
               b_out=w_t["b_out"][: cfg_r.vocab + 1].copy())
    enc, ln = synth.generate_inputs(cfg_t)
    u_cap = cfg_r.T * cfg_r.max_symbols
    rt = oracle_lib.decode_batch(oracle_lib.OracleModel(cfg_t, w_t), enc, ln, cfg_t.max_symbols, u_cap)
    rr = oracle_lib.decode_batch(oracle_lib.OracleModel(cfg_r, w_r), enc, ln, cfg_r.max_symbols, u_cap)
    assert rr["len"].sum() > 0
    for key in ("labels", "frames", "len", "score", "n_joint", "n_pred"):
        assert (rt[key] == rr[key]).all(), key


# --------------------------------------------------------------------------- P6
def test_tdt_unit_duration_one_decision_per_frame(oracle_lib):
    cfg = synth.small_config("p6", pred_kind="lstm", durations=(1,), T=25, len_lo=10, len_hi=25,
                             seed=23, default_blank_bias=0.3)
    w, enc, ln, m = _setup(oracle_lib, cfg)
    r = oracle_lib.decode_batch(m, enc, ln, cfg.max_symbols, cfg.T * cfg.max_symbols)
    assert (r["n_joint"] == ln).all()
    assert r["len"].sum() > 0
    for b in range(cfg.B):
        f = r["frames"][b, : r["len"][b]]
        assert (np.diff(f) >= 1).all()


# --------------------------------------------------------------------------- P7
def test_extreme_blank_bias(oracle_lib):
    cfg = synth.small_config("p7", pred_kind="lstm", T=15, len_lo=0, len_hi=15, seed=24, B=6)
    S = cfg.max_symbols
    w, enc, ln, m = _setup(oracle_lib, cfg, bias=1e4)
    r = oracle_lib.decode_batch(m, enc, ln, S, cfg.T * S)
    assert (r["len"] == 0).all() and (r["score"] == 0).all() and (r["n_joint"] == ln).all()
    w, enc, ln, m = _setup(oracle_lib, cfg, bias=-1e4)
    r = oracle_lib.decode_batch(m, enc, ln, S, cfg.T * S)
    assert (r["len"] == ln * S).all() and (r["status"] == (ln == cfg.T)).all()
    for b in range(cfg.B):
        assert r["frames"][b, : r["len"][b]].tolist() == np.repeat(np.arange(ln[b]), S).tolist()
    # a capacity below len*S stops the hypothesis and says so
    r = oracle_lib.decode_batch(m, enc, ln, S, 7)
    assert (r["len"] == np.minimum(ln * S, 7)).all()
    assert (r["status"] == (ln * S >= 7)).all()


# --------------------------------------------------------------------------- P8
@pytest.mark.parametrize("cfg", [SMALL[2], SMALL[5]], ids=[SMALL[2].name, SMALL[5].name])
def test_rows_independent_permutable_causal(oracle_lib, cfg):
    w, enc, ln, m = _setup(oracle_lib, cfg)
    S, u_cap = cfg.max_symbols, cfg.T * cfg.max_symbols
    r = oracle_lib.decode_batch(m, enc, ln, S, u_cap)
    perm = np.random.default_rng(0).permutation(cfg.B)
    rp = oracle_lib.decode_batch(m, enc[perm], ln[perm], S, u_cap)
    for i, b in enumerate(perm):
        n = r["len"][b]
        assert rp["len"][i] == n and rp["score"][i] == r["score"][b]
        assert (rp["labels"][i, :n] == r["labels"][b, :n]).all()
        one = oracle_lib.decode_utt(m, enc[b], int(ln[b]), S, u_cap)
        assert one["len"] == n and (one["labels"] == r["labels"][b, :n]).all()
        # other rows' content, and this row's padding, never matter
        noisy = enc[b].copy()
        noisy[ln[b]:] += 100.0
        two = oracle_lib.decode_utt(m, noisy, int(ln[b]), S, u_cap)
        assert (two["labels"] == one["labels"]).all() and two["score"] == one["score"]
        # causality: a shorter length keeps exactly the emissions found before it
        for cut in range(0, int(ln[b]) + 1, 3):
            short = oracle_lib.decode_utt(m, enc[b], cut, S, u_cap)
            keep = r["frames"][b, :n] < cut
            assert short["labels"].tolist() == r["labels"][b, :n][keep].tolist()
            assert short["frames"].tolist() == r["frames"][b, :n][keep].tolist()


# --------------------------------------------------------------------------- P9
@pytest.mark.parametrize("cfg", SMALL + [synth.CFG1], ids=IDS + ["cfg1"])
def test_structural_invariants(oracle_lib, cfg):
    w, enc, ln, m = _setup(oracle_lib, cfg)
    S = cfg.max_symbols
    r = oracle_lib.decode_batch(m, enc, ln, S, cfg.T * S)
    assert r["len"].sum() > 0
    for b in range(cfg.B):
        n = r["len"][b]
        lab, fr, du = r["labels"][b, :n], r["frames"][b, :n], r["durs"][b, :n]
        assert ((lab >= 0) & (lab < cfg.vocab)).all()
        assert (np.diff(fr) >= 0).all() and (fr < ln[b]).all() and (fr >= 0).all()
        assert r["score"][b] <= 0.0
        assert r["n_pred"][b] == n + 1
        # frame index moves exactly by the recorded advance of each label, blanks add more
        assert (np.diff(fr) >= du[:-1]).all()
        # never more than S labels without the frame index moving
        run = 0
        for i in range(n):
            run = run + 1 if (i > 0 and fr[i] == fr[i - 1] and du[i - 1] == 0) else 1
            assert run <= S
        if not cfg.durations:
            assert r["n_joint"][b] == ln[b] + n - int((du > 0).sum())


def test_cfg1_matches_recorded_statistics(oracle_lib):
    """Config 1 keeps the stated +2.0 bias; its realised blank share is what the
    calibration script recorded (about 70%)."""
    cfg = synth.CFG1
    w, enc, ln, m = _setup(oracle_lib, cfg)
    r = oracle_lib.decode_batch(m, enc, ln, cfg.max_symbols, cfg.T * cfg.max_symbols)
    frac = 1.0 - r["len"].sum() / r["n_joint"].sum()
    assert 0.6 < frac < 0.8


# --------------------------------------------------------------------------- replay
def test_replay_accepts_exact_and_rejects_edits(oracle_lib):
    for cfg in (SMALL[2], SMALL[5]):
        w, enc, ln, m = _setup(oracle_lib, cfg)
        S, u_cap = cfg.max_symbols, cfg.T * cfg.max_symbols
        r = oracle_lib.decode_batch(m, enc, ln, S, u_cap)
        for b in range(cfg.B):
            n = r["len"][b]
            lab, fr = r["labels"][b, :n], r["frames"][b, :n]
            ok = oracle_lib.replay_utt(m, enc[b], int(ln[b]), S, u_cap, lab, fr, tol=1e-6)
            assert ok["ok"] and ok["n_tie"] == 0 and abs(ok["score"] - r["score"][b]) < 1e-5
            if n == 0:
                continue
            bad = lab.copy()
            bad[n // 2] = (bad[n // 2] + 1) % cfg.vocab
            assert not oracle_lib.replay_utt(m, enc[b], int(ln[b]), S, u_cap, bad, fr)["ok"]
            assert not oracle_lib.replay_utt(m, enc[b], int(ln[b]), S, u_cap, lab[:-1], fr[:-1])["ok"]
            badf = fr.copy()
            badf[0] += 1
            assert not oracle_lib.replay_utt(m, enc[b], int(ln[b]), S, u_cap, lab, badf)["ok"]


def test_replay_tolerates_only_near_ties(oracle_lib):
    cfg = synth.small_config("tie", pred_kind="lstm", T=20, len_lo=20, len_hi=20, seed=31, B=2,
                             default_blank_bias=0.4)
    w = synth.generate_model(cfg)
    enc, ln = synth.generate_inputs(cfg)
    S, u_cap = cfg.max_symbols, cfg.T * cfg.max_symbols
    base = oracle_lib.decode_batch(oracle_lib.OracleModel(cfg, w), enc, ln, S, u_cap)
    a = int(np.bincount(base["labels"][0, : base["len"][0]], minlength=cfg.vocab).argmax())
    z = (a + 1) % cfg.vocab
    # label z becomes a copy of label a lifted by 5e-4: every win of z over a is a near-tie
    w["w_out"][z] = w["w_out"][a]
    w["b_out"][z] = w["b_out"][a] + 5e-4
    m = oracle_lib.OracleModel(cfg, w)
    hit = 0
    for b in range(cfg.B):
        r = oracle_lib.decode_utt(m, enc[b], int(ln[b]), S, u_cap, trace=True)
        assert (r["labels"] != a).all()
        pos = np.nonzero(r["labels"] == z)[0]
        if len(pos) == 0:
            continue
        hit += 1
        tr = r["trace"]
        assert (tr["margin_lab"][tr["k"] == z] < 1e-3).all()      # flagged in the trace
        # Candidate: the oracle's hypothesis up to and including the first z, with that z
        # swapped for its twin a.  With a capacity of exactly that many labels the decode
        # stops there, so what follows the swapped label does not matter.
        p = int(pos[0])
        cand, fr = r["labels"][: p + 1].copy(), r["frames"][: p + 1]
        cand[p] = a
        got = oracle_lib.replay_utt(m, enc[b], int(ln[b]), S, p + 1, cand, fr, tol=1e-3)
        assert got["ok"] and got["n_tie"] == 1
        assert not oracle_lib.replay_utt(m, enc[b], int(ln[b]), S, p + 1, cand, fr, tol=1e-4)["ok"]
        # and the unswapped prefix needs no tolerance at all
        exact = oracle_lib.replay_utt(m, enc[b], int(ln[b]), S, p + 1, r["labels"][: p + 1], fr,
                                      tol=0.0)
        assert exact["ok"] and exact["n_tie"] == 0
    assert hit >= 1


def test_replay_tolerates_near_ties_of_the_duration_head(oracle_lib):
    """The TDT twin of the test above (Sec. 3.3: the frame step comes from the duration head).  The
    class of duration 2 is a copy of the class of duration 1, in model A lifted by 5e-4 (so 2 wins
    wherever the pair is on top), in model B lowered by 5e-4 (1 wins).  The label logits are the same
    in both, so B's hypothesis is a greedy decode of A up to near-ties of the duration head: A's
    replay accepts it at a tolerance of 1e-3, counting the ties, and rejects it at 1e-4."""
    cfg = synth.small_config("tie_dur", pred_kind="lstm", durations=(0, 1, 2), T=24, len_lo=24, len_hi=24,
                             seed=33, B=3, default_blank_bias=0.4)
    V = cfg.vocab
    wa = synth.generate_model(cfg)
    wa["w_out"][V + 1 + 2] = wa["w_out"][V + 1 + 1]
    wa["b_out"][V + 1 + 1] = wa["b_out"][V + 1 + 2] = 2.0      # the pair is usually on top
    wb = {k: v.copy() for k, v in wa.items()}
    wa["b_out"][V + 1 + 2] += 5e-4
    wb["b_out"][V + 1 + 2] -= 5e-4
    enc, ln = synth.generate_inputs(cfg)
    S, u_cap = cfg.max_symbols, cfg.T * cfg.max_symbols
    ma, mb = oracle_lib.OracleModel(cfg, wa), oracle_lib.OracleModel(cfg, wb)
    ra = oracle_lib.decode_batch(ma, enc, ln, S, u_cap)
    rb = oracle_lib.decode_batch(mb, enc, ln, S, u_cap)
    differ = 0
    for b in range(cfg.B):
        na, nb = ra["len"][b], rb["len"][b]
        lab, fr = rb["labels"][b, :nb], rb["frames"][b, :nb]
        same = na == nb and (lab == ra["labels"][b, :na]).all() and (fr == ra["frames"][b, :na]).all()
        got = oracle_lib.replay_utt(ma, enc[b], int(ln[b]), S, u_cap, lab, fr, tol=1e-3)
        assert got["ok"], b
        assert abs(got["score"] - rb["score"][b]) < 1e-4      # the label logits are the same
        if same:
            continue
        differ += 1
        assert got["n_tie"] >= 1
        assert not oracle_lib.replay_utt(ma, enc[b], int(ln[b]), S, u_cap, lab, fr, tol=1e-4)["ok"]
    assert differ >= 1


# --------------------------------------------------------------------------- P11
# Piecewise decoding (an extension beyond the paper) is defined by one requirement:
# the chunks of an utterance, decoded in order with the carried state, give the
# hypothesis of the whole utterance.  The whole-utterance decoder is pinned above.
@pytest.mark.parametrize("mode,n_chunks", [("random", 4), ("random", 9), ("even", 2), ("single", 0)],
                         ids=["random4", "random9", "halves", "frame_by_frame"])
@pytest.mark.parametrize("cfg", SMALL + [synth.CFG1], ids=IDS + ["cfg1"])
def test_chunks_decode_like_the_whole(oracle_lib, cfg, mode, n_chunks):
    w, enc, ln, m = _setup(oracle_lib, cfg)
    S, u_cap = cfg.max_symbols, cfg.T * cfg.max_symbols
    whole = oracle_lib.decode_batch(m, enc, ln, S, u_cap)
    rng = np.random.default_rng(100 + n_chunks)
    bounds = chunks.split_plan(ln, n_chunks, rng, mode)
    state = oracle_lib.stream_state(m, cfg.B)
    parts = []
    for c in range(bounds.shape[1] - 1):
        ec, lc = chunks.make_chunk(enc, bounds, c, rng)
        parts.append(oracle_lib.decode_batch_chunk(m, ec, lc, S, u_cap, state))
        # what is carried over is how far the last step reached past the chunk's end
        assert (state["time"] >= 0).all()
        assert (state["time"] <= (max(cfg.durations) if cfg.durations else 1)).all()
    got = chunks.stitch(parts, bounds, u_cap)
    assert (got["len"] == whole["len"]).all()
    for b in range(cfg.B):
        n = whole["len"][b]
        assert (got["labels"][b, :n] == whole["labels"][b, :n]).all()
        assert (got["frames"][b, :n] == whole["frames"][b, :n]).all()
    np.testing.assert_allclose(got["score"], whole["score"], rtol=0, atol=2e-5 * (1 + whole["len"].max()))
    # the carried predictor state is the state after start-of-sequence and the emitted labels
    for b in range(cfg.B):
        if ln[b] == 0:
            assert state["started"][b] == 0
            continue
        assert state["started"][b] == 1
        st = m.init_state()
        for lab in [cfg.vocab] + whole["labels"][b, :whole["len"][b]].tolist():
            _, st = m.predictor_step(st, lab)
        if cfg.pred_kind == "lstm":
            n = cfg.pred_layers * cfg.h_pred
            assert (state["h"][b] == st[0][:n]).all() and (state["c"][b] == st[0][n:]).all()
        else:
            assert (state["ctx"][b, :cfg.pred_layers] == st[1][:cfg.pred_layers]).all()


def test_fig2_in_two_chunks(oracle_lib):
    """The caption's example cut between frames 1 and 2: C | A T and D | O G."""
    ex = fig2_model.build()
    cfg, w, enc, ln = fig2_model.real_model(ex)
    m = oracle_lib.OracleModel(cfg, w)
    state = oracle_lib.stream_state(m, ex["B"])
    two = np.full(ex["B"], 2, np.int32)
    first = oracle_lib.decode_batch_chunk(m, enc[:, :2], two, cfg.max_symbols, 16, state)
    second = oracle_lib.decode_batch_chunk(m, enc[:, 2:4], two, cfg.max_symbols, 16, state)
    for b, em in enumerate(ex["expected"]):
        a = [(k, t) for k, t in em if t < 2]
        z = [(k, t - 2) for k, t in em if t >= 2]
        assert list(zip(first["labels"][b, :first["len"][b]], first["frames"][b, :first["len"][b]])) == a
        assert list(zip(second["labels"][b, :second["len"][b]], second["frames"][b, :second["len"][b]])) == z


def test_chunk_stopped_at_capacity_loses_its_rest(oracle_lib):
    """A chunk whose hypothesis fills its label capacity is flagged; the next chunk starts
    at its own first frame with the predictor state of the labels kept so far."""
    cfg = SMALL[2]
    w, enc, ln, m = _setup(oracle_lib, cfg, bias=-3.0)   # many labels
    S = cfg.max_symbols
    state = oracle_lib.stream_state(m, cfg.B)
    r = oracle_lib.decode_batch_chunk(m, enc, ln, S, 3, state)
    assert (r["status"][ln > 0] == 1).all() and (r["len"][ln > 0] == 3).all()
    assert (state["time"] == 0).all()
    for b in range(cfg.B):
        if ln[b] == 0:
            continue
        st = m.init_state()
        for lab in [cfg.vocab] + r["labels"][b, :3].tolist():
            _, st = m.predictor_step(st, lab)
        n = cfg.pred_layers * cfg.h_pred
        assert (state["h"][b] == st[0][:n]).all()


# --------------------------------------------------------------------------- multi-blank
# Multi-blank Transducer (Sec. 1, related work): big-blank symbols in the label head, each with a
# fixed frame increment.  Besides the dense lattice and the label-looping re-ordering above (both
# run on the two multi-blank models of SMALL), the reductions and closed forms below.
def _mb_pair(seed, durs, extra_bias):
    """A plain Transducer and the multi-blank model that has its outputs plus big blanks whose
    rows are given by `extra_bias` (weights zero, so their logits are exactly that bias)."""
    cfg_r = synth.small_config("mb_r", pred_kind="lstm", T=25, len_lo=10, len_hi=25, seed=seed,
                               default_blank_bias=0.6)
    cfg_m = synth.small_config("mb_m", pred_kind="lstm", T=25, len_lo=10, len_hi=25, seed=seed,
                               default_blank_bias=0.6, durations=durs, multi_blank=True)
    w_r = synth.generate_model(cfg_r)
    V, K = cfg_r.vocab, len(durs)
    w_out = np.concatenate([w_r["w_out"], np.zeros((K, cfg_r.h_joint), np.float32)])
    b_out = np.concatenate([w_r["b_out"], np.asarray(extra_bias, np.float32)])
    w_m = dict(w_r, w_out=w_out, b_out=b_out)
    enc, ln = synth.generate_inputs(cfg_r)
    return cfg_r, w_r, cfg_m, w_m, enc, ln


def test_multi_blank_that_never_wins_is_rnnt(oracle_lib):
    # big blanks whose logits are -1e30: never the argmax, exp() of them is exactly 0, so labels,
    # frames, scores and call counts are those of the plain Transducer bit for bit
    cfg_r, w_r, cfg_m, w_m, enc, ln = _mb_pair(41, (2, 7), (-1e30, -1e30))
    u_cap = cfg_r.T * cfg_r.max_symbols
    rr = oracle_lib.decode_batch(oracle_lib.OracleModel(cfg_r, w_r), enc, ln, cfg_r.max_symbols, u_cap)
    rm = oracle_lib.decode_batch(oracle_lib.OracleModel(cfg_m, w_m), enc, ln, cfg_m.max_symbols, u_cap)
    assert rr["len"].sum() > 0
    for key in ("labels", "frames", "len", "score", "n_joint", "n_pred"):
        assert (rm[key] == rr[key]).all(), key


def test_big_blank_of_one_frame_is_the_blank(oracle_lib):
    # one big blank of duration 1 whose row is a copy of the blank's: wherever the blank would win
    # the two tie and the first maximum (the blank) is taken; had the big blank won it would move
    # by one frame all the same.  Labels, frames and call counts equal the plain Transducer's; the
    # score differs by the one more term in every softmax: log(sum exp) grows by
    # log(1 + p_blank), so each emitted label's log-probability drops by exactly that.
    cfg_r, w_r, cfg_m, w_m, enc, ln = _mb_pair(42, (1,), (0.0,))
    V = cfg_r.vocab
    w_m["w_out"][V + 1] = w_m["w_out"][V]
    w_m["b_out"][V + 1] = w_m["b_out"][V]
    u_cap = cfg_r.T * cfg_r.max_symbols
    m_r, m_m = oracle_lib.OracleModel(cfg_r, w_r), oracle_lib.OracleModel(cfg_m, w_m)
    rr = oracle_lib.decode_batch(m_r, enc, ln, cfg_r.max_symbols, u_cap)
    rm = oracle_lib.decode_batch(m_m, enc, ln, cfg_m.max_symbols, u_cap)
    for key in ("labels", "frames", "len", "n_joint", "n_pred"):
        assert (rm[key] == rr[key]).all(), key
    for b in range(cfg_r.B):
        n = rr["len"][b]
        lat = dense_lattice.lattice(cfg_r, w_r, enc[b], rr["labels"][b, :n])
        drop = 0.0
        for u in range(n):
            row = lat[rr["frames"][b, u], u, : V + 1]
            p_blank = np.exp(row[V] - np.logaddexp.reduce(row))
            drop += np.log1p(p_blank)
        assert abs((rr["score"][b] - rm["score"][b]) - drop) < 2e-4 * max(1, n)


def test_multi_blank_predictor_off_closed_form(oracle_lib):
    # with the predictor's projection switched off the logits depend on the frame only, and the
    # hypothesis can be read off a per-frame table: a label frame emits S copies and moves on by
    # one, a blank frame moves by one, big blank i by durations[i]
    durs = (2, 3, 6)
    cfg = synth.small_config("mb_p4", pred_kind="lstm", durations=durs, multi_blank=True, T=40,
                             len_lo=25, len_hi=40, seed=43, default_blank_bias=0.5, max_symbols=3, B=4)
    w = synth.generate_model(cfg)
    w["w_pred"][:] = 0.0
    w["b_pred"][:] = 0.0
    enc, ln = synth.generate_inputs(cfg)
    m = oracle_lib.OracleModel(cfg, w)
    r = oracle_lib.decode_batch(m, enc, ln, cfg.max_symbols, cfg.T * cfg.max_symbols)
    V, S = cfg.vocab, cfg.max_symbols
    seen = set()
    for b in range(cfg.B):
        hid = np.maximum(enc[b].astype(np.float64) @ w["w_enc"].T.astype(np.float64), 0.0)
        k = (hid @ w["w_out"].T.astype(np.float64) + w["b_out"]).argmax(1)
        exp_l, exp_f, t, n_joint = [], [], 0, 0
        while t < ln[b]:
            seen.add(min(int(k[t]), V) if k[t] <= V else int(k[t]))
            if k[t] < V:
                exp_l += [k[t]] * S
                exp_f += [t] * S
                n_joint += S
                t += 1
            else:
                n_joint += 1
                t += 1 if k[t] == V else durs[k[t] - V - 1]
        n = r["len"][b]
        assert r["labels"][b, :n].tolist() == exp_l
        assert r["frames"][b, :n].tolist() == exp_f
        assert r["n_joint"][b] == n_joint
    # the example exercises labels, the blank and at least two of the big blanks
    assert len([x for x in seen if x > V]) >= 2 and V in seen and any(x < V for x in seen)


def test_multi_blank_longest_big_blank_skips_the_utterance(oracle_lib):
    # a big blank that always wins and is as long as the longest utterance: one joint call per
    # utterance, nothing emitted; with increment 3: ceil(len / 3) calls
    for inc in (50, 3):
        cfg = synth.small_config("mb_skip", pred_kind="lstm", durations=(2, inc), multi_blank=True,
                                 T=30, len_lo=0, len_hi=30, seed=44, B=6)
        w = synth.generate_model(cfg)
        w["b_out"][cfg.vocab + 2] = 1e4
        enc, ln = synth.generate_inputs(cfg)
        r = oracle_lib.decode_batch(oracle_lib.OracleModel(cfg, w), enc, ln, cfg.max_symbols, 90)
        assert (r["len"] == 0).all() and (r["score"] == 0).all()
        assert (r["n_joint"] == -(-ln // inc)).all()
        assert (r["n_pred"] == 1).all()


def test_multi_blank_replay(oracle_lib):
    # the tolerant replay accepts the oracle's own multi-blank hypotheses with no tie taken and
    # rejects an edited one
    cfg = SMALL[IDS.index("s_mb_lstm")]
    w, enc, ln, m = _setup(oracle_lib, cfg)
    u_cap = cfg.T * cfg.max_symbols
    r = oracle_lib.decode_batch(m, enc, ln, cfg.max_symbols, u_cap)
    assert r["len"].sum() > 0
    for b in range(cfg.B):
        n = int(r["len"][b])
        got = oracle_lib.replay_utt(m, enc[b], int(ln[b]), cfg.max_symbols, u_cap,
                                    r["labels"][b, :n], r["frames"][b, :n], tol=1e-6)
        assert got["ok"] and got["n_tie"] == 0 and abs(got["score"] - r["score"][b]) < 1e-5
        if n:
            bad = r["frames"][b, :n].copy()
            bad[n - 1] += 1
            assert not oracle_lib.replay_utt(m, enc[b], int(ln[b]), cfg.max_symbols, u_cap,
                                             r["labels"][b, :n], bad)["ok"]
