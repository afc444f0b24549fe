"""The paper's Fig. 2 example as (a) a scripted lookup model and (b) real weights.

(Not collected by pytest.)  The fixture ``golden/fig2_alignments.txt`` holds the
two alignments the figure's caption prints.  From them this module derives

* the decision table  (utterance, frame, last label) -> next symbol,
* the emissions the alignments imply (label, frame), and
* a genuine stateless-predictor Transducer whose greedy decode follows the table:
  encoder features are one-hot over (utterance, frame), embeddings are one-hot
  over the last label, hidden unit (f, l) computes relu(e_f + p_l - 1), i.e. the
  AND of "this frame" and "this last label", and the output layer puts weight 5
  on the scripted symbol of each unit (blank gets bias 1 everywhere else).
"""
from __future__ import annotations

import os
from typing import Dict, List, Tuple

import numpy as np

from paper_2406_06220_amd import synth

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "fig2_alignments.txt")


def load_fixture():
    aligns: Dict[int, List[str]] = {}
    vals: Dict[str, int] = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if line.startswith("alignment"):
                head, body = line.split(":")
                aligns[int(head.split()[1])] = body.split()
            else:
                k, v = line.split()
                vals[k] = int(v)
    return [aligns[i] for i in sorted(aligns)], vals


def build():
    aligns, vals = load_fixture()
    T = vals["frames"]
    tokens = sorted({s for a in aligns for s in a if s != "<b>"})
    tok_id = {s: i for i, s in enumerate(tokens)}
    V = len(tokens)
    B = len(aligns)
    table: Dict[Tuple[int, int, int], int] = {}
    expected = []
    for b, a in enumerate(aligns):
        t, last, em = 0, V, []
        for s in a:
            k = V if s == "<b>" else tok_id[s]
            table[(b, t, last)] = k
            if k == V:
                t += 1
            else:
                em.append((k, t))
                last = k
        assert t == T, "every alignment must consume all frames"
        expected.append(em)
    return dict(aligns=aligns, vals=vals, T=T, B=B, V=V, tokens=tokens, table=table,
                expected=expected)


def scripted_fns(ex):
    """ModelFns for tests/loops.py: the predictor state is just the last label."""
    from loops import ModelFns
    V = ex["V"]

    def joiner(b, t, dec):
        logits = np.zeros(V + 1, np.float32)
        logits[V] = 1.0
        logits[ex["table"].get((b, t, int(dec)), V)] = 5.0
        return logits

    return ModelFns(init_state=lambda: None, predictor=lambda s, label: (label, None),
                    joiner=joiner, vocab=V)


def real_model(ex):
    """(cfg, weights, enc, enc_len) of a Transducer that realises the decision table."""
    V, B, T = ex["V"], ex["B"], ex["T"]
    E = 8 * ((V + 1 + 7) // 8)            # embedding width, padded to a multiple of 8
    F = B * T                             # one-hot frame features
    d_enc = 8 * ((F + 7) // 8)
    H = 8 * ((F * (V + 1) + 7) // 8)
    cfg = synth.small_config(name="fig2", dtype="fp32", B=B, T=T, len_lo=T, len_hi=T, d_enc=d_enc,
                             pred_kind="stateless", pred_layers=1, h_pred=E, emb_dim=E, h_joint=H,
                             vocab=V, durations=(), max_symbols=10)
    w = dict(w_enc=np.zeros((H, d_enc), np.float32), b_enc=np.full(H, -1.0, np.float32),
             emb=np.zeros((1, V + 1, E), np.float32), w_pred=np.zeros((H, E), np.float32),
             b_pred=np.zeros(H, np.float32), w_out=np.zeros((V + 1, H), np.float32),
             b_out=np.zeros(V + 1, np.float32))
    for l in range(V + 1):
        w["emb"][0, l, l] = 1.0
    for f in range(F):
        for l in range(V + 1):
            unit = f * (V + 1) + l
            w["w_enc"][unit, f] = 1.0
            w["w_pred"][unit, l] = 1.0
            k = ex["table"].get((f // T, f % T, l))
            if k is not None:
                w["w_out"][k, unit] = 5.0
    w["b_out"][V] = 1.0
    enc = np.zeros((B, T, d_enc), np.float32)
    for b in range(B):
        for t in range(T):
            enc[b, t, b * T + t] = 1.0
    return cfg, w, enc, np.full(B, T, np.int32)
