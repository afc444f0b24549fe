"""Host logic that needs no GPU: the benchmark's bookkeeping, the seeded generators, the chunk
helpers of the tests."""
from __future__ import annotations

import os
import subprocess
import sys

import numpy as np
import torch

import chunks
from paper_2406_06220_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_algorithmic_bytes_closed_form():
    """The two byte counts of the roofline figure, retyped for config 2 (one LSTM layer whose input
    product is a per-label table, so only its recurrent matrix is streamed) and for the stateless
    config 4 (no predictor-side matrix at all: two table rows per scored row)."""
    import bench
    cfg = synth.CONFIGS["cfg2_rnnt_lstm"]
    stats = dict(pred_passes=30, joint_passes=50, joint_rows=70, pred_rows=11, outer_max=7, joint_passes_max=9)
    pred = 4 * 640 * 640 * 2 + 640 * 640 * 2      # W_hh and W_pred, bf16
    joint = 1025 * 640 * 2                        # W_out
    rows = 11 * 11 * 640 * 4 + 70 * 2 * 640 * 4   # table row, pre-activations, cell r/w, h | enc + pred row
    per_group, one_stream = bench.algorithmic_bytes(cfg, stats)
    assert per_group == 30 * pred + 50 * joint + rows
    assert one_stream == 7 * pred + 9 * joint + rows
    cfg = synth.CONFIGS["cfg4_rnnt_stateless"]
    per_group, one_stream = bench.algorithmic_bytes(cfg, stats)
    assert per_group == 50 * joint + 70 * 3 * 640 * 4
    assert one_stream == 9 * joint + 70 * 3 * 640 * 4
    cfg = synth.CONFIGS["cfg5_large_tdt"]          # two layers: the second streams both its matrices
    assert bench.matrix_bytes(cfg)[0] == 1024 * 640 * 2 + 4 * 640 * 640 * 2 + 8 * 640 * 640 * 2


def test_generators_are_seeded_and_round_to_nearest_even():
    cfg = synth.small_config("g", dtype="bf16", pred_kind="lstm", d_enc=16, h_pred=16, emb_dim=16,
                             h_joint=24, vocab=11, seed=5)
    w1, w2 = synth.generate_model(cfg), synth.generate_model(cfg)
    assert sorted(w1) == sorted(w2) and all((w1[k] == w2[k]).all() for k in w1)
    e1, l1 = synth.generate_inputs(cfg)
    e2, l2 = synth.generate_inputs(cfg)
    assert (e1 == e2).all() and (l1 == l2).all()
    assert ((l1 >= cfg.len_lo) & (l1 <= cfg.len_hi)).all()
    assert (w1["emb"][cfg.vocab] == 0).all()           # the start-of-sequence / blank row
    # bfloat16 rounding against an independent implementation (torch), ties included
    x = np.random.default_rng(1).standard_normal(4096).astype(np.float32)
    x[:4] = np.array([1.00390625, 1.01171875, -1.00390625, 3.0e-39], np.float32)   # two ties, a denormal
    ours = synth.round_to_bf16(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert (ours == ref).all()
    bits = synth.bf16_bits(ours)
    back = (bits.astype(np.uint32) << 16).view(np.float32)
    assert (back == ours).all()
    # matrices of a bf16 model hold bf16 values already
    assert (synth.round_to_bf16(w1["w_out"]) == w1["w_out"]).all() and (synth.round_to_bf16(e1) == e1).all()


def test_chunk_helpers_cut_and_stitch():
    rng = np.random.default_rng(0)
    ln = np.array([0, 1, 7, 12, 5], np.int32)
    enc = rng.standard_normal((5, 12, 3)).astype(np.float32)
    for mode, n in (("random", 4), ("even", 3), ("single", 0)):
        b = chunks.split_plan(ln, n, rng, mode)
        assert (b[:, 0] == 0).all() and (b[:, -1] == ln).all() and (np.diff(b, axis=1) >= 0).all()
        pieces = [chunks.make_chunk(enc, b, c, rng) for c in range(b.shape[1] - 1)]
        for u in range(5):
            got = np.concatenate([e[u, :l[u]] for e, l in pieces]) if ln[u] else np.zeros((0, 3), np.float32)
            assert (got == enc[u, :ln[u]]).all()
    # stitching: labels in order, frames shifted by each chunk's start
    b = np.array([[0, 3, 5]])
    parts = [dict(labels=np.array([[4, 9]]), frames=np.array([[0, 2]]), len=np.array([2]),
                  score=np.array([-1.0], np.float32), status=np.array([0])),
             dict(labels=np.array([[7, 0]]), frames=np.array([[1, 0]]), len=np.array([1]),
                  score=np.array([-0.5], np.float32), status=np.array([1]))]
    s = chunks.stitch(parts, b, 4)
    assert s["len"][0] == 3 and s["labels"][0, :3].tolist() == [4, 9, 7]
    assert s["frames"][0, :3].tolist() == [0, 2, 4] and s["score"][0] == -1.5 and s["status"][0] == 1
