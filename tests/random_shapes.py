"""Seeded random model shapes and call options for the GPU parity tests (not collected by pytest).

Every width is a multiple of 8 (the library's requirement); the draws cover both dtypes and
predictors, one to four LSTM layers, with and without durations, lengths from 0, and the option
space (window, groups, loop order, projections ahead of the loops or on the fly, the streaming
joint pass, big blanks)."""
from __future__ import annotations

import numpy as np

from paper_2406_06220_amd import synth


def draw(seed: int, hi: int = 320, v_hi: int = 400, b_hi: int = 70, t_hi: int = 40):
    rng = np.random.default_rng(seed)
    m8 = lambda lo, top: int(rng.integers(lo // 8, top // 8 + 1)) * 8
    kind = rng.choice(["lstm", "stateless"])
    kw = dict(dtype=str(rng.choice(["fp32", "bf16"])), d_enc=m8(8, hi), h_joint=m8(8, hi),
              vocab=int(rng.integers(2, v_hi)), B=int(rng.integers(1, b_hi)), T=int(rng.integers(1, t_hi)),
              seed=5000 + seed, default_blank_bias=float(rng.uniform(-0.5, 1.5)),
              max_symbols=int(rng.integers(1, 6)))
    kw["len_lo"] = int(rng.integers(0, kw["T"] + 1))
    kw["len_hi"] = kw["T"]
    if rng.random() < 0.5:
        d = sorted(set(rng.integers(0, 6, size=int(rng.integers(1, 7))).tolist()))
        if max(d) == 0:
            d.append(2)
        kw["durations"] = tuple(d)
    if kind == "lstm":
        kw.update(pred_kind="lstm", pred_layers=int(rng.integers(1, 5)), h_pred=m8(8, hi), emb_dim=m8(8, hi))
    else:
        c, e = int(rng.integers(1, 3)), m8(8, hi // 2)
        kw.update(pred_layers=c, emb_dim=e, h_pred=c * e)
    cfg = synth.small_config(f"random{seed}", **kw)
    opts = dict(window=int(rng.choice([0, 0, 1, 2, 9, 64])), n_clusters=int(rng.choice([0, 0, 1, 2, 3, 5, 8])),
                algorithm=int(rng.choice([0, 0, 0, 1])))
    if opts["n_clusters"] > cfg.B:
        opts["n_clusters"] = 0
    n_chunks = int(rng.integers(2, 6))
    # (drawn last, so that the draws above are what they were before this option existed)
    opts["projections"] = int(opts["algorithm"] == 0 and rng.random() < 0.35)
    # later options, drawn after everything above for the same reason: the streaming joint pass
    # where it can run, and the extra outputs read as big blanks of the label head
    if (rng.random() < 0.7 and cfg.dtype == "bf16" and opts["algorithm"] == 0 and not opts["projections"]
            and opts["n_clusters"] in (0,) + tuple(range(4, 9))):
        opts["joint_kernel"] = 2
    if rng.random() < 0.5 and cfg.durations:
        import dataclasses
        cfg = dataclasses.replace(cfg, multi_blank=True,
                                  durations=tuple(sorted(set(max(1, d) + 1 for d in cfg.durations))))
    return cfg, opts, n_chunks
