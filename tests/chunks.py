"""Cutting a batch of utterances into chunks and stitching chunk results together.

(Not collected by pytest.)  Used by the pins of the oracle's piecewise decoding
and by the GPU parity tests of ``tdt_greedy_decode_chunk``; holds none of the
method's arithmetic.
"""
from __future__ import annotations

from typing import List

import numpy as np


def split_plan(ln: np.ndarray, n_chunks: int, rng: np.random.Generator, mode: str = "random"):
    """bounds[b] = n_chunks + 1 ascending cut points of utterance b, from 0 to ln[b].

    "random": independent uniform cuts (equal cuts give empty chunks);
    "even": equal pieces; "single": one frame a chunk for as long as frames last
    (n_chunks is then max(ln))."""
    B = len(ln)
    if mode == "single":
        n_chunks = int(max(int(ln.max()), 1))
        return np.stack([np.minimum(np.arange(n_chunks + 1), int(l)) for l in ln]).astype(np.int64)
    out = np.zeros((B, n_chunks + 1), np.int64)
    for b in range(B):
        L = int(ln[b])
        if mode == "even":
            cuts = [(L * i) // n_chunks for i in range(1, n_chunks)]
        else:
            cuts = sorted(rng.integers(0, L + 1, size=n_chunks - 1).tolist())
        out[b] = [0] + list(cuts) + [L]
    return out


def make_chunk(enc: np.ndarray, bounds: np.ndarray, c: int, rng: np.random.Generator):
    """(enc_chunk [B, Tc, d], len_chunk [B]) of chunk c; rows past a length hold noise."""
    B = enc.shape[0]
    seg = bounds[:, c + 1] - bounds[:, c]
    Tc = int(max(int(seg.max()), 1))
    out = rng.standard_normal((B, Tc, enc.shape[2])).astype(np.float32) * 3.0
    for b in range(B):
        out[b, :seg[b]] = enc[b, bounds[b, c]:bounds[b, c + 1]]
    return out, seg.astype(np.int32)


def stitch(chunk_results: List[dict], bounds: np.ndarray, u_cap: int) -> dict:
    """Concatenates per-chunk hypotheses; frames become utterance-relative, scores add up."""
    B = bounds.shape[0]
    labels = np.zeros((B, u_cap), np.int32)
    frames = np.zeros((B, u_cap), np.int32)
    lens = np.zeros(B, np.int32)
    score = np.zeros(B, np.float64)
    status = np.zeros(B, np.int32)
    for c, r in enumerate(chunk_results):
        for b in range(B):
            n = int(r["len"][b])
            o = int(lens[b])
            labels[b, o:o + n] = r["labels"][b, :n]
            frames[b, o:o + n] = r["frames"][b, :n] + bounds[b, c]
            lens[b] = o + n
            score[b] += float(r["score"][b])
            status[b] |= int(r["status"][b])
    return dict(labels=labels, frames=frames, len=lens, score=score.astype(np.float32), status=status)
