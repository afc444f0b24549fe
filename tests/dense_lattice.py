"""Dense (frame x label-count) lattice of a small Transducer in float64 numpy.

An independent construction used to pin the oracle: the predictor is teacher
forced over a given label sequence, every joint output logit[t, u, :] is computed
with library matrix products, and the greedy path is then read off the lattice
node by node.  Nothing here is shared with ``oracle/`` or with the GPU library.
(Not collected by pytest.)
"""
from __future__ import annotations

import numpy as np
from scipy.special import log_softmax


def _sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


def teacher_forced_dec(cfg, w, labels):
    """dec[u] for u = 0..len(labels): predictor output after BOS and after each label."""
    V = cfg.vocab
    seq = [V] + [int(x) for x in labels]
    out = []
    if cfg.pred_kind == "stateless":
        ctx = [V] * cfg.pred_layers
        emb = w["emb"].astype(np.float64).reshape(cfg.pred_layers, V + 1, cfg.emb_dim)
        for tok in seq:
            ctx = ctx[1:] + [tok]
            out.append(np.concatenate([emb[i, ctx[i]] for i in range(cfg.pred_layers)]))
        return np.stack(out)
    Hp = cfg.h_pred
    h = [np.zeros(Hp) for _ in range(cfg.pred_layers)]
    c = [np.zeros(Hp) for _ in range(cfg.pred_layers)]
    emb = w["emb"].astype(np.float64)
    for tok in seq:
        x = emb[tok]
        for l in range(cfg.pred_layers):
            g = (w[f"w_ih{l}"].astype(np.float64) @ x + w[f"w_hh{l}"].astype(np.float64) @ h[l]
                 + w[f"b_lstm{l}"].astype(np.float64))
            i, f, gg, o = g[:Hp], g[Hp:2 * Hp], g[2 * Hp:3 * Hp], g[3 * Hp:]
            c[l] = _sigmoid(f) * c[l] + _sigmoid(i) * np.tanh(gg)
            h[l] = _sigmoid(o) * np.tanh(c[l])
            x = h[l]
        out.append(x.copy())
    return np.stack(out)


def lattice(cfg, w, enc_b, labels):
    """logit[t, u, :] for every frame of enc_b and u = 0..len(labels)."""
    dec = teacher_forced_dec(cfg, w, labels)
    ep = enc_b.astype(np.float64) @ w["w_enc"].astype(np.float64).T + w["b_enc"]
    pp = dec @ w["w_pred"].astype(np.float64).T + w["b_pred"]
    hid = np.maximum(ep[:, None, :] + pp[None, :, :], 0.0)
    return hid @ w["w_out"].astype(np.float64).T + w["b_out"]


def greedy_walk(cfg, logits, length, u_cap):
    """Greedy path through a lattice whose label axis was teacher forced with the
    path's own labels; returns the emissions it reads off, so a caller can check
    self-consistency.  Also returns the smallest top-2 margin met on the way."""
    V, D, S = cfg.vocab, len(cfg.durations), cfg.max_symbols
    MB = bool(getattr(cfg, "multi_blank", False))
    t = u = sym = 0
    labels, frames, score = [], [], 0.0
    min_margin = np.inf
    n_dec = 0
    while t < length and u < u_cap and u < logits.shape[1]:
        row = logits[t, u]
        lab = row if MB else row[: V + 1]      # multi-blank: one head over all outputs
        k = int(np.argmax(lab))
        srt = np.sort(lab)
        min_margin = min(min_margin, srt[-1] - srt[-2])
        n_dec += 1
        if MB:
            d = 0 if k < V else 1 if k == V else max(int(cfg.durations[k - V - 1]), 1)
        elif D:
            dl = row[V + 1:]
            d = int(cfg.durations[int(np.argmax(dl))])
            if D > 1:
                ds = np.sort(dl)
                min_margin = min(min_margin, ds[-1] - ds[-2])
        else:
            d = 1 if k == V else 0
        if k >= V:                              # the blank, or a big blank
            t += max(d, 1)
            sym = 0
        else:
            labels.append(k)
            frames.append(t)
            score += log_softmax(lab)[k]
            u += 1
            sym += 1
            if d == 0 and sym >= S:
                d = 1
            if d > 0:
                t += d
                sym = 0
    return dict(labels=labels, frames=frames, score=score, end_t=t, end_u=u,
                min_margin=min_margin, n_dec=n_dec)
