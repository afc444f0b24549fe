"""Test-side re-orderings of the decoding loops (not collected by pytest).

Two batched decoders written from the paper's pseudo-code, with the model passed
in as callables so that either the oracle's row primitives or a scripted lookup
table can stand behind them:

* ``label_looping``   -- Algorithm 3 (outer loop over labels, inner loop over
  frames for the rows whose last decision was blank), with the Sec. 3.3 change
  for TDT and the symbols-per-frame cap;
* ``frame_looping_batched`` -- Algorithm 2 (shared frame index, inner loop until
  every row is blank), plain Transducer only.

They exist to show that the per-utterance definition in ``oracle/`` and the
label-looping order give the same hypotheses, and to count predictor / joiner
calls on the paper's worked example (Fig. 2).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, List, Sequence

import numpy as np


@dataclass
class BatchedHyps:
    """Sec. 3.1: [B, max_length] transcripts plus per-row lengths, time-stamps, scores."""
    B: int
    max_length: int
    transcripts: np.ndarray = field(init=False)
    timestamps: np.ndarray = field(init=False)
    current_lengths: np.ndarray = field(init=False)
    scores: np.ndarray = field(init=False)

    def __post_init__(self):
        self.transcripts = np.zeros((self.B, self.max_length), np.int64)
        self.timestamps = np.zeros((self.B, self.max_length), np.int64)
        self.current_lengths = np.zeros(self.B, np.int64)
        self.scores = np.zeros(self.B, np.float32)

    def add_results(self, add_mask, labels, frames, score_inc):
        rows = np.nonzero(add_mask)[0]
        self.transcripts[rows, self.current_lengths[rows]] = labels[rows]
        self.timestamps[rows, self.current_lengths[rows]] = frames[rows]
        self.scores[rows] = (self.scores[rows] + score_inc[rows]).astype(np.float32)
        self.current_lengths += add_mask.astype(np.int64)


@dataclass
class ModelFns:
    """predictor(state, label) -> (dec, new_state); joiner(b, t, dec) -> logits[V+1+D]."""
    init_state: Callable[[], object]
    predictor: Callable[[object, int], tuple]
    joiner: Callable[[int, int, object], np.ndarray]
    vocab: int
    durations: Sequence[int] = ()
    multi_blank: bool = False                    # the D extra outputs are big blanks of the label head


def _decide(fns: ModelFns, logits: np.ndarray):
    V, D = fns.vocab, len(fns.durations)
    lab = logits[: V + 1 + D] if fns.multi_blank else logits[: V + 1]
    k = int(np.argmax(lab))                      # first maximum
    if fns.multi_blank:                          # the chosen symbol says how far to move
        d = 0 if k < V else 1 if k == V else max(int(fns.durations[k - V - 1]), 1)
    elif D:
        d = int(fns.durations[int(np.argmax(logits[V + 1: V + 1 + D]))])
    else:
        d = 1 if k == V else 0
    m = np.float32(lab.max())
    lse = np.float32(m + np.log(np.sum(np.exp((lab - m).astype(np.float32)), dtype=np.float32)))
    return k, d, np.float32(lab[k] - lse)


def label_looping(fns: ModelFns, lens: Sequence[int], max_symbols: int, u_cap: int) -> dict:
    B, V = len(lens), fns.vocab
    lens = np.asarray(lens, np.int64)
    hyps = BatchedHyps(B, max(u_cap, 1))
    state = [fns.init_state() for _ in range(B)]
    predictions = np.full(B, V, np.int64)        # BOS
    b2time = np.zeros(B, np.int64)
    sym = np.zeros(B, np.int64)
    b2active = (b2time < lens) & (u_cap > 0)
    n_pred = n_joint = 0
    k = np.zeros(B, np.int64)
    d = np.zeros(B, np.int64)
    inc = np.zeros(B, np.float32)
    found = np.zeros(B, np.int64)
    while b2active.any():
        decs = [None] * B
        for b in range(B):                       # one batched predictor call, state kept for all
            decs[b], state[b] = fns.predictor(state[b], int(predictions[b]))
        n_pred += 1
        live = b2active.copy()
        need = live.copy()
        blank_mask = np.ones(B, bool)
        first = True
        while first or need.any():
            first = False
            n_joint += 1                         # one batched joiner call
            for b in np.nonzero(need)[0]:
                k[b], d[b], inc[b] = _decide(fns, fns.joiner(b, int(b2time[b]), decs[b]))
                found[b] = b2time[b]
                blank_mask[b] = (k[b] >= V)      # the blank, or a big blank
                if blank_mask[b]:
                    b2time[b] += max(int(d[b]), 1)
                    sym[b] = 0
            b2active = b2time < lens
            need = need & blank_mask & b2active
        add_mask = live & ~blank_mask
        hyps.add_results(add_mask, k, found, inc)
        for b in np.nonzero(add_mask)[0]:
            predictions[b] = k[b]
            sym[b] += 1
            dd = int(d[b])
            if dd == 0 and sym[b] >= max_symbols:
                dd = 1
            if dd > 0:
                b2time[b] += dd
                sym[b] = 0
        b2active = (b2time < lens) & (hyps.current_lengths < u_cap)
    return dict(labels=hyps.transcripts, frames=hyps.timestamps, len=hyps.current_lengths,
                score=hyps.scores, n_pred=n_pred, n_joint=n_joint)


def frame_looping_batched(fns: ModelFns, lens: Sequence[int], max_symbols: int, u_cap: int) -> dict:
    """Algorithm 2 with per-row length checks; plain Transducer (no durations)."""
    assert not fns.durations
    B, V = len(lens), fns.vocab
    lens = np.asarray(lens, np.int64)
    T = int(lens.max()) if B else 0
    hyps: List[list] = [[] for _ in range(B)]
    frames: List[list] = [[] for _ in range(B)]
    scores = np.zeros(B, np.float32)
    states = [fns.init_state() for _ in range(B)]
    last = np.full(B, V, np.int64)               # label the predictor is fed
    n_pred = n_joint = 0
    t = 0
    while t < T:
        sym = np.zeros(B, np.int64)
        done = ~((t < lens) & (np.array([len(h) for h in hyps]) < u_cap))
        blank_mask = done.copy()
        first = True
        while first or not blank_mask.all():
            first = False
            new_states, decs = [None] * B, [None] * B
            for b in range(B):
                decs[b], new_states[b] = fns.predictor(states[b], int(last[b]))
            n_pred += 1
            n_joint += 1
            for b in range(B):
                if blank_mask[b]:
                    continue
                k, _, inc = _decide(fns, fns.joiner(b, t, decs[b]))
                if k == V:
                    blank_mask[b] = True
                    continue
                states[b] = new_states[b]
                hyps[b].append(k)
                frames[b].append(t)
                scores[b] = np.float32(scores[b] + inc)
                last[b] = k
                sym[b] += 1
                if sym[b] >= max_symbols or len(hyps[b]) >= u_cap:
                    blank_mask[b] = True
        t += 1
    return dict(labels=hyps, frames=frames, len=np.array([len(h) for h in hyps]), score=scores,
                n_pred=n_pred, n_joint=n_joint)


def oracle_fns(model, enc: np.ndarray) -> ModelFns:
    """Callables backed by the oracle's row primitives (same fp32 arithmetic as its decoder)."""
    cache = {}

    def joiner(b, t, dec):
        key = (b, t)
        if key not in cache:
            cache[key] = model.enc_proj_frame(enc[b, t])
        return model.joint(cache[key], dec)

    def predictor(state, label):
        dec, new_state = model.predictor_step(state, label)
        return model.pred_proj(dec), new_state

    return ModelFns(init_state=model.init_state, predictor=predictor, joiner=joiner,
                    vocab=model.cfg.vocab, durations=tuple(model.cfg.durations),
                    multi_blank=bool(getattr(model.cfg, "multi_blank", False)))
