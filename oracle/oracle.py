"""ctypes front end of the CPU oracle (TEST INFRASTRUCTURE -- not part of the product).

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this module.  It compiles ``transducer_oracle.c`` with gcc
on first use and exposes the frame-looping greedy decoder (Algorithm 1 of the
paper, extended with TDT durations and the symbols-per-frame cap), its
chunk-by-chunk form with a carried state, the tolerant replay check, and the
model primitives that test-side re-orderings of the loops
call row by row.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Dict, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "transducer_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

_f32p = C.POINTER(C.c_float)
_i32p = C.POINTER(C.c_int32)
_i64p = C.POINTER(C.c_int64)
MAX_LAYERS = 4   # ORC_MAX_LAYERS of the C source


class _Model(C.Structure):
    _fields_ = [
        ("d_enc", C.c_int32), ("h_joint", C.c_int32), ("vocab", C.c_int32), ("n_dur", C.c_int32),
        ("pred_kind", C.c_int32), ("pred_layers", C.c_int32), ("h_pred", C.c_int32),
        ("emb_dim", C.c_int32),
        ("w_enc", _f32p), ("b_enc", _f32p), ("emb", _f32p),
        ("w_ih", _f32p * MAX_LAYERS), ("w_hh", _f32p * MAX_LAYERS), ("b_lstm", _f32p * MAX_LAYERS),
        ("w_pred", _f32p), ("b_pred", _f32p), ("w_out", _f32p), ("b_out", _f32p),
        ("multi_blank", C.c_int32),
    ]


class _Trace(C.Structure):
    _fields_ = [
        ("cap", C.c_int32), ("n", C.c_int32),
        ("t", _i32p), ("u", _i32p), ("k", _i32p), ("j", _i32p),
        ("margin_lab", _f32p), ("margin_dur", _f32p),
    ]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, no fast-math) and return the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-shared", "-fPIC", _SRC,
                               "-o", _LIB, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_decode_utt.restype = C.c_int
        _lib.orc_decode_batch.restype = C.c_int
        _lib.orc_decode_batch_chunk.restype = C.c_int
        _lib.orc_replay_utt.restype = C.c_int
        _lib.orc_num_threads.restype = C.c_int
    return _lib


def _fp(a: Optional[np.ndarray]):
    return a.ctypes.data_as(_f32p) if a is not None else None


def _ip(a: Optional[np.ndarray]):
    return a.ctypes.data_as(_i32p) if a is not None else None


class OracleModel:
    """Holds float32 copies of the weights and the C descriptor that points at them."""

    def __init__(self, cfg, weights: Dict[str, np.ndarray]):
        self.cfg = cfg
        self._keep = {k: np.ascontiguousarray(v, dtype=np.float32) for k, v in weights.items()}
        w = self._keep
        m = _Model()
        m.d_enc, m.h_joint, m.vocab, m.n_dur = cfg.d_enc, cfg.h_joint, cfg.vocab, len(cfg.durations)
        m.pred_kind = 1 if cfg.pred_kind == "lstm" else 0
        m.pred_layers, m.h_pred, m.emb_dim = cfg.pred_layers, cfg.h_pred, cfg.emb_dim
        m.w_enc, m.b_enc, m.emb = _fp(w["w_enc"]), _fp(w["b_enc"]), _fp(w["emb"])
        if cfg.pred_kind == "lstm":
            for l in range(cfg.pred_layers):
                m.w_ih[l] = _fp(w[f"w_ih{l}"])
                m.w_hh[l] = _fp(w[f"w_hh{l}"])
                m.b_lstm[l] = _fp(w[f"b_lstm{l}"])
        m.w_pred, m.b_pred = _fp(w["w_pred"]), _fp(w["b_pred"])
        m.w_out, m.b_out = _fp(w["w_out"]), _fp(w["b_out"])
        m.multi_blank = 1 if getattr(cfg, "multi_blank", False) else 0
        self.c = m
        self.durations = (np.asarray(cfg.durations, np.int32) if len(cfg.durations)
                          else None)

    # -- model primitives (one row at a time) ---------------------------------
    def enc_proj_frame(self, enc_t: np.ndarray) -> np.ndarray:
        out = np.empty(self.cfg.h_joint, np.float32)
        _load().orc_enc_proj_frame(C.byref(self.c), _fp(np.ascontiguousarray(enc_t, np.float32)),
                                   _fp(out))
        return out

    def init_state(self):
        n = 2 * self.cfg.pred_layers * self.cfg.h_pred if self.cfg.pred_kind == "lstm" else 0
        return np.zeros(max(n, 1), np.float32), np.full(2, self.cfg.vocab, np.int32)

    def predictor_step(self, state, label: int):
        """Returns (dec, new_state); the input state is left untouched."""
        buf, ctx = state[0].copy(), state[1].copy()
        dec = np.empty(self.cfg.h_pred, np.float32)
        _load().orc_predictor_step(C.byref(self.c), _fp(buf), _ip(ctx), C.c_int(int(label)),
                                   _fp(dec))
        return dec, (buf, ctx)

    def pred_proj(self, dec: np.ndarray) -> np.ndarray:
        out = np.empty(self.cfg.h_joint, np.float32)
        _load().orc_pred_proj(C.byref(self.c), _fp(np.ascontiguousarray(dec, np.float32)), _fp(out))
        return out

    def joint(self, enc_proj: np.ndarray, pred_proj: np.ndarray) -> np.ndarray:
        out = np.empty(self.cfg.n_out, np.float32)
        _load().orc_joint(C.byref(self.c), _fp(np.ascontiguousarray(enc_proj, np.float32)),
                          _fp(np.ascontiguousarray(pred_proj, np.float32)), _fp(out))
        return out

    def lattice_logits(self, enc_t: np.ndarray, labels: Sequence[int], u: int) -> np.ndarray:
        out = np.empty(self.cfg.n_out, np.float32)
        lab = np.ascontiguousarray(labels, np.int32) if len(labels) else np.zeros(1, np.int32)
        _load().orc_lattice_logits(C.byref(self.c), _fp(np.ascontiguousarray(enc_t, np.float32)),
                                   _ip(lab), C.c_int(int(u)), _fp(out))
        return out


def decode_utt(model: OracleModel, enc: np.ndarray, length: int, max_symbols: int, u_cap: int,
               trace: bool = False) -> dict:
    """Frame-looping greedy decode of one utterance; enc is [>=length, d_enc]."""
    lib = _load()
    enc = np.ascontiguousarray(enc, np.float32)
    labels = np.zeros(max(u_cap, 1), np.int32)
    frames = np.zeros(max(u_cap, 1), np.int32)
    durs = np.zeros(max(u_cap, 1), np.int32)
    n = C.c_int32(0)
    score = C.c_float(0.0)
    counts = np.zeros(2, np.int64)
    tr = None
    tr_arrays = None
    if trace:
        cap = int(length) * (max_symbols + 1) + 2
        tr_arrays = dict(t=np.zeros(cap, np.int32), u=np.zeros(cap, np.int32),
                         k=np.zeros(cap, np.int32), j=np.zeros(cap, np.int32),
                         margin_lab=np.zeros(cap, np.float32), margin_dur=np.zeros(cap, np.float32))
        tr = _Trace(cap, 0, _ip(tr_arrays["t"]), _ip(tr_arrays["u"]), _ip(tr_arrays["k"]),
                    _ip(tr_arrays["j"]), _fp(tr_arrays["margin_lab"]), _fp(tr_arrays["margin_dur"]))
    status = lib.orc_decode_utt(
        C.byref(model.c), _fp(enc), C.c_int(int(length)), _ip(model.durations),
        C.c_int(max_symbols), C.c_int(u_cap), _ip(labels), _ip(frames), _ip(durs), C.byref(n),
        C.byref(score), C.byref(tr) if tr is not None else None,
        counts.ctypes.data_as(_i64p))
    L = n.value
    out = dict(labels=labels[:L].copy(), frames=frames[:L].copy(), durs=durs[:L].copy(), len=L,
               score=float(np.float32(score.value)), status=int(status),
               n_pred=int(counts[0]), n_joint=int(counts[1]))
    if trace:
        nt = min(tr.n, tr.cap)
        out["trace"] = {k: v[:nt].copy() for k, v in tr_arrays.items()}
    return out


def decode_batch(model: OracleModel, enc: np.ndarray, enc_len: np.ndarray, max_symbols: int,
                 u_cap: int, n_threads: int = 0) -> dict:
    """B independent utterances; threads split the utterance loop only."""
    lib = _load()
    enc = np.ascontiguousarray(enc, np.float32)
    B, T, _ = enc.shape
    enc_len = np.ascontiguousarray(enc_len, np.int32)
    labels = np.zeros((B, u_cap), np.int32)
    frames = np.zeros((B, u_cap), np.int32)
    durs = np.zeros((B, u_cap), np.int32)
    lens = np.zeros(B, np.int32)
    score = np.zeros(B, np.float32)
    status = np.zeros(B, np.int32)
    counts = np.zeros((B, 2), np.int64)
    used = lib.orc_decode_batch(
        C.byref(model.c), _fp(enc), _ip(enc_len), C.c_int(B), C.c_int(T), _ip(model.durations),
        C.c_int(max_symbols), C.c_int(u_cap), _ip(labels), _ip(frames), _ip(durs), _ip(lens),
        _fp(score), _ip(status), counts.ctypes.data_as(_i64p), C.c_int(n_threads))
    return dict(labels=labels, frames=frames, durs=durs, len=lens, score=score, status=status,
                n_pred=counts[:, 0].copy(), n_joint=counts[:, 1].copy(), threads=int(used))


def stream_state(model: OracleModel, B: int) -> dict:
    """State of B utterances none of which has been decoded yet (all zero)."""
    cfg = model.cfg
    n = cfg.pred_layers * cfg.h_pred if cfg.pred_kind == "lstm" else 1
    return dict(started=np.zeros(B, np.int32), time=np.zeros(B, np.int32),
                ctx=np.zeros((B, 2), np.int32), h=np.zeros((B, n), np.float32),
                c=np.zeros((B, n), np.float32))


def decode_batch_chunk(model: OracleModel, enc: np.ndarray, enc_len: np.ndarray, max_symbols: int,
                       u_cap: int, state: dict, n_threads: int = 0) -> dict:
    """The next chunk of B utterances decoded piece by piece; `state` is updated in place.
    Frames are counted from the chunk's start, the score is the chunk's own sum."""
    lib = _load()
    enc = np.ascontiguousarray(enc, np.float32)
    B, T, _ = enc.shape
    enc_len = np.ascontiguousarray(enc_len, np.int32)
    labels = np.zeros((B, u_cap), np.int32)
    frames = np.zeros((B, u_cap), np.int32)
    lens = np.zeros(B, np.int32)
    score = np.zeros(B, np.float32)
    status = np.zeros(B, np.int32)
    for k in ("started", "time", "ctx", "h", "c"):
        assert state[k].flags["C_CONTIGUOUS"] and state[k].shape[0] == B
    lib.orc_decode_batch_chunk(
        C.byref(model.c), _fp(enc), _ip(enc_len), C.c_int(B), C.c_int(T), _ip(model.durations),
        C.c_int(max_symbols), C.c_int(u_cap), _ip(labels), _ip(frames), _ip(lens), _fp(score),
        _ip(status), _ip(state["started"]), _ip(state["time"]), _ip(state["ctx"]),
        _fp(state["h"]), _fp(state["c"]), C.c_int(n_threads))
    return dict(labels=labels, frames=frames, len=lens, score=score, status=status)


def replay_utt(model: OracleModel, enc: np.ndarray, length: int, max_symbols: int, u_cap: int,
               cand_labels: np.ndarray, cand_frames: np.ndarray, tol: float = 1e-3) -> dict:
    """Is the candidate a greedy decode under an argmax tolerant to `tol`?"""
    lib = _load()
    enc = np.ascontiguousarray(enc, np.float32)
    cl = np.ascontiguousarray(cand_labels, np.int32)
    cf = np.ascontiguousarray(cand_frames, np.int32)
    n = int(cl.shape[0])
    if n == 0:
        cl = np.zeros(1, np.int32)
        cf = np.zeros(1, np.int32)
    n_tie = C.c_int32(0)
    score = C.c_float(0.0)
    ok = lib.orc_replay_utt(C.byref(model.c), _fp(enc), C.c_int(int(length)), _ip(model.durations),
                            C.c_int(max_symbols), C.c_int(u_cap), _ip(cl), _ip(cf), C.c_int(n),
                            C.c_float(tol), C.byref(n_tie), C.byref(score))
    return dict(ok=bool(ok), n_tie=int(n_tie.value), score=float(np.float32(score.value)))


def num_threads() -> int:
    return int(_load().orc_num_threads())
