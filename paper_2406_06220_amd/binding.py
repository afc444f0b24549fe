"""ctypes binding of ``libtdt_decode.so`` -- argument marshalling only.

The functions carry the names of the C ABI in ``include/tdt_decode.h``.  Device
memory and streams come from PyTorch; every step of the decode runs in the HIP
library.  There is no fallback: if the library has not been built the import of
its symbols raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Sequence

import numpy as np

from . import synth

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libtdt_decode.so")
# the same library built with -DTDT_PHASE_TIMERS=1 (``python -m paper_2406_06220_amd.build --phase-timers``);
# set LIB_PATH to it before the first call to get the per-phase ticks in the statistics
TIMERS_LIB_PATH = os.path.join(_PKG, "libtdt_decode_timers.so")

TDT_MAX_LSTM_LAYERS = 4
TDT_STAT_NAMES = {"pred_passes": 0, "pred_rows": 1, "joint_passes": 2, "joint_rows": 3,
                  "outer_max": 4, "abort": 5, "joint_passes_max": 6, "ticks_pred": 8, "ticks_proj": 9, "ticks_joint": 10,
                  "ticks_decide": 11, "ticks_barrier": 12, "ticks_total": 13,
                  **{f"ticks_{ph}_{part}": 14 + 3 * a + b
                     for a, ph in enumerate(("pred", "proj", "joint"))
                     for b, part in enumerate(("stage", "mma", "epilogue"))}}
TDT_STAT_COUNT = 24
TDT_ALG_LABEL_LOOPING = 0
TDT_ALG_FRAME_LOOPING = 1
TDT_HYP_TRUNCATED = 1
TDT_HYP_LEN_CLAMPED = 2
TDT_HYP_ABORTED = 4
TDT_ERR_TOO_LARGE = -7
TDT_ERR_ALIGN = -8
TDT_STATIC_SCRATCH_BYTES = 64 << 20

EXPORTS = ("tdt_workspace_bytes", "tdt_greedy_decode", "tdt_greedy_decode_static", "tdt_state_bytes",
           "tdt_greedy_decode_chunk", "tdt_encoder_projection", "tdt_encoder_projection_valid",
           "tdt_status_string")


class tdt_weights_t(C.Structure):
    _fields_ = [
        ("dtype", C.c_int32), ("d_enc", C.c_int32), ("h_joint", C.c_int32), ("vocab", C.c_int32),
        ("n_dur", C.c_int32), ("pred_kind", C.c_int32), ("pred_layers", C.c_int32),
        ("h_pred", C.c_int32), ("emb_dim", C.c_int32),
        ("w_enc", C.c_void_p), ("b_enc", C.c_void_p), ("emb", C.c_void_p),
        ("w_ih", C.c_void_p * TDT_MAX_LSTM_LAYERS), ("w_hh", C.c_void_p * TDT_MAX_LSTM_LAYERS),
        ("b_lstm", C.c_void_p * TDT_MAX_LSTM_LAYERS),
        ("w_pred", C.c_void_p), ("b_pred", C.c_void_p), ("w_out", C.c_void_p), ("b_out", C.c_void_p),
        ("multi_blank", C.c_int32),
    ]


class tdt_options_t(C.Structure):
    _fields_ = [("window", C.c_int32), ("n_clusters", C.c_int32), ("reuse_enc_proj", C.c_int32),
                ("joint_tiles", C.c_int32), ("algorithm", C.c_int32), ("wait_timeout_us", C.c_int32),
                ("selftest_stall", C.c_int32), ("projections", C.c_int32), ("joint_kernel", C.c_int32)]


_lib = None


def load_library():
    """Load the HIP library; raises if it is not there (no CPU fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2406_06220_amd.build` "
                               "(or __graft_entry__.build()) first")
        lib = C.CDLL(LIB_PATH)
        lib.tdt_workspace_bytes.restype = C.c_int
        lib.tdt_workspace_bytes.argtypes = [C.POINTER(tdt_weights_t), C.c_int, C.c_int, C.c_int,
                                            C.POINTER(C.c_size_t)]
        lib.tdt_greedy_decode.restype = C.c_int
        lib.tdt_greedy_decode.argtypes = [
            C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.POINTER(tdt_weights_t),
            C.POINTER(C.c_int32), C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
            C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
            C.POINTER(tdt_options_t), C.c_void_p]
        lib.tdt_greedy_decode_static.restype = C.c_int
        lib.tdt_greedy_decode_static.argtypes = [
            C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.POINTER(tdt_weights_t),
            C.POINTER(C.c_int32), C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
            C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(tdt_options_t), C.c_void_p]
        lib.tdt_state_bytes.restype = C.c_int
        lib.tdt_state_bytes.argtypes = [C.POINTER(tdt_weights_t), C.c_int, C.POINTER(C.c_size_t)]
        lib.tdt_greedy_decode_chunk.restype = C.c_int
        lib.tdt_greedy_decode_chunk.argtypes = [
            C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.POINTER(tdt_weights_t),
            C.POINTER(C.c_int32), C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
            C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
            C.POINTER(tdt_options_t), C.c_void_p]
        lib.tdt_encoder_projection.restype = C.c_int
        lib.tdt_encoder_projection.argtypes = [C.c_void_p, C.c_int64, C.POINTER(tdt_weights_t),
                                               C.c_void_p, C.c_void_p]
        lib.tdt_encoder_projection_valid.restype = C.c_int
        lib.tdt_encoder_projection_valid.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int,
                                                     C.POINTER(tdt_weights_t), C.c_void_p, C.c_void_p]
        lib.tdt_status_string.restype = C.c_char_p
        lib.tdt_status_string.argtypes = [C.c_int]
        _lib = lib
    return _lib


class TdtError(RuntimeError):
    def __init__(self, code: int):
        self.code = code
        super().__init__(f"tdt status {code}: {tdt_status_string(code)}")


def _check(code: int):
    if code != 0:
        raise TdtError(code)


# ----------------------------------------------------------------------------
# thin wrappers, same names as the C ABI
# ----------------------------------------------------------------------------
def tdt_status_string(code: int) -> str:
    return load_library().tdt_status_string(int(code)).decode()


def tdt_workspace_bytes(weights: tdt_weights_t, B: int, T: int, u_cap: int) -> int:
    n = C.c_size_t(0)
    _check(load_library().tdt_workspace_bytes(C.byref(weights), B, T, u_cap, C.byref(n)))
    return int(n.value)


def tdt_encoder_projection(enc_ptr: int, rows: int, weights: tdt_weights_t, out_ptr: int,
                           stream: int = 0) -> None:
    _check(load_library().tdt_encoder_projection(enc_ptr, rows, C.byref(weights), out_ptr, stream))


def tdt_encoder_projection_valid(enc_ptr: int, enc_len_ptr: int, B: int, T: int, weights: tdt_weights_t,
                                 out_ptr: int, stream: int = 0) -> None:
    _check(load_library().tdt_encoder_projection_valid(enc_ptr, enc_len_ptr, B, T, C.byref(weights), out_ptr,
                                                       stream))


def tdt_greedy_decode(enc_ptr: int, enc_len_ptr: int, B: int, T: int, weights: tdt_weights_t,
                      durations: Optional[Sequence[int]], max_symbols: int, u_cap: int,
                      out_labels_ptr: int, out_frames_ptr: int, out_len_ptr: int,
                      out_score_ptr: int, out_status_ptr: int, out_stats_ptr: int,
                      workspace_ptr: int, workspace_bytes: int,
                      options: Optional[tdt_options_t] = None, stream: int = 0) -> None:
    dur = None
    if durations is not None and len(durations):
        dur = (C.c_int32 * len(durations))(*[int(d) for d in durations])
    _check(load_library().tdt_greedy_decode(
        enc_ptr, enc_len_ptr, B, T, C.byref(weights), dur, max_symbols, u_cap, out_labels_ptr,
        out_frames_ptr, out_len_ptr, out_score_ptr, out_status_ptr, out_stats_ptr, workspace_ptr,
        workspace_bytes, C.byref(options) if options is not None else None, stream))


def tdt_greedy_decode_static(enc_ptr: int, enc_len_ptr: int, B: int, T: int, weights: tdt_weights_t,
                             durations: Optional[Sequence[int]], max_symbols: int, u_cap: int,
                             out_labels_ptr: int, out_frames_ptr: int, out_len_ptr: int,
                             out_score_ptr: int, out_status_ptr: int, out_stats_ptr: int,
                             options: Optional[tdt_options_t] = None, stream: int = 0) -> None:
    dur = None
    if durations is not None and len(durations):
        dur = (C.c_int32 * len(durations))(*[int(d) for d in durations])
    _check(load_library().tdt_greedy_decode_static(
        enc_ptr, enc_len_ptr, B, T, C.byref(weights), dur, max_symbols, u_cap, out_labels_ptr,
        out_frames_ptr, out_len_ptr, out_score_ptr, out_status_ptr, out_stats_ptr,
        C.byref(options) if options is not None else None, stream))


def tdt_state_bytes(weights: tdt_weights_t, B: int) -> int:
    n = C.c_size_t(0)
    _check(load_library().tdt_state_bytes(C.byref(weights), B, C.byref(n)))
    return int(n.value)


def tdt_greedy_decode_chunk(enc_ptr: int, enc_len_ptr: int, B: int, T: int, weights: tdt_weights_t,
                            durations: Optional[Sequence[int]], max_symbols: int, u_cap: int,
                            out_labels_ptr: int, out_frames_ptr: int, out_len_ptr: int,
                            out_score_ptr: int, out_status_ptr: int, out_stats_ptr: int,
                            state_ptr: int, workspace_ptr: int, workspace_bytes: int,
                            options: Optional[tdt_options_t] = None, stream: int = 0) -> None:
    dur = None
    if durations is not None and len(durations):
        dur = (C.c_int32 * len(durations))(*[int(d) for d in durations])
    _check(load_library().tdt_greedy_decode_chunk(
        enc_ptr, enc_len_ptr, B, T, C.byref(weights), dur, max_symbols, u_cap, out_labels_ptr,
        out_frames_ptr, out_len_ptr, out_score_ptr, out_status_ptr, out_stats_ptr, state_ptr,
        workspace_ptr, workspace_bytes, C.byref(options) if options is not None else None, stream))


# ----------------------------------------------------------------------------
# device-memory plumbing (PyTorch) around the calls above
# ----------------------------------------------------------------------------
def _to_device(a: np.ndarray, dtype: str, matrix: bool, device):
    import torch
    if matrix and dtype == "bf16":
        bits = synth.bf16_bits(a).reshape(a.shape)
        return torch.from_numpy(bits.view(np.int16)).to(device)
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(device)


class DeviceModel:
    """Weights resident in HBM plus the ``tdt_weights_t`` that points at them."""

    def __init__(self, cfg: synth.WorkloadConfig, weights: Dict[str, np.ndarray], device="cuda:0"):
        self.cfg = cfg
        self.device = device
        t: Dict[str, object] = {}
        for k, v in weights.items():
            t[k] = _to_device(v, cfg.dtype, not k.startswith("b_"), device)
        self.tensors = t
        w = tdt_weights_t()
        w.dtype = 1 if cfg.dtype == "bf16" else 0
        w.d_enc, w.h_joint, w.vocab, w.n_dur = cfg.d_enc, cfg.h_joint, cfg.vocab, cfg.n_dur
        w.multi_blank = 1 if getattr(cfg, "multi_blank", False) else 0
        w.pred_kind = 1 if cfg.pred_kind == "lstm" else 0
        w.pred_layers, w.h_pred, w.emb_dim = cfg.pred_layers, cfg.h_pred, cfg.emb_dim
        w.w_enc, w.b_enc, w.emb = t["w_enc"].data_ptr(), t["b_enc"].data_ptr(), t["emb"].data_ptr()
        if cfg.pred_kind == "lstm":
            for l in range(cfg.pred_layers):
                w.w_ih[l] = t[f"w_ih{l}"].data_ptr()
                w.w_hh[l] = t[f"w_hh{l}"].data_ptr()
                w.b_lstm[l] = t[f"b_lstm{l}"].data_ptr()
        w.w_pred, w.b_pred = t["w_pred"].data_ptr(), t["b_pred"].data_ptr()
        w.w_out, w.b_out = t["w_out"].data_ptr(), t["b_out"].data_ptr()
        self.c = w

    def upload_enc(self, enc: np.ndarray):
        return _to_device(enc, self.cfg.dtype, True, self.device)


class Decoder:
    """Owns the output tensors and the workspace for one (model, B, T, u_cap)."""

    def __init__(self, model: DeviceModel, B: int, T: int, u_cap: int,
                 window: int = 0, n_clusters: int = 0, joint_tiles: int = 0, algorithm: int = 0,
                 projections: int = 0, joint_kernel: int = 0):
        import torch
        self.model, self.B, self.T, self.u_cap = model, B, T, u_cap
        dev = model.device
        self.ws_bytes = tdt_workspace_bytes(model.c, B, T, u_cap)
        self.workspace = torch.empty(self.ws_bytes + 256, dtype=torch.uint8, device=dev)
        self.ws_ptr = (self.workspace.data_ptr() + 255) // 256 * 256
        self.labels = torch.zeros((B, u_cap), dtype=torch.int32, device=dev)
        self.frames = torch.zeros((B, u_cap), dtype=torch.int32, device=dev)
        self.lens = torch.zeros(B, dtype=torch.int32, device=dev)
        self.score = torch.zeros(B, dtype=torch.float32, device=dev)
        self.status = torch.zeros(B, dtype=torch.int32, device=dev)
        self.stats = torch.zeros(TDT_STAT_COUNT, dtype=torch.int64, device=dev)
        self.options = tdt_options_t()
        self.options.window = window
        self.options.n_clusters = n_clusters
        self.options.joint_tiles = joint_tiles
        self.options.algorithm = algorithm
        self.options.projections = projections
        self.options.joint_kernel = joint_kernel

    def __call__(self, enc_dev, enc_len_dev, max_symbols: Optional[int] = None, stream=None):
        import torch
        cfg = self.model.cfg
        s = stream if stream is not None else torch.cuda.current_stream(self.model.device)
        tdt_greedy_decode(
            enc_dev.data_ptr(), enc_len_dev.data_ptr(), self.B, self.T, self.model.c,
            list(cfg.durations) if cfg.durations else None,
            cfg.max_symbols if max_symbols is None else max_symbols, self.u_cap,
            self.labels.data_ptr(), self.frames.data_ptr(), self.lens.data_ptr(),
            self.score.data_ptr(), self.status.data_ptr(), self.stats.data_ptr(),
            self.ws_ptr, self.ws_bytes, self.options, s.cuda_stream)

    def results(self) -> dict:
        """Synchronises and copies the outputs to the host."""
        import torch
        torch.cuda.synchronize(self.model.device)
        st = self.stats.cpu().numpy()
        return dict(labels=self.labels.cpu().numpy(), frames=self.frames.cpu().numpy(),
                    len=self.lens.cpu().numpy(), score=self.score.cpu().numpy(),
                    status=self.status.cpu().numpy(),
                    stats={n: int(st[i]) for n, i in TDT_STAT_NAMES.items()})


class StreamState:
    """The device memory ``tdt_greedy_decode_chunk`` keeps between the chunks of B utterances."""

    def __init__(self, model: DeviceModel, B: int):
        import torch
        self.model, self.B = model, B
        self.bytes = tdt_state_bytes(model.c, B)
        self.buf = torch.zeros(self.bytes + 256, dtype=torch.uint8, device=model.device)
        self.ptr = (self.buf.data_ptr() + 255) // 256 * 256

    def reset(self):
        self.buf.zero_()

    def download(self) -> dict:
        """The arrays of the state as the header lays them out (synchronises)."""
        cfg, B = self.model.cfg, self.B
        off = self.ptr - self.buf.data_ptr()
        raw = self.buf.cpu().numpy()[off:off + self.bytes]
        ints = (B * 4 + 255) // 256 * 256
        get = lambda i: raw[i * ints:i * ints + 4 * B].view(np.int32).copy()
        out = dict(started=get(0), time=get(1), last=get(2), last2=get(3))
        if cfg.pred_kind == "lstm":
            n = cfg.pred_layers * B * cfg.h_pred
            fl = (n * 4 + 255) // 256 * 256
            shape = (cfg.pred_layers, B, cfg.h_pred)
            out["h"] = raw[4 * ints:4 * ints + 4 * n].view(np.float32).reshape(shape).copy()
            out["c"] = raw[4 * ints + fl:4 * ints + fl + 4 * n].view(np.float32).reshape(shape).copy()
        return out


class ChunkDecoder(Decoder):
    """``Decoder`` for chunks: each call decodes the next chunk (at most T frames each) of the
    B utterances whose state ``state`` holds."""

    def __init__(self, model: DeviceModel, B: int, T: int, u_cap: int, state: StreamState, **kw):
        super().__init__(model, B, T, u_cap, **kw)
        self.state = state

    def __call__(self, enc_dev, enc_len_dev, T: Optional[int] = None,
                 max_symbols: Optional[int] = None, stream=None):
        import torch
        cfg = self.model.cfg
        T = self.T if T is None else T
        assert 1 <= T <= self.T, "the workspace was sized for chunks of at most self.T frames"
        s = stream if stream is not None else torch.cuda.current_stream(self.model.device)
        tdt_greedy_decode_chunk(
            enc_dev.data_ptr(), enc_len_dev.data_ptr(), self.B, T, self.model.c,
            list(cfg.durations) if cfg.durations else None,
            cfg.max_symbols if max_symbols is None else max_symbols, self.u_cap,
            self.labels.data_ptr(), self.frames.data_ptr(), self.lens.data_ptr(),
            self.score.data_ptr(), self.status.data_ptr(), self.stats.data_ptr(),
            self.state.ptr, self.ws_ptr, self.ws_bytes, self.options, s.cuda_stream)
