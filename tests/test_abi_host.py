"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every function the header declares, and rejects bad arguments before any device
work (so these calls are safe on a machine without a GPU)."""
from __future__ import annotations

import ctypes as C
import glob
import os
import re

import pytest

from paper_2406_06220_amd import binding, build, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        build.build_library()
    return binding.load_library()


def declared_functions():
    names = []
    for h in glob.glob(os.path.join(ROOT, "include", "*.h")):
        src = re.sub(r"/\*.*?\*/", "", open(h).read(), flags=re.S)
        names += re.findall(r"^\s*(?:const\s+)?(?:int|char|void|size_t)\s*\*?\s*(tdt_\w+)\s*\(", src,
                            flags=re.M)
    return sorted(set(names))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert set(binding.EXPORTS) <= set(names) and len(names) >= 4
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/ but not exported"


def _weights(cfg, fake_ptr=4096):
    w = binding.tdt_weights_t()
    w.dtype = 1 if cfg.dtype == "bf16" else 0
    w.d_enc, w.h_joint, w.vocab, w.n_dur = cfg.d_enc, cfg.h_joint, cfg.vocab, cfg.n_dur
    w.pred_kind = 1 if cfg.pred_kind == "lstm" else 0
    w.pred_layers, w.h_pred, w.emb_dim = cfg.pred_layers, cfg.h_pred, cfg.emb_dim
    for f in ("w_enc", "b_enc", "emb", "w_pred", "b_pred", "w_out", "b_out"):
        setattr(w, f, fake_ptr)
    for l in range(binding.TDT_MAX_LSTM_LAYERS):
        w.w_ih[l] = w.w_hh[l] = w.b_lstm[l] = fake_ptr
    return w


def _decode(lib, w, *, enc=4096, enc_len=4096, B=2, T=10, durations=None, S=3, u_cap=30,
            outs=4096, ws=4096, ws_bytes=1 << 40, options=None):
    dur = None
    if durations is not None:
        dur = (C.c_int32 * len(durations))(*durations)
    return lib.tdt_greedy_decode(enc, enc_len, B, T, C.byref(w), dur, S, u_cap, outs, outs, outs,
                                 outs, outs, None, ws, ws_bytes,
                                 C.byref(options) if options is not None else None, None)


def test_status_strings(lib):
    for code in range(0, -9, -1):
        s = binding.tdt_status_string(code)
        assert s and s != "unknown status"
    assert binding.tdt_status_string(-99) == "unknown status"


def test_workspace_bytes(lib):
    cfg = synth.CFG2
    w = _weights(cfg)
    n = binding.tdt_workspace_bytes(w, cfg.B, cfg.T, 100)
    assert n >= cfg.B * cfg.T * cfg.h_joint * 4          # holds the projected encoder frames
    assert n < cfg.B * cfg.T * cfg.h_joint * 4 + (128 << 20)
    assert binding.tdt_workspace_bytes(w, 2 * cfg.B, cfg.T, 100) > n
    size = C.c_size_t()
    assert lib.tdt_workspace_bytes(None, 1, 1, 1, C.byref(size)) == -1
    assert lib.tdt_workspace_bytes(C.byref(w), 0, 1, 1, C.byref(size)) == -2
    assert lib.tdt_workspace_bytes(C.byref(w), 1, 1, 1, None) == -1


def test_workspace_holds_the_fragment_major_copies(lib):
    """A bfloat16 model's workspace is the float32 model's plus the fragment-major copies of the
    matrices the decode kernel streams: per matrix [N][K], ceil(N / 16) column tiles (an LSTM gate
    matrix: ceil(h_pred / 4) tiles of 4 units x 4 gates) times ceil(K / 32) steps of 1 KiB."""
    import dataclasses

    def packed(cfg):
        tiles = lambda n: -(-n // 16)
        steps = lambda k: -(-k // 32)
        H, Hp = cfg.h_joint, cfg.h_pred
        n = tiles(H) * steps(cfg.d_enc) + tiles(H) * steps(Hp) + tiles(cfg.n_out) * steps(H)
        if cfg.pred_kind == "lstm":
            n += (2 * cfg.pred_layers - 1) * (-(-Hp // 4)) * steps(Hp)
        return -(-n * 1024 // 256) * 256

    for cfg in (synth.CFG2, synth.CFG4, synth.CFG5, dataclasses.replace(synth.CFG3, h_pred=648, emb_dim=648, h_joint=1000)):
        bf = binding.tdt_workspace_bytes(_weights(cfg), cfg.B, cfg.T, 100)
        f32 = binding.tdt_workspace_bytes(_weights(dataclasses.replace(cfg, dtype="fp32")), cfg.B, cfg.T, 100)
        assert bf - f32 == packed(cfg), cfg.name


def test_rejects_bad_arguments_before_device_work(lib):
    cfg = synth.CFG3
    w = _weights(cfg)
    dur = list(cfg.durations)
    # null pointers
    assert _decode(lib, w, enc=None, durations=dur) == -1
    assert _decode(lib, w, enc_len=None, durations=dur) == -1
    assert _decode(lib, w, outs=None, durations=dur) == -1
    w2 = _weights(cfg); w2.w_out = None
    assert _decode(lib, w2, durations=dur) == -1
    w2 = _weights(cfg); w2.w_hh[0] = None
    assert _decode(lib, w2, durations=dur) == -1
    # arrays that do not start at a 16-byte boundary (rows are read 16 bytes at a time)
    assert _decode(lib, w, enc=4096 + 8, durations=dur) == -8
    for field in ("w_enc", "b_enc", "emb", "w_pred", "b_pred", "w_out", "b_out"):
        w2 = _weights(cfg); setattr(w2, field, 4096 + 4)
        assert _decode(lib, w2, durations=dur) == -8, field
    w2 = _weights(cfg); w2.b_lstm[0] = 4096 + 2
    assert _decode(lib, w2, durations=dur) == -8
    assert lib.tdt_encoder_projection(4096, 10, C.byref(w), 4096 + 4, None) == -8
    assert lib.tdt_encoder_projection_valid(4096 + 2, 4096, 2, 5, C.byref(w), 4096, None) == -8
    # sizes
    for kw in (dict(B=0), dict(T=0), dict(u_cap=0), dict(S=0)):
        assert _decode(lib, w, durations=dur, **kw) == -2
    for field, val in (("h_joint", 12), ("d_enc", 0), ("h_pred", 4096), ("vocab", 0), ("n_dur", 17)):
        w2 = _weights(cfg); setattr(w2, field, val)
        assert _decode(lib, w2, durations=dur) == -2
    # unsupported model kinds
    for field, val in (("dtype", 2), ("pred_kind", 3), ("pred_layers", 5), ("pred_layers", 0)):
        w2 = _weights(cfg); setattr(w2, field, val)
        assert _decode(lib, w2, durations=dur) == -3
    ws = _weights(synth.CFG4); ws.h_pred = 320       # stateless: h_pred must be ctx * emb_dim
    assert _decode(lib, ws) == -2
    # durations
    assert _decode(lib, w, durations=None) == -4                 # TDT model without a list
    assert _decode(lib, w, durations=[0, 0, 0, 0, 0]) == -4      # no positive entry
    assert _decode(lib, w, durations=[0, 1, -1, 3, 4]) == -4     # negative entry
    assert _decode(lib, _weights(synth.CFG2), durations=[1]) == -4   # list given to a Transducer
    wm = _weights(cfg); wm.multi_blank = 1                           # multi-blank: increments of at least one frame
    assert _decode(lib, wm, durations=[0, 1, 2, 3, 4]) == -4
    wm = _weights(synth.CFG2); wm.multi_blank = 1                    # ... and at least one big blank
    assert _decode(lib, wm) == -4
    # options
    o = binding.tdt_options_t(); o.window = 65
    assert _decode(lib, w, durations=dur, options=o) == -3
    o = binding.tdt_options_t(); o.projections = 2
    assert _decode(lib, w, durations=dur, options=o) == -3
    o = binding.tdt_options_t(); o.projections = 1; o.reuse_enc_proj = 1   # nothing to reuse on the fly
    assert _decode(lib, w, durations=dur, options=o) == -3
    o = binding.tdt_options_t(); o.projections = 1; o.algorithm = 1        # label-looping only
    assert _decode(lib, w, durations=dur, options=o) == -3
    o = binding.tdt_options_t(); o.joint_tiles = 65
    assert _decode(lib, w, durations=dur, options=o) == -3
    o = binding.tdt_options_t(); o.algorithm = 2
    assert _decode(lib, w, durations=dur, options=o) == -3
    o = binding.tdt_options_t(); o.wait_timeout_us = -1
    assert _decode(lib, w, durations=dur, options=o) == -3
    # workspace
    assert _decode(lib, w, durations=dur, ws=None) == -5
    assert _decode(lib, w, durations=dur, ws=4096 + 8) == -5
    assert _decode(lib, w, durations=dur, ws_bytes=1024) == -5
    # encoder projection entry point
    assert lib.tdt_encoder_projection(None, 10, C.byref(w), 4096, None) == -1
    assert lib.tdt_encoder_projection(4096, -1, C.byref(w), 4096, None) == -2
    assert lib.tdt_encoder_projection(4096, 10, None, 4096, None) == -1


def test_chunk_entry_point_rejects_before_device_work(lib):
    cfg = synth.CFG3
    w = _weights(cfg)
    dur = (C.c_int32 * len(cfg.durations))(*cfg.durations)

    def call(state, **kw):
        a = dict(enc=4096, B=2, T=10, S=3, u_cap=30, ws=4096)
        a.update(kw)
        return lib.tdt_greedy_decode_chunk(a["enc"], 4096, a["B"], a["T"], C.byref(w), dur, a["S"],
                                           a["u_cap"], 4096, 4096, 4096, 4096, 4096, None, state,
                                           a["ws"], 1 << 40, None, None)

    assert call(None) == -1                  # no state
    assert call(4096 + 4) == -5              # misaligned state
    assert call(4096, enc=None) == -1        # then the checks of tdt_greedy_decode
    assert call(4096, B=0) == -2
    assert call(4096, ws=None) == -5
    # a chunk may be shorter than the longest duration
    dur_long = (C.c_int32 * 5)(0, 1, 2, 3, 1 << 21)
    assert lib.tdt_greedy_decode_chunk(4096, 4096, 2, 1, C.byref(w), dur_long, 3, 30, 4096, 4096,
                                       4096, 4096, 4096, None, 4096, None, 0, None, None) == -4
    assert call(4096, T=1, ws=None) == -5    # durations {0..4} pass with one-frame chunks


def test_state_bytes(lib):
    cfg = synth.CFG5                          # two LSTM layers
    w = _weights(cfg)
    n = binding.tdt_state_bytes(w, cfg.B)
    ints = (cfg.B * 4 + 255) // 256 * 256
    fl = (cfg.pred_layers * cfg.B * cfg.h_pred * 4 + 255) // 256 * 256
    assert n == 4 * ints + 2 * fl
    assert binding.tdt_state_bytes(_weights(synth.CFG4), 128) == 4 * 512      # stateless: labels only
    size = C.c_size_t()
    assert lib.tdt_state_bytes(None, 1, C.byref(size)) == -1
    assert lib.tdt_state_bytes(C.byref(w), 0, C.byref(size)) == -2
    assert lib.tdt_state_bytes(C.byref(w), 1, None) == -1


def test_static_entry_point_refuses_sizes_beyond_its_array(lib):
    """tdt_greedy_decode_static checks the sizes against the array it holds before any device
    work (so this is safe without a GPU)."""
    cfg = synth.CFG2_B128                    # 82 MB of projected frames alone
    w = _weights(cfg)
    assert binding.tdt_workspace_bytes(w, cfg.B, cfg.T, 100) > binding.TDT_STATIC_SCRATCH_BYTES
    rc = lib.tdt_greedy_decode_static(4096, 4096, cfg.B, cfg.T, C.byref(w), None, 3, 30, 4096, 4096,
                                      4096, 4096, 4096, None, None, None)
    assert rc == binding.TDT_ERR_TOO_LARGE
    assert binding.tdt_status_string(rc) != "unknown status"
    assert lib.tdt_greedy_decode_static(4096, 4096, 0, 10, C.byref(w), None, 3, 30, 4096, 4096, 4096,
                                        4096, 4096, None, None, None) == -2
    assert lib.tdt_greedy_decode_static(4096, 4096, 2, 10, None, None, 3, 30, 4096, 4096, 4096,
                                        4096, 4096, None, None, None) == -1
