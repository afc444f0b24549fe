"""The entry point that allocates nothing (tdt_greedy_decode_static): its workspace is an array
inside the library's device image.  Called through the C ABI and compared with
tdt_greedy_decode on the same inputs -- the same kernels in the same launch shape, so every
output must be identical bit for bit -- on two calls in a row, the second with a smaller input
(the array still holds what the first call left there)."""
from __future__ import annotations

import ctypes as C

import numpy as np
import pytest

import parity
from paper_2406_06220_amd import synth

pytestmark = pytest.mark.gpu


def _both(binding, cfg, w, enc, ln, u_cap):
    import torch
    model = binding.DeviceModel(cfg, w)
    B, T = len(ln), enc.shape[1]
    enc_d = model.upload_enc(enc)
    len_d = torch.from_numpy(np.ascontiguousarray(ln, np.int32)).to(model.device)
    ref = binding.Decoder(model, B, T, u_cap)
    assert ref.ws_bytes <= binding.TDT_STATIC_SCRATCH_BYTES
    ref(enc_d, len_d)
    want = ref.results()
    assert want["stats"]["abort"] == 0
    dev = model.device
    out = dict(labels=torch.full((B, u_cap), -1, dtype=torch.int32, device=dev),
               frames=torch.full((B, u_cap), -1, dtype=torch.int32, device=dev),
               len=torch.full((B,), -1, dtype=torch.int32, device=dev),
               score=torch.full((B,), 7.0, dtype=torch.float32, device=dev),
               status=torch.full((B,), -1, dtype=torch.int32, device=dev))
    stats = torch.zeros(binding.TDT_STAT_COUNT, dtype=torch.int64, device=dev)
    parity.announce(f"tdt_greedy_decode_static cfg={cfg.name} B={B} T={T} u_cap={u_cap}")
    binding.tdt_greedy_decode_static(
        enc_d.data_ptr(), len_d.data_ptr(), B, T, model.c,
        list(cfg.durations) if cfg.durations else None, cfg.max_symbols, u_cap,
        out["labels"].data_ptr(), out["frames"].data_ptr(), out["len"].data_ptr(),
        out["score"].data_ptr(), out["status"].data_ptr(), stats.data_ptr(), None,
        torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    got = {k: v.cpu().numpy() for k, v in out.items()}
    assert int(stats[binding.TDT_STAT_NAMES["abort"]]) == 0
    for key in ("len", "score", "status"):
        assert (got[key] == want[key]).all(), key
    for b in range(B):
        n = int(want["len"][b])
        assert (got["labels"][b, :n] == want["labels"][b, :n]).all()
        assert (got["frames"][b, :n] == want["frames"][b, :n]).all()
    return got


def test_static_scratch_entry_point_matches_the_workspace_one(oracle_lib):
    import torch
    assert torch.cuda.is_available(), "this test needs the MI355X"
    from paper_2406_06220_amd import binding
    binding.load_library()
    # first call: the TDT model of the benchmark at full size (B=32, T=250: 37 MB of the 64 MiB)
    cfg = synth.CFG3
    w = synth.generate_model(cfg)
    enc, ln = synth.generate_inputs(cfg)
    u_cap = cfg.T * cfg.max_symbols
    got = _both(binding, cfg, w, enc, ln, u_cap)
    res = parity.compare(oracle_lib, oracle_lib.OracleModel(cfg, w), cfg, enc, ln, got, u_cap)
    assert res["replayed"] <= 3, res
    # second call right behind it, smaller: fewer utterances, fewer frames, another model
    cfg2 = synth.small_config("g_static_small", dtype="bf16", pred_kind="lstm", pred_layers=2,
                              durations=(0, 1, 2, 3), d_enc=40, h_pred=72, emb_dim=24, h_joint=104,
                              vocab=45, B=9, T=33, len_lo=0, len_hi=33, seed=157,
                              default_blank_bias=0.6, max_symbols=5)
    w2 = synth.generate_model(cfg2)
    enc2, ln2 = synth.generate_inputs(cfg2)
    u2 = cfg2.T * cfg2.max_symbols
    got2 = _both(binding, cfg2, w2, enc2, ln2, u2)
    res2 = parity.compare(oracle_lib, oracle_lib.OracleModel(cfg2, w2), cfg2, enc2, ln2, got2, u2)
    assert res2["replayed"] <= 1, res2
    # sizes beyond the array are refused before anything is enqueued
    big = synth.CFG2_B128
    wb = binding.DeviceModel(big, synth.generate_model(big))
    with pytest.raises(binding.TdtError) as e:
        binding.tdt_greedy_decode_static(4096, 4096, big.B, big.T, wb.c, None, 10, 100,
                                         4096, 4096, 4096, 4096, 4096, 0, None, 0)
    assert e.value.code == binding.TDT_ERR_TOO_LARGE
