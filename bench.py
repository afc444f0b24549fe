"""Benchmark of the label-looping greedy decoder on one MI355X.

A "step" is one pass of the whole hot path over one synthetic batch: encoder
projection of all B*T frames, then the device-resident label-looping decode
(predictor steps, predictor projections, fused joint + argmax, hypothesis
updates) -- the paper's "non-encoder" time (Sec. 4).  Inputs and weights are
resident in HBM before the timed region starts.

Prints ONE JSON line: whole-job throughput in decoded encoder frames/s, the
roofline figures of the dominant kernel (the persistent decode kernel), and the
CPU oracle timed beside it on the host cores of the same box.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth


def matrix_bytes(cfg):
    """Bytes of the matrices the decode kernel streams: per predictor pass (the recurrent matrix of
    the first LSTM layer -- its input product is a per-label table --, both matrices of every
    deeper layer and the predictor projection; nothing for a stateless predictor, whose
    projected output is tabulated per label) and per joint pass (the output matrix)."""
    wb = 2 if cfg.dtype == "bf16" else 4
    H, Hp, O = cfg.h_joint, cfg.h_pred, cfg.n_out
    pred = 0
    if cfg.pred_kind == "lstm":
        pred = H * Hp * wb + 4 * Hp * Hp * wb + (cfg.pred_layers - 1) * 8 * Hp * Hp * wb
    return pred, O * H * wb


def row_bytes(cfg):
    """Bytes per predictor row (LSTM: the label's table row of the first layer, the recurrent
    pre-activations, cell state read and written, hidden state written, per layer) and per scored
    (hypothesis, frame) row (the projected encoder frame and the projected predictor output, or
    the table rows that make it up), all float32."""
    H, Hp = cfg.h_joint, cfg.h_pred
    if cfg.pred_kind == "lstm":
        return cfg.pred_layers * (4 + 4 + 2 + 1) * Hp * 4, 2 * H * 4
    return 0, (1 + cfg.pred_layers) * H * 4


def algorithmic_bytes(cfg, stats):
    """Two counts of the bytes the method has to move for the passes the decode kernel executed.
    `per_group_pass`: every pass of every hypothesis group streams the matrices (each group runs
    its own label loop); it grows with the number of groups at constant time.  `one_stream_per_step`:
    the matrices once per dependent step of the slowest group -- its label-loop iterations and its
    joint passes -- which does not depend on how the batch is split.  Both include the per-row
    bytes of all rows."""
    pred, joint = matrix_bytes(cfg)
    prow, jrow = row_bytes(cfg)
    rows = stats["pred_rows"] * prow + stats["joint_rows"] * jrow
    per_group = stats["pred_passes"] * pred + stats["joint_passes"] * joint + rows
    one_stream = stats["outer_max"] * pred + stats["joint_passes_max"] * joint + rows
    return float(per_group), float(one_stream)


def roofline_block(cfg, stats, kernel_ms, kernel_ms_min=None):
    per_group, one_stream = algorithmic_bytes(cfg, stats)
    k_s = kernel_ms * 1e-3
    blk = {"bound": "hbm", "kernel": "decode_kernel",
           "achieved": per_group / k_s / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
           "frac": per_group / k_s / 1e9 / HBM_PEAK_GBS,
           "algorithmic_bytes_per_launch": per_group,
           "achieved_one_stream_per_step": one_stream / k_s / 1e9,
           "frac_one_stream_per_step": one_stream / k_s / 1e9 / HBM_PEAK_GBS,
           "algorithmic_bytes_one_stream_per_step": one_stream,
           "kernel_ms": kernel_ms,
           "traffic": traffic_from_profiles(cfg.name),
           "traffic_source": "profiles/hbm_traffic.json (rocprofv3 FETCH_SIZE / WRITE_SIZE of an earlier "
                             "run of this command, not measured in this run)"}
    if kernel_ms_min is not None:
        blk["kernel_ms_min"] = kernel_ms_min
    return blk


def time_workload(cfg, steps, warmup, window=0, n_clusters=0, joint_tiles=0, algorithm=0, projections=0,
                  joint_kernel=0):
    import torch
    from paper_2406_06220_amd import binding, synth
    dev = "cuda:0"
    w = synth.generate_model(cfg)
    enc, ln = synth.generate_inputs(cfg)
    u_cap = cfg.T * cfg.max_symbols
    model = binding.DeviceModel(cfg, w, dev)
    dec = binding.Decoder(model, cfg.B, cfg.T, u_cap, window=window, n_clusters=n_clusters,
                          joint_tiles=joint_tiles, algorithm=algorithm, projections=projections,
                          joint_kernel=joint_kernel)
    enc_d = model.upload_enc(enc)
    len_d = torch.from_numpy(ln).to(dev)
    stream = torch.cuda.current_stream(dev)
    for _ in range(max(warmup, 1)):
        dec(enc_d, len_d, stream=stream)
    out = dec.results()
    assert out["stats"]["abort"] == 0, "device-side wait timed out"
    # ---- whole hot path, K steps
    torch.cuda.synchronize(dev)
    t0 = time.perf_counter()
    for _ in range(steps):
        dec(enc_d, len_d, stream=stream)
    torch.cuda.synchronize(dev)
    dt = (time.perf_counter() - t0) / steps
    frames = int(np.clip(ln, 0, cfg.T).sum())
    if projections:   # no projection is left in the workspace to time the kernel apart with
        return dict(cfg=cfg, out=out, sec_per_step=dt, frames=frames, u_cap=u_cap)
    # ---- the decode kernel on its own: HIP events on the launch stream around a call
    #      that reuses the projection already in the workspace
    dec.options.reuse_enc_proj = 1
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(steps)]
    for a, b in ev:
        a.record(stream)
        dec(enc_d, len_d, stream=stream)
        b.record(stream)
    torch.cuda.synchronize(dev)
    dec.options.reuse_enc_proj = 0
    k_all = [a.elapsed_time(b) for a, b in ev]
    k_ms = float(np.mean(k_all))
    # ---- the encoder projection on its own (the dense contraction of the path), as the decode
    #      call runs it: over the valid frames of every utterance
    proj = torch.empty((cfg.B * cfg.T, cfg.h_joint), dtype=torch.float32, device=dev)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(steps)]
    for a, b in ev:
        a.record(stream)
        binding.tdt_encoder_projection_valid(enc_d.data_ptr(), len_d.data_ptr(), cfg.B, cfg.T, model.c,
                                             proj.data_ptr(), stream.cuda_stream)
        b.record(stream)
    torch.cuda.synchronize(dev)
    e_ms = float(np.mean([a.elapsed_time(b) for a, b in ev]))
    return dict(cfg=cfg, weights=w, enc=enc, len=ln, out=out, sec_per_step=dt, decode_kernel_ms=k_ms,
                decode_kernel_ms_min=float(np.min(k_all)), enc_proj_ms=e_ms, frames=frames, u_cap=u_cap)


def enc_proj_figures(cfg, ms, rows):
    """Rates of the encoder-projection GEMM over the `rows` valid frames of the batch."""
    wb = 2 if cfg.dtype == "bf16" else 4
    flops = 2.0 * rows * cfg.d_enc * cfg.h_joint
    nbytes = rows * cfg.d_enc * wb + cfg.d_enc * cfg.h_joint * wb + rows * cfg.h_joint * 4
    peak = 2500.0 if cfg.dtype == "bf16" else 157.3
    return {"kernel": "enc_proj", "ms": ms, "achieved_tflops": flops / (ms * 1e-3) / 1e12,
            "peak_tflops": peak, "frac_of_mfma_peak": flops / (ms * 1e-3) / 1e12 / peak,
            "achieved_gbs": nbytes / (ms * 1e-3) / 1e9, "frac_of_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "note": "an event pair around one launch; at this size launch overhead is part of it"}


def time_chunked(cfg, chunk_frames, steps, warmup):
    """The same batch fed in chunks of `chunk_frames` frames per utterance through
    tdt_greedy_decode_chunk (state cleared, then every chunk in turn = one step)."""
    import torch
    from paper_2406_06220_amd import binding, synth
    dev = "cuda:0"
    w = synth.generate_model(cfg)
    enc, ln = synth.generate_inputs(cfg)
    ln = np.clip(ln, 0, cfg.T)
    model = binding.DeviceModel(cfg, w, dev)
    state = binding.StreamState(model, cfg.B)
    dec = binding.ChunkDecoder(model, cfg.B, chunk_frames, chunk_frames * cfg.max_symbols, state)
    n_chunks = (int(ln.max()) + chunk_frames - 1) // chunk_frames
    feeds = []
    for c in range(n_chunks):
        lc = np.clip(ln - c * chunk_frames, 0, chunk_frames).astype(np.int32)
        ec = np.ascontiguousarray(enc[:, c * chunk_frames:(c + 1) * chunk_frames])
        if ec.shape[1] < chunk_frames:
            ec = np.concatenate([ec, np.zeros((cfg.B, chunk_frames - ec.shape[1], cfg.d_enc), np.float32)], 1)
        feeds.append((model.upload_enc(ec), torch.from_numpy(lc).to(dev)))
    stream = torch.cuda.current_stream(dev)

    def one_pass():
        state.reset()
        for e, l in feeds:
            dec(e, l, stream=stream)

    labels = 0
    for _ in range(max(warmup, 1)):
        state.reset()
        labels = 0
        for e, l in feeds:
            dec(e, l, stream=stream)
            r = dec.results()
            assert r["stats"]["abort"] == 0, "device-side wait timed out"
            labels += int(r["len"].sum())
    torch.cuda.synchronize(dev)
    t0 = time.perf_counter()
    for _ in range(steps):
        one_pass()
    torch.cuda.synchronize(dev)
    dt = (time.perf_counter() - t0) / steps
    frames = int(ln.sum())
    return dict(workload=cfg.name, chunk_frames=chunk_frames, chunks=n_chunks, value=frames / dt,
                unit="frames/s", us_per_chunk=dt / n_chunks * 1e6, labels=labels)


def cpu_baseline(res, min_seconds=10.0, max_runs=64):
    """The oracle as it stands on the host cores: the same batch decoded again and again with
    all threads until about `min_seconds` of wall time have passed (one utterance per
    thread at a time), and one pass over its first utterances on a single thread."""
    from oracle import oracle
    cfg = res["cfg"]
    om = oracle.OracleModel(cfg, res["weights"])
    frames = int(np.clip(res["len"], 0, cfg.T).sum())
    runs, r = 0, None
    t0 = time.perf_counter()
    while runs < max_runs and (runs == 0 or time.perf_counter() - t0 < min_seconds):
        r = oracle.decode_batch(om, res["enc"], res["len"], cfg.max_symbols, res["u_cap"])
        runs += 1
    dt = time.perf_counter() - t0
    # while we are here: the GPU result must be the oracle's
    same = all((res["out"]["len"][b] == r["len"][b]
                and (res["out"]["labels"][b, :r["len"][b]] == r["labels"][b, :r["len"][b]]).all())
               for b in range(cfg.B))
    n1 = min(cfg.B, 4)
    t1 = time.perf_counter()
    oracle.decode_batch(om, res["enc"][:n1], res["len"][:n1], cfg.max_symbols, res["u_cap"], n_threads=1)
    dt1 = time.perf_counter() - t1
    return dict(value=runs * frames / dt, unit="frames/s", cores=int(r["threads"]), kind="oracle",
                sample=f"the same batch of {cfg.B} utterances ({frames} frames) decoded {runs} times, "
                       f"{dt:.1f} s wall",
                single_thread={"value": int(np.clip(res["len"][:n1], 0, cfg.T).sum()) / dt1, "unit": "frames/s",
                               "sample": f"first {n1} utterances, one pass, {dt1:.1f} s wall"},
                labels_match_gpu=bool(same))


def describe(cfg):
    return (f"{cfg.name}: B={cfg.B} T={cfg.T} d_enc={cfg.d_enc} {cfg.pred_kind}x{cfg.pred_layers} "
            f"h_pred={cfg.h_pred} H={cfg.h_joint} V={cfg.vocab} D={cfg.n_dur} S={cfg.max_symbols}, "
            f"{cfg.dtype} weights, fp32 accumulation")


def config_block(cfg, r):
    """The figures of one workload as time_workload measured it."""
    st = r["out"]["stats"]
    return {"workload": describe(cfg), "value": r["frames"] / r["sec_per_step"], "unit": "frames/s",
            "ms_per_step": r["sec_per_step"] * 1e3, "us_per_batch": r["sec_per_step"] * 1e6,
            "frames_per_batch": r["frames"], "labels_per_batch": int(r["out"]["len"].sum()),
            "roofline": roofline_block(cfg, st, r["decode_kernel_ms"], r["decode_kernel_ms_min"]),
            "enc_proj": enc_proj_figures(cfg, r["enc_proj_ms"], r["frames"]),
            "decode_stats": st}


def release_device_memory():
    """Give what the finished workloads held back to the driver (the large configuration needs
    several GB)."""
    import gc
    import torch
    gc.collect()
    torch.cuda.synchronize()
    torch.cuda.empty_cache()


def traffic_from_profiles(name):
    """HBM bytes per launch from the committed rocprofv3 counter summary, if there is one."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(path):
        with open(path) as f:
            return json.load(f).get(name)
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg2_rnnt_lstm")
    ap.add_argument("--window", type=int, default=0)
    ap.add_argument("--clusters", type=int, default=0)
    ap.add_argument("--joint-kernel", type=int, default=0, help="0 automatic, 1 tiled, 2 streaming joint pass")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--no-extra", action="store_true", help="skip the B=128 line")
    ap.add_argument("--phase-timers", action="store_true",
                    help="load the profiling build of the library (python -m paper_2406_06220_amd.build "
                         "--phase-timers), whose statistics carry the per-phase wall-clock ticks")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device-to-device copy and a 256 MiB elementwise "
                         "kernel, so that a rocprofv3 --pmc run of this command holds dispatches of "
                         "known HBM traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU (hypotheses are independent, so a batch would "
              "shard across GPUs without any exchange); --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2406_06220_amd import binding, synth
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    if args.phase_timers:
        binding.LIB_PATH = binding.TIMERS_LIB_PATH
    binding.load_library()

    if args.copy_calibration:
        src = torch.ones(64 << 20, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                   # reads 256 MiB, writes 256 MiB (the runtime's copy kernel)
        torch.add(src, 1.0, out=dst)     # the same traffic from an ordinary elementwise kernel
        torch.cuda.synchronize()
        del src, dst

    cfg = synth.CONFIGS[args.workload]
    res = time_workload(cfg, args.steps, args.warmup, args.window, args.clusters, joint_kernel=args.joint_kernel)
    st = res["out"]["stats"]
    line = {
        "metric": "decoded encoder frames/sec (greedy decode only)",
        "value": res["frames"] / res["sec_per_step"],
        "unit": "frames/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["sec_per_step"] * 1e3,
        "us_per_batch": res["sec_per_step"] * 1e6,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == "bf16" else "f32", "data": "synthetic",
        "dtype_detail": ("bfloat16 weights and encoder output on the bf16 matrix cores; float32 activations, each "
                         "split exactly into three bfloat16 terms; float32 accumulation"
                         if cfg.dtype == "bf16" else "float32 throughout, float32 matrix-core products"),
        "config": {"workload": describe(cfg),
                   "frames_per_batch": res["frames"],
                   "labels_per_batch": int(res["out"]["len"].sum()),
                   "window": args.window or "auto", "clusters": args.clusters or "auto"},
        "decode_stats": st,
        "roofline": roofline_block(cfg, st, res["decode_kernel_ms"], res["decode_kernel_ms_min"]),
        "enc_proj": enc_proj_figures(cfg, res["enc_proj_ms"], res["frames"]),
    }
    if not args.no_extra and args.workload == "cfg2_rnnt_lstm":
        cfg_b = synth.CONFIGS["cfg2_rnnt_lstm_b128"]
        rb = time_workload(cfg_b, max(args.steps // 2, 3), max(args.warmup, 1), args.window, args.clusters)
        line["b128"] = config_block(cfg_b, rb)
        del rb
        # the other benchmark configurations (the TDT model at both batch sizes, the stateless
        # model, the large TDT model), each timed like the headline workload, fewer steps
        line["configs"] = {}
        for name, steps in (("cfg3_tdt_lstm", 10), ("cfg3_tdt_lstm_b128", 10), ("cfg4_rnnt_stateless", 10),
                            ("cfg5_large_tdt", 3)):
            c = synth.CONFIGS[name]
            r = time_workload(c, min(steps, args.steps), 1)
            line["configs"][name] = config_block(c, r)
            del r
            release_device_memory()
        # the same batch fed piece by piece (50 frames = 2 s of audio at config 2's frame rate)
        line["chunked"] = time_chunked(cfg, 50, max(args.steps // 2, 3), max(args.warmup, 1))
        line["chunked"]["labels_match_whole"] = bool(line["chunked"]["labels"] == int(res["out"]["len"].sum()))
        # the conventional loop order (Algorithm 2) on the same kernels: one lock step as
        # printed, and with the batch split into independent groups like the default path
        fl = {}
        for key, ncl in (("as_printed", 1), ("independent_groups", 0)):
            rf = time_workload(cfg, max(args.steps // 4, 2), 1, n_clusters=ncl, algorithm=1)
            same = bool((rf["out"]["len"] == res["out"]["len"]).all()
                        and (rf["out"]["labels"] == res["out"]["labels"]).all())
            fl[key] = {"ms_per_batch": rf["sec_per_step"] * 1e3, "value": rf["frames"] / rf["sec_per_step"],
                       "unit": "frames/s", "steps_of_the_slowest_group": rf["out"]["stats"]["outer_max"],
                       "label_looping_speedup": rf["sec_per_step"] / res["sec_per_step"],
                       "labels_match_label_looping": same}
        line["frame_looping"] = fl
        # the paper's other ablation (Sec. 3.4, Table 3): no projections ahead of the loops, every
        # joint pass projects the encoder frames and predictor outputs it is about to score
        ro = time_workload(cfg, max(args.steps // 2, 3), 1, args.window, args.clusters, projections=1)
        line["projections_on_the_fly"] = {
            "ms_per_batch": ro["sec_per_step"] * 1e3, "value": ro["frames"] / ro["sec_per_step"],
            "unit": "frames/s", "joint_passes": ro["out"]["stats"]["joint_passes"],
            "joint_rows": ro["out"]["stats"]["joint_rows"],
            "precomputed_speedup": ro["sec_per_step"] / res["sec_per_step"],
            "labels_match_precomputed": bool((ro["out"]["len"] == res["out"]["len"]).all()
                                             and (ro["out"]["labels"] == res["out"]["labels"]).all())}
    if not args.no_cpu:
        line["cpu_baseline"] = cpu_baseline(res)
    print(json.dumps(line))
    sys.stdout.flush()
    # Nothing of this program's should still hold device memory, events or streams when the
    # interpreter runs its exit handlers (under a profiler the runtime may be finalised before
    # them): drop the tensors, drain the device, return the cached blocks.
    del res
    release_device_memory()


if __name__ == "__main__":
    main()
