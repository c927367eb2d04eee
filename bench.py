#!/usr/bin/env python3
"""Benchmark of the LoMA attention hot path on one MI355X.

One step = one pass of the whole hot path at the two largest single-GPU configurations:
    mask leg      1 x loma_mask_attn_fwd    config 4: B1 H32 d128 t32 c8, 60 chunks (S = 32640), bf16
                                            (two tensor sets in rotation: a set is 1.07 GB, the Infinity Cache 256 MB)
    compress leg  1 x loma_compress_step    config 5: B64 H32 d128 t16 c16, 512 prior chunks
    decode leg    128 x loma_decode_attn    config 5: 8208 memory KVs + the reading zone growing from 1 to 128 rows
                                            (8.9 GB of cache; after the leg the next step starts from the same state)
`value` is the useful TFLOP/s of the mask leg (unmasked pairs only), the decode leg's GB/s is reported next to
it, each against the chip's published peak; `roofline` describes the kernel the step spends its time in (decode),
`roofline_long_context_mask` the mask kernel.  Legs are bracketed by HIP events on the launch stream.  The smaller
configurations (2: Llama-7B-shaped mask pass, 3: generation with 32 layer caches), the prompt form, the gradients
and the layered decode are timed afterwards on their own: median of 20 samples after 5 warm-up samples, every
sample over tensors in rotation.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--layers 32] [--no-extra] [--no-cpu] [--no-peaks]
    python bench.py --copy-calibration     three plain 1 GiB device copies and nothing else: the known
                                           traffic the FETCH_SIZE / WRITE_SIZE counters are scaled by
No random-number kernel runs on the GPU: tensors are tiled from a seeded pool drawn on the host (bit patterns
differ from call to call of the tiling, values are unit normals), so the script also runs under counter collection.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E
MFMA_BF16_PEAK_TF = 2500.0  # MI355X dense bf16
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "bench_hbm_traffic_pmc.md")


def profile_traffic(path=TRAFFIC_PROFILE):
    """HBM bytes per launch of every kernel listed in the committed counter profile: rocprofv3 FETCH_SIZE and
    WRITE_SIZE (KiB per dispatch), each scaled by the factor the same counter showed for a plain copy of known
    size (the profile's calibration table).  Counters cannot be read inside a timed run, so these are the
    profile's figures, keyed by kernel name; a kernel that is not in the profile has no traffic figure."""
    if not os.path.exists(path):
        return {}
    text = open(path).read()
    factor = {}
    for name in ("FETCH_SIZE", "WRITE_SIZE"):
        m = re.search(r"^\|\s*%s\s*\|[^|]*\|[^|]*\|\s*x\s*([0-9.]+)\s*\|" % name, text, flags=re.M)
        if not m:
            return {}
        factor[name] = float(m.group(1))
    out = {}
    # rows: | `kernel` | config N ... | dispatches | FETCH_SIZE | WRITE_SIZE | ...   keyed "kernel @cN" ("@cNxL": L layers per launch)
    for m in re.finditer(r"^\|\s*`([^`]+)`\s*\|\s*config (\d+)(?: \((\d+) layers per launch\))?[^|]*\|\s*\d+\s*\|\s*([0-9.]+)\s*\|\s*([0-9.]+)\s*\|",
                         text, flags=re.M):
        key = "%s @c%s%s" % (m.group(1), m.group(2), ("x" + m.group(3)) if m.group(3) else "")
        out[key] = (factor["FETCH_SIZE"] * float(m.group(4)) + factor["WRITE_SIZE"] * float(m.group(5))) * 1024.0
    return out


# Kernels behind every roofline object of the output line, with the configuration tag the committed counter profile
# lists them under ("c3x{L}": L layer caches per launch).
ROOFLINE_KERNELS = {
    "roofline": ("c5", ("decode_split_kernel<128, 4, false, false>", "decode_combine_kernel<128, false>")),
    "roofline_long_context_mask": ("c4", ("mask_attn_kernel<128, 4, 64, true>",)),
    "roofline_high_ratio_compress": ("c5", ("compress_kernel<128, 1, 32, false>",)),
    "roofline_long_context_mask_bwd": ("c4", ("bwd_dq_kernel<128, 4>", "bwd_dkv_kernel<128, 4>")),
    "roofline_mask": ("c2", ("mask_attn_kernel<128, 2, 32, false>",)),
    "roofline_mask_bwd": ("c2", ("bwd_dq_kernel<128, 2>", "bwd_dkv_kernel<128, 2>", "bwd_reduce_kernel<128>")),
    "roofline_decode": ("c3", ("decode_split_kernel<128, 16, false, false>",)),
    "roofline_decode_layers": ("c3x{L}", ("decode_split_kernel<128, 16, true, false>",)),
    "roofline_prefill": ("c3", ("prefill_kernel<128, 4, 64, 2, 4>",)),
    "roofline_decode_gqa": ("c5", ("decode_split_gqa_kernel<128, 4, 16, 4, false>",)),
}


def traffic_of(table, config, *kernels):
    """Sum of the profile's traffic over the kernels of one call on one configuration ("c4", "c3x32": 32 layers per
    launch), or None if one of them is missing."""
    keys = ["%s @%s" % (k, config) for k in kernels]
    if not all(k in table for k in keys):
        return None
    return sum(table[k] for k in keys)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--layers", type=int, default=32, help="layer caches of the generation configuration (extras)")
    ap.add_argument("--samples", type=int, default=20, help="timed samples per extra (median reported)")
    ap.add_argument("--no-extra", action="store_true", help="only the step: skip configurations 2 and 3, prompt form, gradients")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-peaks", action="store_true", help="skip the measured MFMA-loop and stream peaks")
    ap.add_argument("--copy-calibration", action="store_true", help="run three 1 GiB device copies and exit")
    return ap.parse_args()


def time_median(fn, calls, samples=20, warmup=5):
    """Median over `samples` samples of the milliseconds per call; a sample is `calls` back-to-back calls fn(i)
    bracketed by HIP events on the current stream.  `warmup` untimed samples come first."""
    import torch
    k = 0
    for _ in range(warmup):
        for _ in range(calls):
            fn(k)
            k += 1
    torch.cuda.synchronize()
    pairs = []
    for _ in range(samples):
        a = torch.cuda.Event(enable_timing=True)
        b = torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(calls):
            fn(k)
            k += 1
        b.record()
        pairs.append((a, b))
    torch.cuda.synchronize()
    return statistics.median(a.elapsed_time(b) for a, b in pairs) / calls


def measured_peaks(samples):
    """What this machine reaches with nothing in the way: a pure v_mfma_f32_32x32x16_bf16 loop on every SIMD, a plain
    copy and a plain read of 2 GiB."""
    import torch
    from paper_2401_09486_amd import build as hb
    lib = ctypes.CDLL(hb.PEAKS_LIB)
    vp = ctypes.c_void_p
    lib.loma_peaks_mfma_loop.argtypes = [ctypes.c_int, ctypes.c_int, vp, vp]
    lib.loma_peaks_mfma_loop.restype = ctypes.c_double
    lib.loma_peaks_stream_copy.argtypes = [vp, vp, ctypes.c_size_t, ctypes.c_int, vp]
    lib.loma_peaks_stream_read.argtypes = [vp, ctypes.c_size_t, ctypes.c_int, vp, vp]
    st = torch.cuda.current_stream().cuda_stream
    sink = torch.zeros(64, dtype=torch.float32, device="cuda")
    wgs, iters = 256 * 8, 2048
    flops = [0.0]

    def mfma(i):
        flops[0] = lib.loma_peaks_mfma_loop(wgs, iters, sink.data_ptr(), st)
    ms = time_median(mfma, 1, samples)
    assert flops[0] > 0
    n = 1 << 31
    src = torch.ones(n, dtype=torch.uint8, device="cuda")
    dst = torch.empty(n, dtype=torch.uint8, device="cuda")
    cms = time_median(lambda i: lib.loma_peaks_stream_copy(src.data_ptr(), dst.data_ptr(), n, 256 * 16, st), 1, samples)
    rms = time_median(lambda i: lib.loma_peaks_stream_read(src.data_ptr(), n, 256 * 16, sink.data_ptr(), st), 1, samples)
    tf = flops[0] / (ms * 1e-3) / 1e12
    # what a vector instruction of the softmax occupies a SIMD for, next to the 32x32x16 MFMA (nanoseconds per
    # instruction and SIMD; the clock differs between the loops, so no cycle counts)
    lib.loma_peaks_valu_loop.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, vp]
    lib.loma_peaks_valu_loop.restype = ctypes.c_double
    simd_ns = {"v_mfma_f32_32x32x16_bf16_8_waves_per_simd": ms * 1e6 / (wgs * 4 / 1024 * iters * 8)}
    for kind, name in ((0, "v_exp_f32"), (1, "v_fma_f32")):
        for waves in (4, 8):
            count = [0.0]

            def run(i):
                count[0] = lib.loma_peaks_valu_loop(kind, waves, 256, 8192, sink.data_ptr(), st)
            vms = time_median(run, 1, samples)
            assert count[0] > 0
            simd_ns[f"{name}_{waves // 4}_wave{'s' if waves > 4 else ''}_per_simd"] = vms * 1e6 / (count[0] * (waves // 4))
    return {"mfma_loop_tflops": tf, "ns_per_instruction_and_simd": simd_ns, "mfma_loop_frac_of_peak": tf / MFMA_BF16_PEAK_TF,
            "mfma_loop": f"v_mfma_f32_32x32x16_bf16, {wgs} workgroups x 4 waves x {iters * 8} instructions",
            "stream_copy_GBps": 2.0 * n / (cms * 1e-3) / 1e9, "stream_read_GBps": n / (rms * 1e-3) / 1e9,
            "stream_copy_frac_of_peak": 2.0 * n / (cms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "stream_read_frac_of_peak": n / (rms * 1e-3) / 1e9 / HBM_PEAK_GBS, "stream_bytes": n}


def cpu_baseline(wl):
    """The fp64 oracle as it stands, on the host cores, on a bounded sample of the step's workload: whole (b,h)
    pairs of the long-context mask pass, and a few decode steps of a few (b,h) pairs of the high-ratio cache."""
    import numpy as np
    from oracle import c_oracle
    c_oracle.build()
    threads = c_oracle.num_threads()
    c4, c5 = wl.CONFIGS[3], wl.CONFIGS[4]
    npairs = c4.B * c4.H
    sub = wl.shrink(c4, H=npairs)
    q, k, v = wl.mask_inputs(sub)
    t0 = time.perf_counter()
    c_oracle.mask_attn(q, k, v, sub.t, sub.c, sub.n_chunks, sub.scale)
    dt_mask = time.perf_counter() - t0
    flops = wl.mask_pass_useful_flops(sub)
    # decode: 64 (b,h) pairs, 64 steps over 8192 memory keys + the first reading rows
    nb, nsteps = 64, 64
    g = wl.shrink(c5, B=1, H=nb, steps=nsteps)
    st = wl.gen_initial_state(g)
    orc = c_oracle.GenerationCache(st["k_mem"], st["v_mem"], g.prior_chunks, st["k_read"], st["v_read"], 0, g.t, g.c, g.scale)
    toks = [wl.gen_step_inputs(g, s) for s in range(nsteps)]
    t0 = time.perf_counter()
    for s in range(nsteps):
        orc.decode(*toks[s])
    dt_dec = time.perf_counter() - t0
    dec_bytes = sum(wl.decode_bytes(1, nb, g.d, g.prior_chunks * g.t + s + 1, g.dtype) for s in range(nsteps))
    return {"value": flops / dt_mask / 1e12, "unit": "TFLOP/s (useful, fp64, mask pass)", "cores": threads, "kind": "oracle",
            "seconds": dt_mask + dt_dec, "decode_GBps": dec_bytes / dt_dec / 1e9,
            "sample": f"mask leg: all {sub.S} rows of {npairs} of the {c4.B * c4.H} (b,h) pairs of {c4.name} ({dt_mask:.1f} s); "
                      f"decode leg: {nsteps} steps of {nb} of the {c5.B * c5.H} (b,h) pairs of {c5.name} over {g.prior_chunks * g.t} "
                      f"memory KVs ({dt_dec:.1f} s)"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (every (b,h) pair is independent, so the path would shard over "
              "batch or heads without any exchange); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2401_09486_amd import loma
    from paper_2401_09486_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.copy_calibration:
        src = torch.ones(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda")
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"bytes_read_per_copy": 1 << 30, "bytes_written_per_copy": 1 << 30, "copies": 3}}))
        return
    pool = wl.TiledPool(wl.SEED_BASE)
    traffic = profile_traffic()
    K, NS = args.steps, args.samples
    c2, c3, c4, c5 = wl.CONFIGS[1], wl.CONFIGS[2], wl.CONFIGS[3], wl.CONFIGS[4]

    def bf16_empty(shape):
        return torch.empty(shape, dtype=torch.bfloat16, device="cuda")

    # ---- the step: config 4 mask pass, config 5 compress + 128 decode steps -------------------------------------
    shp4 = (c4.B, c4.H, c4.S, c4.d)
    sets4 = [tuple(pool.tensor(shp4, c4.value_scale) for _ in range(3)) + (bf16_empty(shp4),) for _ in range(2)]
    cap5 = c5.mem_capacity
    st5 = {"k_mem": pool.tensor((c5.B, c5.H, cap5, c5.d)), "v_mem": pool.tensor((c5.B, c5.H, cap5, c5.d))}
    reads5 = [(pool.tensor((c5.B, c5.H, c5.R, c5.d)), pool.tensor((c5.B, c5.H, c5.R, c5.d))) for _ in range(2)]
    qm5, km5, vm5 = (pool.tensor((c5.B, c5.H, c5.t, c5.d), s) for s in (c5.q_scale, 1.0, 1.0))
    om5 = bf16_empty((c5.B, c5.H, c5.t, c5.d))
    q5 = pool.tensor((c5.B, c5.H, 1, c5.d), c5.q_scale)
    kn5, vn5 = pool.tensor((c5.B, c5.H, 1, c5.d)), pool.tensor((c5.B, c5.H, 1, c5.d))
    o5 = bf16_empty((c5.B, c5.H, 1, c5.d))
    ws5 = torch.empty(max(loma.loma_decode_workspace_bytes(c5.B, c5.H, c5.d, c5.t, c5.c, c5.prior_chunks + 1), 16),
                      dtype=torch.uint8, device="cuda")
    nm5 = c5.prior_chunks + 1
    marks = []

    def mark():
        e = torch.cuda.Event(enable_timing=True)
        e.record()
        return e

    def step(i, record):
        q, k, v, o = sets4[i % 2]
        kr, vr = reads5[i % 2]
        e0 = mark()
        loma.loma_mask_attn_fwd(q, k, v, c4.t, c4.c, c4.n_chunks, c4.scale, out=o)
        e1 = mark()
        loma.loma_compress_step(qm5, km5, vm5, kr, vr, st5["k_mem"], st5["v_mem"], c5.t, c5.c, c5.prior_chunks, c5.scale, out=om5)
        e2 = mark()
        for f in range(c5.steps):
            loma.loma_decode_attn(q5, kn5, vn5, st5["k_mem"], st5["v_mem"], kr, vr, c5.t, c5.c, nm5, f, c5.scale, out=o5,
                                  workspace=ws5)
        e3 = mark()
        if record:
            marks.append((e0, e1, e2, e3))

    for i in range(args.warmup):
        step(i, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        step(args.warmup + i, True)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3

    mask_ms = sum(a.elapsed_time(b) for a, b, _, _ in marks) / K
    comp_ms = sum(b.elapsed_time(c) for _, b, c, _ in marks) / K
    dec_ms = sum(c.elapsed_time(d) for _, _, c, d in marks) / (K * c5.steps)
    mask_flops = wl.mask_pass_useful_flops(c4)
    mask_bytes = wl.mask_pass_bytes(c4)
    mask_tf = mask_flops / (mask_ms * 1e-3) / 1e12
    dec_bytes = sum(wl.decode_bytes(c5.B, c5.H, c5.d, nm5 * c5.t + f + 1, c5.dtype) for f in range(c5.steps)) / c5.steps
    dec_gbs = dec_bytes / (dec_ms * 1e-3) / 1e9
    comp_bytes = wl.compress_bytes(c5.B, c5.H, c5.d, c5.t, c5.c, c5.dtype)
    comp_flops = wl.compress_useful_flops(c5.B, c5.H, c5.d, c5.t, c5.c)
    (KDEC5, KCOMB5), (KMASK4,), (KCOMP5,) = (ROOFLINE_KERNELS[k][1] for k in ("roofline", "roofline_long_context_mask",
                                                                                 "roofline_high_ratio_compress"))

    result = {
        "metric": "LoMA-mask attn useful TFLOP/s + decode GB/s (frac of MI355X roofline)",
        "value": mask_tf, "unit": "TFLOP/s (useful, mask pass)",
        "n_gpus": 1, "steps": K, "warmup": args.warmup, "ms_per_step": wall_ms / K,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{c4.name} (B{c4.B} H{c4.H} d{c4.d} t{c4.t} c{c4.c} n{c4.n_chunks}, S={c4.S}) mask pass + "
                               f"{c5.name} (B{c5.B} H{c5.H} d{c5.d} t{c5.t} c{c5.c}, {c5.prior_chunks * c5.t} memory KVs) "
                               f"1 compress + {c5.steps} decode steps"},
        "long_context_mask": {"workload": c4.name, "useful_tflops": mask_tf, "frac_of_mfma_peak": mask_tf / MFMA_BF16_PEAK_TF,
                              "us_per_call": mask_ms * 1e3, "useful_flops": mask_flops, "bytes": mask_bytes,
                              "algorithmic_GBps": mask_bytes / (mask_ms * 1e-3) / 1e9,
                              "frac_of_hbm_peak": mask_bytes / (mask_ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "high_ratio_decode": {"workload": c5.name, "value": dec_gbs, "unit": "GB/s (algorithmic)",
                              "frac_of_hbm_peak": dec_gbs / HBM_PEAK_GBS, "ms_per_step": dec_ms, "bytes_per_step": dec_bytes,
                              "keys": f"{nm5 * c5.t}+1..{nm5 * c5.t}+{c5.steps}", "calls": K * c5.steps,
                              "compress_us": comp_ms * 1e3, "compress_GBps": comp_bytes / (comp_ms * 1e-3) / 1e9,
                              "compress_useful_tflops": comp_flops / (comp_ms * 1e-3) / 1e12},
        # the kernel the step spends its time in: the split-K decode kernel (HBM-bound); the figure includes the
        # tiny combine kernel that follows every launch of it
        "roofline": {"kernel": KDEC5, "bound": "hbm", "achieved": dec_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": dec_gbs / HBM_PEAK_GBS, "traffic": traffic_of(traffic, "c5", KDEC5, KCOMB5)},
        "roofline_long_context_mask": {"kernel": KMASK4, "bound": "mfma", "achieved": mask_tf, "peak": MFMA_BF16_PEAK_TF,
                                       "unit": "TFLOP/s", "frac": mask_tf / MFMA_BF16_PEAK_TF,
                                       "traffic": traffic_of(traffic, "c4", KMASK4)},
        "roofline_high_ratio_compress": {"kernel": KCOMP5, "bound": "hbm", "achieved": comp_bytes / (comp_ms * 1e-3) / 1e9,
                                         "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                         "frac": comp_bytes / (comp_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                         "traffic": traffic_of(traffic, "c5", KCOMP5)},
    }

    def roof_hbm(which, gbs, **fmt):
        config, kernels = ROOFLINE_KERNELS[which]
        config = config.format(**fmt)
        return {"kernel": " + ".join(kernels), "bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": gbs / HBM_PEAK_GBS, "traffic": traffic_of(traffic, config, *kernels)}

    def roof_mfma(which, tf):
        config, kernels = ROOFLINE_KERNELS[which]
        return {"kernel": " + ".join(kernels), "bound": "mfma", "achieved": tf, "peak": MFMA_BF16_PEAK_TF, "unit": "TFLOP/s",
                "frac": tf / MFMA_BF16_PEAK_TF, "traffic": traffic_of(traffic, config, *kernels)}

    def time_backward(cfg, sets):
        """sets: (q, k, v, out) tuples; forward once per set for out and lse, then the gradients in rotation."""
        packs = []
        for (q, k, v, o) in sets:
            lse = torch.empty((cfg.B, cfg.H, cfg.S), dtype=torch.float32, device="cuda")
            loma.loma_mask_attn_fwd(q, k, v, cfg.t, cfg.c, cfg.n_chunks, cfg.scale, out=o, lse=lse)
            packs.append((q, k, v, o, lse, pool.tensor(tuple(q.shape)), [torch.empty_like(q) for _ in range(3)]))
        wsb = torch.empty(loma.loma_mask_attn_bwd_workspace_bytes(cfg.B, cfg.H, cfg.d, cfg.t, cfg.c, cfg.n_chunks),
                          dtype=torch.uint8, device="cuda")

        def call(i):
            q, k, v, o, lse, g, gr = packs[i % len(packs)]
            loma.loma_mask_attn_bwd(q, k, v, o, lse, g, cfg.t, cfg.c, cfg.n_chunks, cfg.scale, dq=gr[0], dk=gr[1], dv=gr[2],
                                    workspace=wsb)
        ms = time_median(call, len(packs), NS)
        fl = 2.5 * wl.mask_pass_useful_flops(cfg)      # five products per visible pair against the forward's two
        by = 2.0 * wl.mask_pass_bytes(cfg)             # q, k, v, out, dout in; dq, dk, dv out
        return {"workload": cfg.name, "us_per_call": ms * 1e3, "useful_tflops": fl / (ms * 1e-3) / 1e12,
                "frac_of_mfma_peak": fl / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TF, "useful_flops": fl,
                "algorithmic_GBps": by / (ms * 1e-3) / 1e9, "frac_of_hbm_peak": by / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                "tensor_sets": len(packs)}

    if not args.no_extra:
        # ---- config 4 gradients (one set: 2.4 GB of tensors per call) -----------------------------------------------
        bw = time_backward(c4, sets4[:1])
        result["long_context_mask_bwd"] = bw
        result["roofline_long_context_mask_bwd"] = roof_mfma("roofline_long_context_mask_bwd", bw["useful_tflops"])
        del sets4
        torch.cuda.empty_cache()

        # ---- config 2: Llama-7B-shaped mask pass and its gradients, tensor sets in rotation --------------------------
        shp2 = (c2.B, c2.H, c2.S, c2.d)
        sets2 = [tuple(pool.tensor(shp2, c2.value_scale) for _ in range(3)) + (bf16_empty(shp2),) for _ in range(8)]
        ms = time_median(lambda i: loma.loma_mask_attn_fwd(*sets2[i % 8][:3], c2.t, c2.c, c2.n_chunks, c2.scale, out=sets2[i % 8][3]), 8, NS)
        fl2, by2 = wl.mask_pass_useful_flops(c2), wl.mask_pass_bytes(c2)
        result["mask"] = {"workload": c2.name, "useful_tflops": fl2 / (ms * 1e-3) / 1e12,
                          "frac_of_mfma_peak": fl2 / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TF, "us_per_call": ms * 1e3,
                          "algorithmic_GBps": by2 / (ms * 1e-3) / 1e9, "frac_of_hbm_peak": by2 / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                          "useful_flops": fl2, "bytes": by2, "tensor_sets": 8}
        result["roofline_mask"] = roof_hbm("roofline_mask", by2 / (ms * 1e-3) / 1e9)
        b2 = time_backward(c2, sets2[:3])
        result["mask_bwd"] = b2
        result["roofline_mask_bwd"] = roof_hbm("roofline_mask_bwd", b2["algorithmic_GBps"])
        del sets2
        torch.cuda.empty_cache()

        # ---- config 3: generation with one cache per layer (32 x 151 MB), per-layer launches and one launch for all --
        L = args.layers
        cap3 = (c3.prior_chunks + 1) * c3.t
        lay = []
        for _ in range(L):
            lay.append({"k_mem": pool.tensor((c3.B, c3.H, cap3, c3.d)), "v_mem": pool.tensor((c3.B, c3.H, cap3, c3.d)),
                        "k_read": pool.tensor((c3.B, c3.H, c3.R, c3.d)), "v_read": pool.tensor((c3.B, c3.H, c3.R, c3.d)),
                        "q_m": pool.tensor((c3.B, c3.H, c3.t, c3.d)), "k_m": pool.tensor((c3.B, c3.H, c3.t, c3.d)),
                        "v_m": pool.tensor((c3.B, c3.H, c3.t, c3.d)), "q": pool.tensor((c3.B, c3.H, 1, c3.d)),
                        "k_new": pool.tensor((c3.B, c3.H, 1, c3.d)), "v_new": pool.tensor((c3.B, c3.H, 1, c3.d)),
                        "out_m": bf16_empty((c3.B, c3.H, c3.t, c3.d)), "out": bf16_empty((c3.B, c3.H, 1, c3.d))})
        ws3 = torch.empty(max(loma.loma_decode_layers_workspace_bytes(L, c3.B, c3.H, c3.d, c3.t, c3.c, c3.prior_chunks + 1), 16),
                          dtype=torch.uint8, device="cuda")
        nm3 = c3.prior_chunks + 1
        nkeys3 = nm3 * c3.t

        def dec_single(i):
            g, f = lay[i % L], (i // L) % c3.R
            loma.loma_decode_attn(g["q"], g["k_new"], g["v_new"], g["k_mem"], g["v_mem"], g["k_read"], g["v_read"],
                                  c3.t, c3.c, nm3, f, c3.scale, out=g["out"], workspace=ws3)
        dms = time_median(dec_single, L * c3.R, NS, warmup=2)      # a sample = 64 tokens through all layers
        db3 = sum(wl.decode_bytes(c3.B, c3.H, c3.d, nkeys3 + f + 1, c3.dtype) for f in range(c3.R)) / c3.R
        result["decode"] = {"workload": f"{c3.name}: {L} layer caches, one launch per layer and token", "value": db3 / (dms * 1e-3) / 1e9,
                            "unit": "GB/s (algorithmic)", "frac_of_hbm_peak": db3 / (dms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                            "us_per_call": dms * 1e3, "bytes_per_call": db3, "keys": f"{nkeys3}+1..{nkeys3}+{c3.R}"}
        result["roofline_decode"] = roof_hbm("roofline_decode", db3 / (dms * 1e-3) / 1e9)
        tabs = {n: loma.pointer_table([g[n] for g in lay]) for n in ("q", "k_new", "v_new", "k_mem", "v_mem", "k_read", "v_read", "out")}

        def dec_layers(i):
            loma.loma_decode_attn_layers(tabs["q"], tabs["k_new"], tabs["v_new"], tabs["k_mem"], tabs["v_mem"], tabs["k_read"],
                                         tabs["v_read"], tabs["out"], L, c3.B, c3.H, c3.d, c3.t, c3.c, nm3, cap3, i % c3.R, c3.scale,
                                         workspace=ws3)
        lms = time_median(dec_layers, c3.R, NS, warmup=2)          # a sample = 64 tokens, one launch per token
        result["decode_layers"] = {"workload": f"{c3.name}: {L} layer caches, one launch per token for all layers",
                                   "value": L * db3 / (lms * 1e-3) / 1e9, "unit": "GB/s (algorithmic)",
                                   "frac_of_hbm_peak": L * db3 / (lms * 1e-3) / 1e9 / HBM_PEAK_GBS, "us_per_token": lms * 1e3,
                                   "us_per_token_layer_by_layer": L * dms * 1e3, "speedup_vs_layer_by_layer": L * dms / lms}
        result["roofline_decode_layers"] = roof_hbm("roofline_decode_layers", L * db3 / (lms * 1e-3) / 1e9, L=L)
        cms = time_median(lambda i: loma.loma_compress_step(lay[i % L]["q_m"], lay[i % L]["k_m"], lay[i % L]["v_m"], lay[i % L]["k_read"],
                                                            lay[i % L]["v_read"], lay[i % L]["k_mem"], lay[i % L]["v_mem"], c3.t, c3.c,
                                                            c3.prior_chunks, c3.scale, out=lay[i % L]["out_m"]), L, NS)
        cb3 = wl.compress_bytes(c3.B, c3.H, c3.d, c3.t, c3.c, c3.dtype)
        result["compress"] = {"workload": c3.name, "us_per_call": cms * 1e3, "algorithmic_GBps": cb3 / (cms * 1e-3) / 1e9,
                              "useful_tflops": wl.compress_useful_flops(c3.B, c3.H, c3.d, c3.t, c3.c) / (cms * 1e-3) / 1e12}
        # the prompt form on the same caches: a whole reading zone of new tokens per call
        npre = min(L, 8)
        pre = [tuple(pool.tensor((c3.B, c3.H, c3.R, c3.d)) for _ in range(3)) + (bf16_empty((c3.B, c3.H, c3.R, c3.d)),) for _ in range(npre)]
        pms = time_median(lambda i: loma.loma_prefill_attn(pre[i % npre][0], pre[i % npre][1], pre[i % npre][2], lay[i % L]["k_mem"],
                                                           lay[i % L]["v_mem"], lay[i % L]["k_read"], lay[i % L]["v_read"], c3.t, c3.c,
                                                           nm3, 0, c3.scale, out=pre[i % npre][3]), L, NS)
        nbh3 = c3.B * c3.H
        pbytes = nbh3 * (2 * nkeys3 * c3.d + 6 * c3.R * c3.d) * 2   # cache read once; q, k, v in, out and the appended K/V out
        pflops = 4.0 * c3.d * nbh3 * (c3.R * nkeys3 + c3.R * (c3.R + 1) / 2)
        result["prefill"] = {"workload": f"{c3.name}: {c3.R} new tokens per sequence over {nkeys3} memory KVs",
                             "us_per_call": pms * 1e3, "algorithmic_GBps": pbytes / (pms * 1e-3) / 1e9,
                             "frac_of_hbm_peak": pbytes / (pms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                             "useful_tflops": pflops / (pms * 1e-3) / 1e12, "vs_token_by_token": c3.R * dms / pms}
        result["roofline_prefill"] = roof_hbm("roofline_prefill", pbytes / (pms * 1e-3) / 1e9)
        del lay, pre, tabs
        torch.cuda.empty_cache()

        # ---- grouped-query decode: config 5's 32 query heads over 8 shared KV heads (a quarter of the cache per step) ---
        Hkv = 8
        gq = {"k_mem": pool.tensor((c5.B, Hkv, cap5, c5.d)), "v_mem": pool.tensor((c5.B, Hkv, cap5, c5.d)),
              "k_read": pool.tensor((c5.B, Hkv, c5.R, c5.d)), "v_read": pool.tensor((c5.B, Hkv, c5.R, c5.d)),
              "k_new": pool.tensor((c5.B, Hkv, 1, c5.d)), "v_new": pool.tensor((c5.B, Hkv, 1, c5.d))}
        wsg = torch.empty(max(loma.loma_decode_gqa_workspace_bytes(c5.B, c5.H, Hkv, c5.d), 16), dtype=torch.uint8, device="cuda")

        def dec_gqa(i):
            loma.loma_decode_attn_gqa(q5, gq["k_new"], gq["v_new"], gq["k_mem"], gq["v_mem"], gq["k_read"], gq["v_read"],
                                      c5.t, c5.c, nm5, i % c5.steps, c5.scale, out=o5, workspace=wsg)
        gms = time_median(dec_gqa, 16, NS, warmup=2)
        # K and V of the 8 KV heads once, their new rows in and out, q and out of all 32 heads
        nk5 = nm5 * c5.t
        gb5 = sum(c5.B * (Hkv * (2 * (nk5 + f + 1) * c5.d + 2 * c5.d) + c5.H * 2 * c5.d) * 2 for f in range(16)) / 16
        result["decode_gqa"] = {"workload": f"{c5.name} with {Hkv} KV heads under {c5.H} query heads", "value": gb5 / (gms * 1e-3) / 1e9,
                                "unit": "GB/s (algorithmic)", "frac_of_hbm_peak": gb5 / (gms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                "us_per_call": gms * 1e3, "bytes_per_call": gb5, "us_per_call_all_kv_heads": dec_ms * 1e3}
        result["roofline_decode_gqa"] = roof_hbm("roofline_decode_gqa", gb5 / (gms * 1e-3) / 1e9)
        del gq
        torch.cuda.empty_cache()

    if not args.no_peaks:
        mp = measured_peaks(NS)
        result["measured_peaks"] = mp
        result["long_context_mask"]["frac_of_measured_mfma_loop"] = mask_tf / mp["mfma_loop_tflops"]
        result["high_ratio_decode"]["frac_of_measured_stream_read"] = dec_gbs / mp["stream_read_GBps"]

    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(wl)

    print(json.dumps(result))


if __name__ == "__main__":
    main()
