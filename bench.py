#!/usr/bin/env python3
"""Benchmark of the LoMA attention hot path on one MI355X.

One step = one pass of the whole hot path through a 32-layer, Llama-2-7B-shaped stack
(every layer has its own tensors, so nothing is served from a cache warmed by the
previous layer):
    mask leg      32 x loma_mask_attn_fwd   B2 H32 d128 t16 c4, 28 chunks (S = 4032), bf16
    compress leg  32 x loma_compress_step   B8 H32 d128 t16 c4, 64 prior chunks
    decode leg    64 tokens x 32 layers x loma_decode_attn over 1040 memory KVs + the
                  growing reading zone (one full reading zone: after 64 tokens the state is
                  back at a compression boundary, so the step repeats exactly)
`value` is the useful TFLOP/s of the mask leg (unmasked pairs only); the decode leg's
GB/s is reported next to it.  Each leg is bracketed by HIP events on the launch stream.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--layers 32] [--no-extra] [--no-high-ratio] [--no-cpu]
    python bench.py --copy-calibration     three plain 1 GiB device copies and nothing else: the known
                                           traffic the FETCH_SIZE / WRITE_SIZE counters are scaled by
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E
MFMA_BF16_PEAK_TF = 2500.0  # MI355X dense bf16
# HBM bytes per launch from rocprofv3 counter runs over this script (2.000 x FETCH_SIZE + 1.000 x WRITE_SIZE KiB,
# the factors being what the same counters read for 1 GiB device copies: --copy-calibration).  Counters cannot be
# read from inside a timed run, so these are the figures of the committed profile, not of this process.
TRAFFIC_BYTES = {"decode": (2.0 * 68783.5 + 192) * 1024, "mask": (2.0 * 114529 + 64512) * 1024,
                 "long_context_mask": (2.0 * 508406 + 261120) * 1024,
                 # gradients: dQ pass + dK/dV pass (+ the sum of shared blocks at the Llama shape)
                 "mask_bwd": (2.0 * (228791.1 + 119580.9 + 28695.9) + 123949.5 + 114688 + 14336) * 1024,
                 "long_context_mask_bwd": (2.0 * (948240.5 + 1288200.7) + 515043.2 + 276480) * 1024}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--no-extra", action="store_true", help="skip the long-context and high-ratio configurations")
    ap.add_argument("--no-high-ratio", action="store_true", help="skip the high-ratio decode configuration (about 35 GB of state)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--copy-calibration", action="store_true", help="run three 1 GiB device copies and exit")
    return ap.parse_args()


def randn_bf16(shape, gen, scale=1.0):
    import torch
    out = torch.empty(shape, dtype=torch.bfloat16, device="cuda")
    flat = out.view(-1)
    step = 1 << 26
    for i in range(0, flat.numel(), step):
        n = min(step, flat.numel() - i)
        flat[i:i + n] = (torch.randn(n, generator=gen, device="cuda", dtype=torch.float32) * scale).to(torch.bfloat16)
    return out


class Events:
    def __init__(self):
        import torch
        self.torch = torch
        self.pairs = {}

    def mark(self):
        e = self.torch.cuda.Event(enable_timing=True)
        e.record()
        return e

    def add(self, name, a, b):
        self.pairs.setdefault(name, []).append((a, b))

    def total_ms(self, name):
        return sum(a.elapsed_time(b) for a, b in self.pairs.get(name, []))


def time_calls(fn, iters, warmup=2):
    """Average milliseconds per call of fn(i) over `iters` back-to-back calls (HIP events)."""
    import torch
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    a = torch.cuda.Event(enable_timing=True)
    b = torch.cuda.Event(enable_timing=True)
    a.record()
    for i in range(iters):
        fn(i)
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / iters


def cpu_baseline(wl, layers):
    """The fp64 oracle, as it stands, on the host cores: the mask leg of one step (the whole
    mask pass of configs[1], once per layer; the layers reuse one set of host inputs)."""
    from oracle import c_oracle
    cfg = wl.CONFIGS[1]
    q, k, v = wl.mask_inputs(cfg)
    c_oracle.build()
    threads = c_oracle.num_threads()
    t0 = time.perf_counter()
    for _ in range(layers):
        c_oracle.mask_attn(q, k, v, cfg.t, cfg.c, cfg.n_chunks, cfg.scale)
    dt = time.perf_counter() - t0
    flops = wl.mask_pass_useful_flops(cfg) * layers
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s (useful, fp64)", "cores": threads, "kind": "oracle",
            "seconds": dt, "sample": f"mask leg of one step: whole mask pass of {cfg.name} (all {cfg.B * cfg.H} (b,h), "
                                     f"all {cfg.S} rows) x {layers} layers"}


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
    gen = torch.Generator(device="cuda")
    gen.manual_seed(wl.SEED_BASE)
    L = args.layers
    mc, gc = wl.CONFIGS[1], wl.CONFIGS[2]

    # ---- per-layer tensors ---------------------------------------------------------------------
    mshape = (mc.B, mc.H, mc.S, mc.d)
    mask_layers = [tuple(randn_bf16(mshape, gen, mc.value_scale) for _ in range(3)) + (torch.empty(mshape, dtype=torch.bfloat16, device="cuda"),)
                   for _ in range(L)]
    cap = (gc.prior_chunks + 1) * gc.t
    gen_layers = []
    for _ in range(L):
        gen_layers.append({
            "k_mem": randn_bf16((gc.B, gc.H, cap, gc.d), gen), "v_mem": randn_bf16((gc.B, gc.H, cap, gc.d), gen),
            "k_read": randn_bf16((gc.B, gc.H, gc.R, gc.d), gen), "v_read": randn_bf16((gc.B, gc.H, gc.R, gc.d), gen),
            "q_m": randn_bf16((gc.B, gc.H, gc.t, gc.d), gen), "k_m": randn_bf16((gc.B, gc.H, gc.t, gc.d), gen),
            "v_m": randn_bf16((gc.B, gc.H, gc.t, gc.d), gen),
            "q": randn_bf16((gc.B, gc.H, 1, gc.d), gen), "k_new": randn_bf16((gc.B, gc.H, 1, gc.d), gen),
            "v_new": randn_bf16((gc.B, gc.H, 1, gc.d), gen),
            "out_m": torch.empty((gc.B, gc.H, gc.t, gc.d), dtype=torch.bfloat16, device="cuda"),
            "out": torch.empty((gc.B, gc.H, 1, gc.d), dtype=torch.bfloat16, device="cuda"),
        })
    ws = torch.empty(max(loma.loma_decode_workspace_bytes(gc.B, gc.H, gc.d, gc.t, gc.c, gc.prior_chunks + 1), 16),
                     dtype=torch.uint8, device="cuda")
    ev = Events()

    def step(record):
        e0 = ev.mark()
        for (q, k, v, o) in mask_layers:
            loma.loma_mask_attn_fwd(q, k, v, mc.t, mc.c, mc.n_chunks, mc.scale, out=o)
        e1 = ev.mark()
        for g in gen_layers:
            loma.loma_compress_step(g["q_m"], g["k_m"], g["v_m"], g["k_read"], g["v_read"], g["k_mem"], g["v_mem"],
                                    gc.t, gc.c, gc.prior_chunks, gc.scale, out=g["out_m"])
        e2 = ev.mark()
        for tok in range(gc.R):
            for g in gen_layers:
                loma.loma_decode_attn(g["q"], g["k_new"], g["v_new"], g["k_mem"], g["v_mem"], g["k_read"], g["v_read"],
                                      gc.t, gc.c, gc.prior_chunks + 1, tok, gc.scale, out=g["out"], workspace=ws)
        e3 = ev.mark()
        if record:
            ev.add("mask", e0, e1)
            ev.add("compress", e1, e2)
            ev.add("decode", e2, e3)

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    K = args.steps

    # ---- mask leg --------------------------------------------------------------------------------
    mask_ms = ev.total_ms("mask") / (K * L)                    # per launch
    mask_flops = wl.mask_pass_useful_flops(mc)
    mask_bytes = wl.mask_pass_bytes(mc)
    mask_tf = mask_flops / (mask_ms * 1e-3) / 1e12
    mask_gbs = mask_bytes / (mask_ms * 1e-3) / 1e9
    # ---- compress leg ----------------------------------------------------------------------------
    comp_ms = ev.total_ms("compress") / (K * L)
    comp_bytes = wl.compress_bytes(gc.B, gc.H, gc.d, gc.t, gc.c, gc.dtype)
    comp_flops = wl.compress_useful_flops(gc.B, gc.H, gc.d, gc.t, gc.c)
    # ---- decode leg ------------------------------------------------------------------------------
    dec_calls = K * L * gc.R
    dec_ms = ev.total_ms("decode") / dec_calls
    n_mem_keys = (gc.prior_chunks + 1) * gc.t
    dec_bytes = sum(wl.decode_bytes(gc.B, gc.H, gc.d, n_mem_keys + f + 1, gc.dtype) for f in range(gc.R)) / gc.R
    dec_gbs = dec_bytes / (dec_ms * 1e-3) / 1e9

    result = {
        "metric": "LoMA-mask attn useful TFLOP/s + decode GB/s (frac of MI355X roofline)",
        "value": mask_tf, "unit": "TFLOP/s (useful, mask pass)",
        "n_gpus": 1, "steps": K, "warmup": args.warmup, "ms_per_step": wall_ms / K,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{mc.name} (B{mc.B} H{mc.H} d{mc.d} t{mc.t} c{mc.c} n{mc.n_chunks}, S={mc.S}) x {L} layers"
                               f" + {gc.name} slice (1 compress + {gc.R} decode tokens) x {L} layers",
                   "layers": L},
        "decode": {"value": dec_gbs, "unit": "GB/s (algorithmic)", "frac_of_hbm_peak": dec_gbs / HBM_PEAK_GBS,
                   "us_per_call": dec_ms * 1e3, "bytes_per_call": dec_bytes, "calls": dec_calls,
                   "keys": f"{n_mem_keys}+1..{n_mem_keys}+{gc.R}"},
        "mask": {"useful_tflops": mask_tf, "frac_of_mfma_peak": mask_tf / MFMA_BF16_PEAK_TF, "us_per_call": mask_ms * 1e3,
                 "algorithmic_GBps": mask_gbs, "frac_of_hbm_peak": mask_gbs / HBM_PEAK_GBS, "useful_flops": mask_flops,
                 "bytes": mask_bytes},
        "compress": {"us_per_call": comp_ms * 1e3, "algorithmic_GBps": comp_bytes / (comp_ms * 1e-3) / 1e9,
                     "useful_tflops": comp_flops / (comp_ms * 1e-3) / 1e12},
        # dominant kernel of the step by time: the split-K decode kernel (HBM-bound)
        "roofline": {"kernel": "decode_split_kernel<128, 16>", "bound": "hbm", "achieved": dec_gbs,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": dec_gbs / HBM_PEAK_GBS,
                     "traffic": TRAFFIC_BYTES["decode"]},
        # the mask-pass kernel at this shape is HBM-bound too (63 flop/byte)
        "roofline_mask": {"kernel": "mask_attn_kernel<128, 2, 32, 1>", "bound": "hbm", "achieved": mask_gbs,
                          "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": mask_gbs / HBM_PEAK_GBS,
                          "traffic": TRAFFIC_BYTES["mask"]},
    }

    # ---- prompt form on the generation shape: a whole reading zone of new tokens per call --------------
    if not args.no_extra:
        pre = [tuple(randn_bf16((gc.B, gc.H, gc.R, gc.d), gen) for _ in range(3)) + (torch.empty((gc.B, gc.H, gc.R, gc.d), dtype=torch.bfloat16, device="cuda"),)
               for _ in range(min(L, 8))]
        pms = time_calls(lambda i: loma.loma_prefill_attn(pre[i % len(pre)][0], pre[i % len(pre)][1], pre[i % len(pre)][2],
                                                          gen_layers[i % L]["k_mem"], gen_layers[i % L]["v_mem"],
                                                          gen_layers[i % L]["k_read"], gen_layers[i % L]["v_read"],
                                                          gc.t, gc.c, gc.prior_chunks + 1, 0, gc.scale, out=pre[i % len(pre)][3]), 4 * L)
        nbh = gc.B * gc.H
        pbytes = nbh * (2 * n_mem_keys * gc.d + 6 * gc.R * gc.d) * 2   # cache read once; q, k, v in, out and the appended K/V out
        pflops = 4.0 * gc.d * nbh * (gc.R * n_mem_keys + gc.R * (gc.R + 1) / 2)
        result["prefill"] = {"workload": f"{gc.name}: {gc.R} new tokens per sequence over {n_mem_keys} memory KVs",
                             "us_per_call": pms * 1e3, "algorithmic_GBps": pbytes / (pms * 1e-3) / 1e9,
                             "frac_of_hbm_peak": pbytes / (pms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                             "useful_tflops": pflops / (pms * 1e-3) / 1e12,
                             "vs_token_by_token": gc.R * dec_ms / pms}   # time of the same tokens through loma_decode_attn / this

    # ---- gradients of the mask pass (forward output and lse kept, as a training step would) --------------
    def time_backward(cfg, q, k, v, o):
        lse = torch.empty((cfg.B, cfg.H, cfg.S), dtype=torch.float32, device="cuda")
        loma.loma_mask_attn_fwd(q, k, v, cfg.t, cfg.c, cfg.n_chunks, cfg.scale, out=o, lse=lse)
        g = randn_bf16(tuple(q.shape), gen)
        grads = [torch.empty_like(q) for _ in range(3)]
        wsb = torch.empty(loma.loma_mask_attn_bwd_workspace_bytes(cfg.B, cfg.H, cfg.d, cfg.t, cfg.c, cfg.n_chunks),
                          dtype=torch.uint8, device="cuda")
        ms = time_calls(lambda i: loma.loma_mask_attn_bwd(q, k, v, o, lse, g, cfg.t, cfg.c, cfg.n_chunks, cfg.scale,
                                                          dq=grads[0], dk=grads[1], dv=grads[2], workspace=wsb), 10)
        fl = 2.5 * wl.mask_pass_useful_flops(cfg)      # five products per visible pair against the forward's two
        by = 2.0 * wl.mask_pass_bytes(cfg)             # q, k, v, out, dout in; dq, dk, dv out
        return {"workload": cfg.name, "us_per_call": ms * 1e3, "useful_tflops": fl / (ms * 1e-3) / 1e12,
                "frac_of_mfma_peak": fl / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TF, "useful_flops": fl,
                "algorithmic_GBps": by / (ms * 1e-3) / 1e9, "frac_of_hbm_peak": by / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}

    if not args.no_extra:
        result["mask_bwd"] = time_backward(mc, *mask_layers[0])
        b2 = result["mask_bwd"]
        result["roofline_mask_bwd"] = {"kernel": "bwd_dkv_kernel<128, 2> (+ bwd_dq_kernel<128, 2>, bwd_reduce_kernel<128>)", "bound": "hbm",
                                       "achieved": b2["algorithmic_GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                       "frac": b2["frac_of_hbm_peak"], "traffic": TRAFFIC_BYTES["mask_bwd"]}

    # ---- the other single-GPU configurations, timed on their own ---------------------------------
    if not args.no_extra:
        del mask_layers
        torch.cuda.empty_cache()
        c4 = wl.CONFIGS[3]
        shp = (c4.B, c4.H, c4.S, c4.d)
        sets = [tuple(randn_bf16(shp, gen, c4.value_scale) for _ in range(3)) + (torch.empty(shp, dtype=torch.bfloat16, device="cuda"),)
                for _ in range(2)]
        ms = time_calls(lambda i: loma.loma_mask_attn_fwd(*sets[i % 2][:3], c4.t, c4.c, c4.n_chunks, c4.scale, out=sets[i % 2][3]), 10)
        fl = wl.mask_pass_useful_flops(c4)
        result["long_context_mask"] = {"workload": c4.name, "us_per_call": ms * 1e3, "useful_tflops": fl / (ms * 1e-3) / 1e12,
                                       "frac_of_mfma_peak": fl / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TF,
                                       "algorithmic_GBps": wl.mask_pass_bytes(c4) / (ms * 1e-3) / 1e9}
        result["roofline_long_context_mask"] = {"kernel": "mask_attn_kernel<128, 4, 64, 1>", "bound": "mfma",
                                                "achieved": fl / (ms * 1e-3) / 1e12, "peak": MFMA_BF16_PEAK_TF,
                                                "unit": "TFLOP/s", "frac": fl / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TF,
                                                "traffic": TRAFFIC_BYTES["long_context_mask"]}
        result["long_context_mask_bwd"] = time_backward(c4, *sets[0])
        bw = result["long_context_mask_bwd"]
        # its dominant kernel: the dK/dV pass (four of the seven matrix products the two launches issue)
        result["roofline_long_context_mask_bwd"] = {"kernel": "bwd_dkv_kernel<128, 4> (+ bwd_dq_kernel<128, 4>)",
                                                    "bound": "mfma", "achieved": bw["useful_tflops"], "peak": MFMA_BF16_PEAK_TF,
                                                    "unit": "TFLOP/s", "frac": bw["frac_of_mfma_peak"],
                                                    "traffic": TRAFFIC_BYTES["long_context_mask_bwd"]}
        del sets
    if not args.no_extra and not args.no_high_ratio:
        del gen_layers
        torch.cuda.empty_cache()
        c5 = wl.CONFIGS[4]
        st = wl.gen_initial_state_device(c5)
        qm, km, vm = (randn_bf16((c5.B, c5.H, c5.t, c5.d), gen) for _ in range(3))
        om = torch.empty_like(qm)
        q5 = randn_bf16((c5.B, c5.H, 1, c5.d), gen, c5.q_scale)
        kn, vn = randn_bf16((c5.B, c5.H, 1, c5.d), gen), randn_bf16((c5.B, c5.H, 1, c5.d), gen)
        o5 = torch.empty_like(q5)
        ws5 = torch.empty(max(loma.loma_decode_workspace_bytes(c5.B, c5.H, c5.d, c5.t, c5.c, c5.prior_chunks + 1), 16),
                          dtype=torch.uint8, device="cuda")
        cms = time_calls(lambda i: loma.loma_compress_step(qm, km, vm, st["k_read"], st["v_read"], st["k_mem"], st["v_mem"],
                                                           c5.t, c5.c, c5.prior_chunks, c5.scale, out=om), 5)
        nm = c5.prior_chunks + 1
        dms = time_calls(lambda i: loma.loma_decode_attn(q5, kn, vn, st["k_mem"], st["v_mem"], st["k_read"], st["v_read"],
                                                         c5.t, c5.c, nm, i % c5.steps, c5.scale, out=o5, workspace=ws5), c5.steps)
        b5 = sum(wl.decode_bytes(c5.B, c5.H, c5.d, nm * c5.t + f + 1, c5.dtype) for f in range(c5.steps)) / c5.steps
        result["high_ratio_decode"] = {"workload": c5.name, "ms_per_step": dms, "algorithmic_GBps": b5 / (dms * 1e-3) / 1e9,
                                       "frac_of_hbm_peak": b5 / (dms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                       "compress_us": cms * 1e3,
                                       "compress_GBps": wl.compress_bytes(c5.B, c5.H, c5.d, c5.t, c5.c, c5.dtype) / (cms * 1e-3) / 1e9}

    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(wl, L)

    print(json.dumps(result))


if __name__ == "__main__":
    main()
