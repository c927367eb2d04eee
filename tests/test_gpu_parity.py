"""GPU parity: the HIP path (through the C ABI) against the CPU fp64 oracle, element by element.

Small shapes that still span several tiles, ragged tails and every kernel variant; the
full-size configurations are in test_gpu_full_configs.py.
"""
import math

import numpy as np
import pytest
import torch

from gpu_util import check, check_grad, host_bits, to_dev, to_host_f64
from paper_2401_09486_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def loma():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2401_09486_amd import loma as m
    return m


def run_mask(loma, c_oracle, cfg, want_lse=False):
    print(f"[case] mask pass {cfg}", flush=True)
    q, k, v = wl.mask_inputs(cfg)
    dq, dk, dv = to_dev(q), to_dev(k), to_dev(v)
    lse = torch.empty((cfg.B, cfg.H, cfg.S), dtype=torch.float32, device="cuda") if want_lse else None
    out = loma.loma_mask_attn_fwd(dq, dk, dv, cfg.t, cfg.c, cfg.n_chunks, cfg.scale, lse=lse)
    torch.cuda.synchronize()
    ref, ref_lse = c_oracle.mask_attn(q, k, v, cfg.t, cfg.c, cfg.n_chunks, cfg.scale, return_lse=True)
    mx, mean = check(to_host_f64(out), ref, cfg.dtype, cfg.name)
    if want_lse:
        tol = 1e-5 if cfg.dtype == "f32" else 2e-3
        assert np.abs(lse.cpu().numpy().astype(np.float64) - ref_lse).max() <= tol
    return out, ref, mx, mean


def small(name, B, H, d, t, c, n, dtype="bf16", scale=0.5, index=1):
    return wl.MaskConfig(index, name, B, H, d, t, c, n, dtype, scale)


def test_config1_tiny_fp32(loma, c_oracle):
    run_mask(loma, c_oracle, wl.CONFIGS[0], want_lse=True)


@pytest.mark.parametrize("cfg", [
    small("bf16_t16c4_bm64", 1, 2, 128, 16, 4, 3),          # 2-wave kernel, BN 32
    small("bf16_t32c8_bm128", 1, 2, 128, 32, 8, 3),         # 4-wave kernel, BN 64, two row blocks per zone
    small("bf16_t4c4_bm32", 2, 1, 128, 4, 4, 4),            # 1-wave kernel, R = 16 < 32 rows
    small("bf16_t5c7_ragged", 1, 3, 128, 5, 7, 3),          # R = 35, t = 5: nothing aligned
    small("bf16_t24c6_ragged128", 1, 1, 128, 24, 6, 3),     # R = 144: 128 + 16 ragged row block
    small("bf16_t40c1", 1, 2, 128, 40, 1, 2),               # memory zone needs 2 waves
    small("bf16_t1c1", 1, 1, 128, 1, 1, 5),                 # degenerate: every zone one token
    small("bf16_d64_t16c4", 1, 2, 64, 16, 4, 3),
    small("bf16_d64_t32c8", 1, 1, 64, 32, 8, 2),
    small("bf16_nbh8_xcd", 1, 8, 128, 16, 2, 6),            # B*H multiple of 8
], ids=lambda c: c.name)
def test_mask_pass_mfma_small(loma, c_oracle, cfg):
    run_mask(loma, c_oracle, cfg, want_lse=True)


@pytest.mark.parametrize("shape", [(32, 8, 10), (16, 4, 12), (8, 4, 9)], ids=["t32c8_4wave", "t16c4_2wave", "t8c4_1wave"])
@pytest.mark.parametrize("scale", [0.25, 1.0, 4.0])
def test_mask_pass_moving_maximum(loma, c_oracle, shape, scale):
    """A sharp softmax over keys whose norm keeps growing along the sequence: between some tiles a
    row's running maximum moves by far more than the threshold up to which the kernel keeps its
    softmax reference, between others by less, so both the kept-reference and the rescale path run
    (with the default 1/sqrt(d) scale and unit-variance data the maximum settles in the first tile)."""
    t, c, n = shape
    cfg = small(f"moving_max_t{t}c{c}", 1, 2, 128, t, c, n)
    print(f"[case] moving maximum {cfg} scale={scale}", flush=True)
    q, k, v = wl.mask_inputs(cfg)
    ramp = (0.25 + 1.75 * np.arange(cfg.S, dtype=np.float32) / cfg.S)[None, None, :, None]
    k = wl.f32_to_bf16_bits(wl.bf16_bits_to_f32(k) * ramp)
    lse = torch.empty((cfg.B, cfg.H, cfg.S), dtype=torch.float32, device="cuda")
    out = loma.loma_mask_attn_fwd(to_dev(q), to_dev(k), to_dev(v), t, c, n, scale, lse=lse)
    torch.cuda.synchronize()
    ref, ref_lse = c_oracle.mask_attn(q, k, v, t, c, n, scale, return_lse=True)
    check(to_host_f64(out), ref, cfg.dtype, cfg.name)
    lse_err = np.abs(lse.cpu().numpy().astype(np.float64) - ref_lse).max()
    print(f"[result] moving maximum scale {scale}: lse max abs err {lse_err:.3e} (|lse| up to {np.abs(ref_lse).max():.1f})", flush=True)
    assert lse_err <= 1e-4


@pytest.mark.parametrize("cfg", [
    small("f32_d128_t16c2", 1, 2, 128, 16, 2, 3, dtype="f32", scale=1.0),
    small("f32_d40_t3c3", 2, 1, 40, 3, 3, 4, dtype="f32", scale=1.0),
    small("bf16_d96_generic", 1, 2, 96, 8, 2, 3),
    small("bf16_d256_generic", 1, 1, 256, 4, 3, 2),
], ids=lambda c: c.name)
def test_mask_pass_generic_small(loma, c_oracle, cfg):
    run_mask(loma, c_oracle, cfg, want_lse=True)


def test_mask_pass_is_deterministic(loma):
    cfg = small("det", 1, 4, 128, 32, 4, 4)
    q, k, v = (to_dev(x) for x in wl.mask_inputs(cfg))
    a = loma.loma_mask_attn_fwd(q, k, v, cfg.t, cfg.c, cfg.n_chunks, cfg.scale)
    b = loma.loma_mask_attn_fwd(q, k, v, cfg.t, cfg.c, cfg.n_chunks, cfg.scale)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


@pytest.mark.parametrize("cfg", [small("poison_mfma", 1, 1, 128, 16, 4, 3), small("poison_mfma_4wave", 1, 1, 128, 32, 8, 3),
                                 small("poison_f32", 1, 1, 64, 4, 4, 3, dtype="f32")],
                         ids=lambda c: c.name)
def test_masked_keys_never_reach_a_row(loma, cfg):
    """Eq. 8-9: overwrite every key a row may not see and its output must stay bit-identical.
    K is overwritten with NaN everywhere hidden.  V is overwritten with Inf everywhere hidden, except, for a
    reading row of the MFMA path, the later rows of its own workgroup block: those keys sit in the causal
    diagonal tiles, which the block multiplies whole for its later rows, and meet a weight of exactly 0 for
    this row -- exact only for finite V (0 * Inf is NaN in any kernel that multiplies whole tiles), so they get a
    huge finite value instead.  Every other hidden key, also those of other blocks of the same reading zone, of
    other chunks and of the repetition zones, is never loaded for this row and takes Inf."""
    from oracle import loma_oracle as lo
    q, k, v = wl.mask_inputs(cfg)
    dq, dk, dv = to_dev(q), to_dev(k), to_dev(v)
    base = loma.loma_mask_attn_fwd(dq, dk, dv, cfg.t, cfg.c, cfg.n_chunks, cfg.scale)
    torch.cuda.synchronize()
    mask = lo.mask_from_blocks(cfg.t, cfg.c, cfg.n_chunks)
    R, s = cfg.R, cfg.s
    bm = 128 if R >= 128 else (64 if R >= 64 else 32)        # rows per workgroup block of the MFMA kernels
    y = cfg.n_chunks - 1
    rows = [(y * s + R + cfg.t + 3, "rep"), (s + R + cfg.t, "rep"), (y * s + R + 1, "mem"),
            (y * s + 5, "read"), (2, "read"), (s + R - 1, "read"), (s + bm - 1 if R > bm else s + 7, "read")]
    for p, zone in rows:
        hidden = np.nonzero(mask[p] == 0)[0]
        k2, v2 = dk.clone(), dv.clone()
        k2[:, :, torch.from_numpy(hidden).cuda()] = float("nan")
        v2[:, :, torch.from_numpy(hidden).cuda()] = float("inf")
        if zone == "read" and cfg.dtype == "bf16":
            o = p % s
            blk_end = min((o // bm + 1) * bm, R)                # rows o+1 .. blk_end-1 share the block's diagonal tiles
            same_block = np.arange(p + 1, p - o + blk_end)
            assert np.all(mask[p][same_block] == 0)
            if same_block.size:
                v2[:, :, torch.from_numpy(same_block).cuda()] = 1e30
        out = loma.loma_mask_attn_fwd(dq, k2, v2, cfg.t, cfg.c, cfg.n_chunks, cfg.scale)
        torch.cuda.synchronize()
        a = out[:, :, p].contiguous().view(torch.int16 if cfg.dtype == "bf16" else torch.int32)
        b = base[:, :, p].contiguous().view(torch.int16 if cfg.dtype == "bf16" else torch.int32)
        assert torch.equal(a, b), f"row {p} ({zone}) changed when masked K/V were overwritten"


# ---- generation form ---------------------------------------------------------------------------
def run_generation(loma, c_oracle, cfg, check_every=1):
    """Drive compress/decode exactly as the appendix's loop does, on the GPU and in the oracle."""
    print(f"[case] generation {cfg}", flush=True)
    st = wl.gen_initial_state(cfg)
    dev = {k: to_dev(v) for k, v in st.items()}
    orc = c_oracle.GenerationCache(st["k_mem"].copy(), st["v_mem"].copy(), cfg.prior_chunks,
                                   st["k_read"].copy(), st["v_read"].copy(), cfg.R, cfg.t, cfg.c, cfg.scale)
    nws = loma.loma_decode_workspace_bytes(cfg.B, cfg.H, cfg.d, cfg.t, cfg.c, cfg.prior_chunks + cfg.n_compress,
                                           torch.bfloat16 if cfg.dtype == "bf16" else torch.float32)
    ws = torch.empty(max(nws, 16), dtype=torch.uint8, device="cuda")
    n_mem, fill, events = cfg.prior_chunks, cfg.R, 0
    worst = 0.0
    for step in range(cfg.steps):
        if fill == cfg.R:
            qm, km, vm = wl.gen_compress_inputs(cfg, events)
            out = loma.loma_compress_step(to_dev(qm), to_dev(km), to_dev(vm), dev["k_read"], dev["v_read"],
                                          dev["k_mem"], dev["v_mem"], cfg.t, cfg.c, n_mem, cfg.scale)
            ref = orc.compress(qm, km, vm).reshape(cfg.B, cfg.H, cfg.t, cfg.d)
            mx, _ = check(to_host_f64(out), ref, cfg.dtype, f"compress event {events}")
            worst = max(worst, mx)
            n_mem, fill, events = n_mem + 1, 0, events + 1
            # the splice: the cache rows just written are the <m> tokens' K/V, bit for bit
            lo_, hi_ = (n_mem - 1) * cfg.t, n_mem * cfg.t
            assert np.array_equal(host_bits(dev["k_mem"][:, :, lo_:hi_]), km)
            assert np.array_equal(host_bits(dev["v_mem"][:, :, lo_:hi_]), vm)
        q, kn, vn = wl.gen_step_inputs(cfg, step)
        out = loma.loma_decode_attn(to_dev(q), to_dev(kn), to_dev(vn), dev["k_mem"], dev["v_mem"],
                                    dev["k_read"], dev["v_read"], cfg.t, cfg.c, n_mem, fill, cfg.scale, workspace=ws)
        ref = orc.decode(q, kn, vn).reshape(cfg.B, cfg.H, 1, cfg.d)
        fill += 1
        if step % check_every == 0 or step == cfg.steps - 1:
            mx, _ = check(to_host_f64(out), ref, cfg.dtype, f"decode step {step}")
            worst = max(worst, mx)
    # the appended tokens sit in the reading zone, bit for bit
    assert np.array_equal(host_bits(dev["k_read"][:, :, :fill]), orc.k_read[:, :, :fill])
    assert np.array_equal(host_bits(dev["v_read"][:, :, :fill]), orc.v_read[:, :, :fill])
    assert np.array_equal(host_bits(dev["k_mem"][:, :, :n_mem * cfg.t]), orc.k_mem[:, :, :n_mem * cfg.t])
    return worst


def gen_small(name, B, H, d, t, c, prior, steps, dtype="bf16", index=2):
    return wl.GenConfig(index, name, B, H, d, t, c, prior, steps, dtype, 1.0, 1.0)


@pytest.mark.parametrize("cfg", [
    gen_small("gen_bf16_t16c4", 2, 4, 128, 16, 4, 8, 150),          # split-K, 3 compressions
    gen_small("gen_bf16_noprior", 1, 2, 128, 16, 2, 0, 70),         # empty memory cache at the start
    gen_small("gen_bf16_d64", 1, 3, 64, 8, 4, 5, 70),
    gen_small("gen_bf16_t4c3", 1, 2, 128, 4, 3, 40, 30),            # odd reading-zone length 12
    gen_small("gen_bf16_t40", 1, 2, 128, 40, 2, 3, 90),             # compression with 2 waves
    gen_small("gen_bf16_t100", 1, 1, 128, 100, 1, 2, 110),          # compression with 4 waves
    gen_small("gen_bf16_longcache", 1, 2, 128, 16, 4, 300, 10),     # 4800 memory rows: several iterations per split
    gen_small("gen_f32_generic", 1, 2, 64, 4, 4, 6, 40, dtype="f32"),
    gen_small("gen_bf16_d96_generic", 1, 2, 96, 4, 4, 6, 20),
], ids=lambda c: c.name)
def test_generation_small(loma, c_oracle, cfg):
    run_generation(loma, c_oracle, cfg)


def random_shapes(seed, count):
    """Seeded draw of small geometries that mixes every kernel variant: head_dim 64 / 128 (MFMA kernels),
    reading zones below 32, between 32 and 64, 64..127 and 128 and more rows, memory zones from 1 to 70 rows
    (the last needs two tiles for the repetition rows' keys), ragged everything."""
    rng = np.random.default_rng(seed)
    out = []
    for i in range(count):
        d = int(rng.choice([64, 128]))
        t = int(rng.choice([1, 2, 3, 4, 7, 8, 12, 16, 20, 32, 33, 48, 70]))
        c = int(rng.integers(1, 9))
        while t * c > 300:
            c = max(1, c // 2)
        n = int(rng.integers(1, 6))
        B, H = int(rng.integers(1, 3)), int(rng.choice([1, 2, 3, 4, 8]))
        out.append((B, H, d, t, c, n))
    # memory zones wider than one key tile of the kernel that takes them
    return out + [(1, 2, 128, 48, 2, 3), (1, 1, 128, 70, 2, 2), (1, 2, 64, 33, 3, 2), (1, 1, 128, 70, 4, 2)]


@pytest.mark.parametrize("shape", random_shapes(9486, 28), ids=lambda s: "B%d_H%d_d%d_t%d_c%d_n%d" % s)
def test_mask_pass_random_shapes(loma, c_oracle, shape):
    B, H, d, t, c, n = shape
    run_mask(loma, c_oracle, small("rand_%d_%d_%d" % (t, c, n), B, H, d, t, c, n), want_lse=True)


@pytest.mark.parametrize("shape", random_shapes(9487, 16), ids=lambda s: "B%d_H%d_d%d_t%d_c%d_n%d" % s)
def test_generation_and_prefill_random_shapes(loma, c_oracle, shape):
    """Token-by-token generation and the same reading zones fed in two or three random pieces."""
    B, H, d, t, c, n = shape
    R = t * c
    prior = n * 3
    run_generation(loma, c_oracle, gen_small("randgen", B, H, d, t, c, prior, min(2 * R + 1, 70)))
    rng = np.random.default_rng(t * 1000 + c)
    cuts = sorted(set(int(x) for x in rng.integers(1, R, size=2))) if R > 1 else []
    pieces = tuple(b - a for a, b in zip([0] + cuts, cuts + [R]))
    run_prefill(loma, c_oracle, gen_small("randpre", B, H, d, t, c, prior, 2 * R), pieces)


# ---- several tokens at once (Appendix A, inference_input with more than one token) ---------------------
def run_prefill(loma, c_oracle, cfg, pieces):
    """Every reading zone is fed in pieces (token counts in `pieces`, summing to t*c) through
    loma_prefill_attn, with compression steps in between; the oracle takes the same tokens one by one."""
    print(f"[case] prefill {cfg} pieces={pieces}", flush=True)
    assert sum(pieces) == cfg.R
    st = wl.gen_initial_state(cfg)
    dev = {k: to_dev(v) for k, v in st.items()}
    orc = c_oracle.GenerationCache(st["k_mem"].copy(), st["v_mem"].copy(), cfg.prior_chunks,
                                   st["k_read"].copy(), st["v_read"].copy(), cfg.R, cfg.t, cfg.c, cfg.scale)
    n_mem, step = cfg.prior_chunks, 0
    for event in range(cfg.n_compress):
        qm, km, vm = wl.gen_compress_inputs(cfg, event)
        loma.loma_compress_step(to_dev(qm), to_dev(km), to_dev(vm), dev["k_read"], dev["v_read"],
                                dev["k_mem"], dev["v_mem"], cfg.t, cfg.c, n_mem, cfg.scale)
        orc.compress(qm, km, vm)
        n_mem, fill = n_mem + 1, 0
        for l in pieces:
            toks = [wl.gen_step_inputs(cfg, step + i) for i in range(l)]
            q, kn, vn = (np.concatenate([tk[j] for tk in toks], axis=2) for j in range(3))
            lse = torch.empty((cfg.B, cfg.H, l), dtype=torch.float32, device="cuda")
            out = loma.loma_prefill_attn(to_dev(q), to_dev(kn), to_dev(vn), dev["k_mem"], dev["v_mem"],
                                         dev["k_read"], dev["v_read"], cfg.t, cfg.c, n_mem, fill, cfg.scale, lse=lse)
            torch.cuda.synchronize()
            ref = orc.prefill(q, kn, vn).reshape(cfg.B, cfg.H, l, cfg.d)
            check(to_host_f64(out), ref, cfg.dtype, f"prefill event {event} fill {fill} l {l}")
            lse_err = np.abs(lse.cpu().numpy().astype(np.float64) - orc.last_lse.reshape(cfg.B, cfg.H, l)).max()
            assert lse_err <= (1e-5 if cfg.dtype == "f32" else 2e-3), f"prefill lse off by {lse_err:.3e}"
            fill += l
            step += l
            # the new tokens sit in the reading zone, bit for bit, and nothing past them was touched
            assert np.array_equal(host_bits(dev["k_read"][:, :, :fill]), orc.k_read[:, :, :fill])
            assert np.array_equal(host_bits(dev["v_read"][:, :, :fill]), orc.v_read[:, :, :fill])


@pytest.mark.parametrize("cfg,pieces", [
    (gen_small("pre_bf16_t16c4", 2, 4, 128, 16, 4, 8, 128), (1, 31, 32)),         # 1-wave kernel (n_new 1, 31, 32)
    (gen_small("pre_bf16_t16c4_whole", 1, 8, 128, 16, 4, 20, 64), (64,)),         # 2-wave kernel, whole reading zone
    (gen_small("pre_bf16_t32c8", 1, 2, 128, 32, 8, 5, 512), (100, 156)),          # 4-wave kernel, 1 and 2 row blocks
    (gen_small("pre_bf16_t32c8_whole", 1, 2, 128, 32, 8, 12, 256), (256,)),
    (gen_small("pre_bf16_t4c3", 1, 2, 128, 4, 3, 40, 24), (5, 7)),                # nothing aligned
    (gen_small("pre_bf16_d64", 1, 3, 64, 8, 4, 5, 32), (9, 23)),
    (gen_small("pre_f32_generic", 1, 2, 64, 4, 4, 6, 32), (3, 13)),
    (gen_small("pre_bf16_d96_generic", 1, 2, 96, 4, 4, 6, 16), (16,)),
], ids=lambda x: x.name if hasattr(x, "name") else None)
def test_prefill_small(loma, c_oracle, cfg, pieces):
    run_prefill(loma, c_oracle, cfg, pieces)


def test_prefill_into_an_empty_cache(loma):
    """No memory yet, empty reading zone: plain causal attention over the new tokens (numpy oracle)."""
    from oracle import loma_oracle as lo
    B, H, d, t, c, l = 1, 2, 128, 16, 4, 40
    rng = np.random.default_rng(9486 + 77)
    q, kn, vn = (wl.f32_to_bf16_bits(rng.standard_normal((B, H, l, d)).astype(np.float32)) for _ in range(3))
    k_read = torch.zeros((B, H, t * c, d), dtype=torch.bfloat16, device="cuda")
    v_read = torch.zeros_like(k_read)
    lse = torch.empty((B, H, l), dtype=torch.float32, device="cuda")
    out = loma.loma_prefill_attn(to_dev(q), to_dev(kn), to_dev(vn), None, None, k_read, v_read, t, c, 0, 0, 1 / math.sqrt(d),
                                 lse=lse)
    gen = lo.GenerationCache(B, H, d, t, c, 1 / math.sqrt(d))
    ref = gen.prefill(*(wl.bf16_bits_to_f32(x) for x in (q, kn, vn)))
    check(to_host_f64(out), ref, "bf16", "empty cache")
    assert np.abs(lse.cpu().numpy().astype(np.float64) - gen.last_lse).max() <= 2e-3
    assert np.array_equal(host_bits(k_read[:, :, :l]), kn) and np.array_equal(host_bits(v_read[:, :, :l]), vn)
    assert not k_read[:, :, l:].any() and not v_read[:, :, l:].any()


def test_decode_without_new_token(loma, c_oracle):
    cfg = gen_small("nonew", 2, 2, 128, 16, 4, 4, 1)
    st = wl.gen_initial_state(cfg)
    dev = {k: to_dev(v) for k, v in st.items()}
    q, _, _ = wl.gen_step_inputs(cfg, 0)
    nws = loma.loma_decode_workspace_bytes(cfg.B, cfg.H, cfg.d, cfg.t, cfg.c, cfg.prior_chunks)
    ws = torch.empty(max(nws, 16), dtype=torch.uint8, device="cuda")
    for fill in (0, 1, 37, cfg.R):
        before = dev["k_read"].clone()
        out = loma.loma_decode_attn(to_dev(q), None, None, dev["k_mem"], dev["v_mem"], dev["k_read"], dev["v_read"],
                                    cfg.t, cfg.c, cfg.prior_chunks, fill, cfg.scale, workspace=ws)
        ref = c_oracle.attend_segments(q, st["k_mem"], st["v_mem"], cfg.prior_chunks * cfg.t,
                                       st["k_read"], st["v_read"], fill, cfg.scale).reshape(cfg.B, cfg.H, 1, cfg.d)
        check(to_host_f64(out), ref, cfg.dtype, f"fill {fill}")
        assert torch.equal(before.view(torch.int16), dev["k_read"].view(torch.int16))   # cache untouched


def test_generation_entry_points_are_deterministic(loma):
    """Same inputs twice: decode (split over workgroups and single-workgroup shapes), compress and the prompt
    form return the same bits, and leave the same bits in the caches (fixed combine order, no atomics)."""
    for B, H, prior in ((1, 8, 300), (8, 32, 20)):
        cfg = gen_small("det_gen", B, H, 128, 16, 4, prior, 64)
        st = wl.gen_initial_state(cfg)
        q, kn, vn = (to_dev(x) for x in wl.gen_step_inputs(cfg, 3))
        qm, km, vm = (to_dev(x) for x in wl.gen_compress_inputs(cfg, 0))
        toks = [wl.gen_step_inputs(cfg, 10 + i) for i in range(40)]
        pq, pk, pv = (to_dev(np.concatenate([tk[j] for tk in toks], axis=2)) for j in range(3))
        ws = torch.empty(max(loma.loma_decode_workspace_bytes(cfg.B, cfg.H, cfg.d, cfg.t, cfg.c, prior + 1), 16),
                         dtype=torch.uint8, device="cuda")
        results = []
        for rep in range(2):
            dev = {k: to_dev(v) for k, v in st.items()}
            o1 = loma.loma_compress_step(qm, km, vm, dev["k_read"], dev["v_read"], dev["k_mem"], dev["v_mem"],
                                         cfg.t, cfg.c, prior, cfg.scale)
            o2 = loma.loma_decode_attn(q, kn, vn, dev["k_mem"], dev["v_mem"], dev["k_read"], dev["v_read"],
                                       cfg.t, cfg.c, prior + 1, 0, cfg.scale, workspace=ws)
            lse = torch.empty((cfg.B, cfg.H, 40), dtype=torch.float32, device="cuda")
            o3 = loma.loma_prefill_attn(pq, pk, pv, dev["k_mem"], dev["v_mem"], dev["k_read"], dev["v_read"],
                                        cfg.t, cfg.c, prior + 1, 1, cfg.scale, lse=lse)
            torch.cuda.synchronize()
            results.append([o1, o2, o3, lse, dev["k_mem"], dev["v_mem"], dev["k_read"], dev["v_read"]])
        for a, b in zip(*results):
            va = a.view(torch.int16) if a.dtype == torch.bfloat16 else a.view(torch.int32)
            vb = b.view(torch.int16) if b.dtype == torch.bfloat16 else b.view(torch.int32)
            assert torch.equal(va, vb)


def test_decode_without_a_memory_cache(loma, c_oracle):
    """Before the first compression there is no memory cache: k_memcache / v_memcache are NULL."""
    cfg = gen_small("nomem", 2, 4, 128, 16, 4, 0, 40)
    st = wl.gen_initial_state(cfg)
    k_read, v_read = torch.zeros_like(to_dev(st["k_read"])), torch.zeros_like(to_dev(st["v_read"]))
    empty = np.zeros((cfg.B, cfg.H, cfg.t, cfg.d), dtype=np.uint16)
    orc = c_oracle.GenerationCache(empty, empty.copy(), 0, np.zeros_like(st["k_read"]), np.zeros_like(st["v_read"]), 0,
                                   cfg.t, cfg.c, cfg.scale)
    ws = torch.empty(max(loma.loma_decode_workspace_bytes(cfg.B, cfg.H, cfg.d, cfg.t, cfg.c, 0), 16), dtype=torch.uint8,
                     device="cuda")
    for step in range(cfg.steps):
        q, kn, vn = wl.gen_step_inputs(cfg, step)
        out = loma.loma_decode_attn(to_dev(q), to_dev(kn), to_dev(vn), None, None, k_read, v_read, cfg.t, cfg.c, 0, step,
                                    cfg.scale, workspace=ws)
        ref = orc.decode(q, kn, vn).reshape(cfg.B, cfg.H, 1, cfg.d)
        check(to_host_f64(out), ref, cfg.dtype, f"no memory cache, step {step}")
    assert np.array_equal(host_bits(k_read[:, :, :cfg.steps]), orc.k_read[:, :, :cfg.steps])


def test_generation_matches_mask_pass_rows_on_gpu(loma):
    """Sec. 3.1 vs Sec. 4.3 on the device: decode outputs equal reading rows and compress outputs
    equal memory rows of the full-mask pass over the same Q/K/V (both bf16; equal up to rounding)."""
    cfg = small("equiv", 1, 2, 128, 16, 4, 3)
    q, k, v = (to_dev(x) for x in wl.mask_inputs(cfg))
    full = loma.loma_mask_attn_fwd(q, k, v, cfg.t, cfg.c, cfg.n_chunks, cfg.scale).float()
    B, H, d, t, c, R, s = cfg.B, cfg.H, cfg.d, cfg.t, cfg.c, cfg.R, cfg.s
    k_mem = torch.zeros((B, H, cfg.n_chunks * t, d), dtype=torch.bfloat16, device="cuda")
    v_mem = torch.zeros_like(k_mem)
    k_read = torch.zeros((B, H, R, d), dtype=torch.bfloat16, device="cuda")
    v_read = torch.zeros_like(k_read)
    ws = torch.empty(max(loma.loma_decode_workspace_bytes(B, H, d, t, c, cfg.n_chunks), 16), dtype=torch.uint8, device="cuda")
    worst = 0.0
    for y in range(cfg.n_chunks):
        for o in range(R):
            p = y * s + o
            out = loma.loma_decode_attn(q[:, :, p:p + 1].contiguous(), k[:, :, p:p + 1].contiguous(),
                                        v[:, :, p:p + 1].contiguous(), k_mem, v_mem, k_read, v_read, t, c, y, o,
                                        cfg.scale, workspace=ws)
            worst = max(worst, (out.float()[:, :, 0] - full[:, :, p]).abs().max().item())
        m0 = y * s + R
        out = loma.loma_compress_step(q[:, :, m0:m0 + t].contiguous(), k[:, :, m0:m0 + t].contiguous(),
                                      v[:, :, m0:m0 + t].contiguous(), k_read, v_read, k_mem, v_mem, t, c, y, cfg.scale)
        worst = max(worst, (out.float() - full[:, :, m0:m0 + t]).abs().max().item())
    assert worst <= 2e-2, worst


def test_binding_reports_errors(loma):
    q = torch.zeros((1, 1, 144, 64), device="cuda")
    with pytest.raises(ValueError):
        loma.loma_mask_attn_fwd(q, q, q, 4, 4, 5, 0.125)        # S != n*s
    with pytest.raises(loma.LomaError) as e:
        loma.loma_mask_attn_fwd(q, q, q, 4, 4, 4, -1.0)
    assert e.value.status == loma.ERR_INVALID_ARG


# ---- gradients of the mask pass ---------------------------------------------------------------------------
def run_mask_bwd(loma, c_oracle, cfg):
    """Forward (out, lse) and backward both through the C ABI; the oracle differentiates its own forward."""
    print(f"[case] mask pass gradients {cfg}", flush=True)
    q, k, v = wl.mask_inputs(cfg)
    g = wl.mask_grad_input(cfg)
    tq, tk, tv, tg = (to_dev(x) for x in (q, k, v, g))
    lse = torch.empty((cfg.B, cfg.H, cfg.S), dtype=torch.float32, device="cuda")
    out = loma.loma_mask_attn_fwd(tq, tk, tv, cfg.t, cfg.c, cfg.n_chunks, cfg.scale, lse=lse)
    keep = [x.clone() for x in (tq, tk, tv, out, tg)]
    dq, dk, dv = loma.loma_mask_attn_bwd(tq, tk, tv, out, lse, tg, cfg.t, cfg.c, cfg.n_chunks, cfg.scale)
    torch.cuda.synchronize()
    for a, b in zip(keep, (tq, tk, tv, out, tg)):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16)), "the backward pass wrote to an input"
    rq, rk, rv = c_oracle.mask_attn_bwd(q, k, v, g, cfg.t, cfg.c, cfg.n_chunks, cfg.scale)
    for name, got, want in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv)):
        check_grad(to_host_f64(got), want, cfg.dtype, f"{cfg.name} {name}")
    return dq, dk, dv


@pytest.mark.parametrize("cfg", [
    wl.CONFIGS[0],
    small("bwd_f32_d128_t16c2", 1, 2, 128, 16, 2, 3, dtype="f32", scale=1.0),
    small("bwd_f32_d40_t3c3", 2, 1, 40, 3, 3, 4, dtype="f32", scale=1.0),
    small("bwd_f32_t1c1", 1, 1, 64, 1, 1, 5, dtype="f32", scale=1.0),
    small("bwd_bf16_d96", 1, 2, 96, 8, 2, 3),
    small("bwd_bf16_d256", 1, 1, 256, 4, 3, 2),
    small("bwd_f32_long_rows", 1, 1, 64, 40, 3, 3, dtype="f32", scale=1.0),   # more than 64 rows per key and keys per row
], ids=lambda c: c.name)
def test_mask_pass_gradients_generic_small(loma, c_oracle, cfg):
    run_mask_bwd(loma, c_oracle, cfg)


@pytest.mark.parametrize("cfg", [
    small("bwd_bf16_t16c4_bm64", 1, 2, 128, 16, 4, 3),          # 2 waves: memory-key block spans 4 chunks > 3
    small("bwd_bf16_t16c4_n9", 1, 1, 128, 16, 4, 9),            # three memory-key blocks, later chunks see all of a block
    small("bwd_bf16_t32c8_bm128", 1, 2, 128, 32, 8, 6),         # 4 waves, one chunk's memory zone per wave
    small("bwd_bf16_t4c4_bm32", 2, 1, 128, 4, 4, 11),           # 1 wave, 8 chunks per memory-key block
    small("bwd_bf16_t5c7_ragged", 1, 3, 128, 5, 7, 8),          # R = 35, t = 5: nothing aligned
    small("bwd_bf16_t24c6_ragged128", 1, 1, 128, 24, 6, 3),     # R = 144
    small("bwd_bf16_t40c1", 1, 2, 128, 40, 1, 4),               # memory zone longer than a wave's 32 keys
    small("bwd_bf16_t1c1", 1, 1, 128, 1, 1, 5),                 # degenerate: every zone one token
    small("bwd_bf16_d64_t16c4", 1, 2, 64, 16, 4, 5),
    small("bwd_bf16_d64_t32c8", 1, 1, 64, 32, 8, 3),
    small("bwd_bf16_d64_t4c4_bm32", 1, 2, 64, 4, 4, 11),        # head_dim 64 on the 1-wave kernels
    small("bwd_bf16_nbh8_xcd", 1, 8, 128, 16, 2, 6),            # B*H multiple of 8
    small("bwd_bf16_one_chunk", 1, 2, 128, 32, 8, 1),           # a single chunk: no memory key is seen from outside its chunk
    small("bwd_bf16_one_chunk_t16", 2, 1, 64, 16, 4, 1),
    small("bwd_bf16_t32c8_n9_split", 1, 1, 128, 32, 8, 9),      # 4 waves, memory-key streams shared by two workgroups
], ids=lambda c: c.name)
def test_mask_pass_gradients_mfma_small(loma, c_oracle, cfg):
    run_mask_bwd(loma, c_oracle, cfg)


@pytest.mark.parametrize("shape", random_shapes(9488, 24), ids=lambda s: "B%d_H%d_d%d_t%d_c%d_n%d" % s)
def test_mask_pass_gradients_random_shapes(loma, c_oracle, shape):
    B, H, d, t, c, n = shape
    run_mask_bwd(loma, c_oracle, small("bwd_rand_%d_%d_%d" % (t, c, n), B, H, d, t, c, n + 3))


def test_mask_pass_gradients_are_deterministic(loma):
    cfg = small("bwd_det", 1, 4, 128, 32, 4, 4)
    q, k, v = (to_dev(x) for x in wl.mask_inputs(cfg))
    g = to_dev(wl.mask_grad_input(cfg))
    lse = torch.empty((cfg.B, cfg.H, cfg.S), dtype=torch.float32, device="cuda")
    out = loma.loma_mask_attn_fwd(q, k, v, cfg.t, cfg.c, cfg.n_chunks, cfg.scale, lse=lse)
    a = loma.loma_mask_attn_bwd(q, k, v, out, lse, g, cfg.t, cfg.c, cfg.n_chunks, cfg.scale)
    b = loma.loma_mask_attn_bwd(q, k, v, out, lse, g, cfg.t, cfg.c, cfg.n_chunks, cfg.scale)
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x.view(torch.int16), y.view(torch.int16))


def test_mask_pass_gradients_need_their_workspace(loma):
    cfg = small("bwd_ws", 1, 1, 64, 4, 2, 2, dtype="f32")
    q, k, v = (to_dev(x) for x in wl.mask_inputs(cfg))
    g = to_dev(wl.mask_grad_input(cfg))
    lse = torch.empty((1, 1, cfg.S), dtype=torch.float32, device="cuda")
    out = loma.loma_mask_attn_fwd(q, k, v, cfg.t, cfg.c, cfg.n_chunks, cfg.scale, lse=lse)
    need = loma.loma_mask_attn_bwd_workspace_bytes(1, 1, 64, cfg.t, cfg.c, cfg.n_chunks, torch.float32)
    assert need == 8 * cfg.S
    small_ws = torch.empty(need - 4, dtype=torch.uint8, device="cuda")
    with pytest.raises(loma.LomaError) as e:
        loma.loma_mask_attn_bwd(q, k, v, out, lse, g, cfg.t, cfg.c, cfg.n_chunks, cfg.scale, workspace=small_ws)
    assert e.value.status == loma.ERR_WORKSPACE
    with pytest.raises(loma.LomaError) as e:      # an output that aliases an input
        loma.loma_mask_attn_bwd(q, k, v, out, lse, g, cfg.t, cfg.c, cfg.n_chunks, cfg.scale, dq=q)
    assert e.value.status == loma.ERR_INVALID_ARG
