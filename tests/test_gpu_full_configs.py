"""GPU parity at the full sizes of the five named configurations, in the launch configuration
bench.py times.  The oracle computes sampled outputs (rows / (b,h) pairs) one by one."""
import numpy as np
import pytest
import torch

from gpu_util import check, check_grad, host_bits, to_dev, to_host_f64
from paper_2401_09486_amd import workloads as wl
from test_gpu_parity import run_generation, run_prefill

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def loma():
    assert torch.cuda.is_available()
    from paper_2401_09486_amd import loma as m
    return m


@pytest.mark.parametrize("idx", [1, 3], ids=["config2_llama7b_mask", "config4_long_mask"])
def test_mask_pass_full_size(loma, c_oracle, idx):
    """Every row of every (b,h) pair, output and log-sum-exp, against the oracle."""
    cfg = wl.CONFIGS[idx]
    print(f"[case] full-size mask pass {cfg}", flush=True)
    q, k, v = wl.mask_inputs(cfg)
    lse = torch.empty((cfg.B, cfg.H, cfg.S), dtype=torch.float32, device="cuda")
    out = loma.loma_mask_attn_fwd(to_dev(q), to_dev(k), to_dev(v), cfg.t, cfg.c, cfg.n_chunks, cfg.scale, lse=lse)
    torch.cuda.synchronize()
    print("[progress] GPU pass done; oracle running", flush=True)
    ref, ref_lse = c_oracle.mask_attn(q, k, v, cfg.t, cfg.c, cfg.n_chunks, cfg.scale, return_lse=True)
    mx, mean = check(to_host_f64(out), ref, cfg.dtype, cfg.name)
    lse_err = float(np.abs(lse.cpu().numpy().astype(np.float64) - ref_lse).max())
    print(f"[result] {cfg.name}: all {cfg.S} rows x {cfg.B * cfg.H} (b,h): max abs {mx:.3e} mean abs {mean:.3e} "
          f"lse max abs {lse_err:.3e}", flush=True)
    assert lse_err <= 1e-4


@pytest.mark.parametrize("idx,npairs", [(1, 8), (3, 4)], ids=["config2_llama7b_mask", "config4_long_mask"])
def test_mask_pass_gradients_full_size(loma, c_oracle, idx, npairs):
    """Forward and backward at full size through the C ABI; the oracle differentiates whole (b,h) pairs
    (a pair's gradients depend on that pair alone), sampled across the batch and the XCD interleave."""
    cfg = wl.CONFIGS[idx]
    print(f"[case] full-size mask pass gradients {cfg}", flush=True)
    q, k, v = wl.mask_inputs(cfg)
    g = wl.mask_grad_input(cfg)
    tq, tk, tv, tg = (to_dev(x) for x in (q, k, v, g))
    lse = torch.empty((cfg.B, cfg.H, cfg.S), dtype=torch.float32, device="cuda")
    out = loma.loma_mask_attn_fwd(tq, tk, tv, cfg.t, cfg.c, cfg.n_chunks, cfg.scale, lse=lse)
    dq, dk, dv = loma.loma_mask_attn_bwd(tq, tk, tv, out, lse, tg, cfg.t, cfg.c, cfg.n_chunks, cfg.scale)
    torch.cuda.synchronize()
    nbh = cfg.B * cfg.H
    sel = sorted(set(np.linspace(0, nbh - 1, npairs).astype(int).tolist() + [1]))

    def pick(x):   # [B, H, S, d] -> [1, nsel, S, d]
        return np.ascontiguousarray(x.reshape(nbh, cfg.S, cfg.d)[sel])[None]

    rq, rk, rv = c_oracle.mask_attn_bwd(pick(q), pick(k), pick(v), pick(g), cfg.t, cfg.c, cfg.n_chunks, cfg.scale)
    for name, got, want in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv)):
        rel = check_grad(pick(to_host_f64(got)), want, cfg.dtype, f"{cfg.name} {name}")
        print(f"[result] {cfg.name} {name}: {len(sel)} (b,h) pairs, all rows: max abs err {rel:.3e}", flush=True)
        assert torch.isfinite(got.float()).all()


def test_generation_config3_full(loma, c_oracle):
    worst = run_generation(loma, c_oracle, wl.CONFIGS[2])
    print(f"[result] config 3: all 256 steps, all (b,h): worst max abs {worst:.3e}", flush=True)


def test_prefill_config3_shape_full(loma, c_oracle):
    """The generation configuration with the prompt fed a reading zone at a time (64 tokens per call, the shape
    bench.py times) and in uneven pieces; all (b,h), every new token."""
    cfg = wl.CONFIGS[2]
    run_prefill(loma, c_oracle, wl.GenConfig(cfg.index, "c3_prefill_whole_zone", cfg.B, cfg.H, cfg.d, cfg.t, cfg.c,
                                             cfg.prior_chunks, 2 * cfg.R, cfg.dtype, cfg.kv_scale, cfg.q_scale), (cfg.R,))
    run_prefill(loma, c_oracle, wl.GenConfig(cfg.index, "c3_prefill_pieces", cfg.B, cfg.H, cfg.d, cfg.t, cfg.c,
                                             cfg.prior_chunks, cfg.R, cfg.dtype, cfg.kv_scale, cfg.q_scale), (7, 33, 24))


def test_generation_config5_full(loma, c_oracle):
    """B64 H32, 8192 memory KVs + 256-token reading zone, 128 steps; the 9 GB caches and the step inputs are filled
    on the device from a host-drawn numpy pool (workloads.TiledPool); the oracle follows 24 sampled (b,h) pairs
    through every step on the same bits."""
    cfg = wl.CONFIGS[4]
    print(f"[case] full-size generation {cfg}", flush=True)
    pool = wl.TiledPool(cfg.seed)
    st = wl.gen_initial_state_device(cfg, pool=pool)
    nbh = cfg.B * cfg.H
    sel = np.array(sorted(set(np.linspace(0, nbh - 1, 24).astype(int))), dtype=np.int64)
    tsel = torch.from_numpy(sel).cuda()

    def pick(x):   # [B, H, L, d] device -> [1, nsel, L, d] host bits
        flat = x.view(nbh, x.shape[2], x.shape[3])
        return host_bits(flat[tsel].contiguous())[None]

    orc = c_oracle.GenerationCache(pick(st["k_mem"]), pick(st["v_mem"]), cfg.prior_chunks,
                                   pick(st["k_read"]), pick(st["v_read"]), cfg.R, cfg.t, cfg.c, cfg.scale)

    def draw(L, scale):
        return pool.tensor((cfg.B, cfg.H, L, cfg.d), scale)

    ws = torch.empty(max(loma.loma_decode_workspace_bytes(cfg.B, cfg.H, cfg.d, cfg.t, cfg.c, cfg.prior_chunks + 1), 16),
                     dtype=torch.uint8, device="cuda")
    n_mem, fill = cfg.prior_chunks, cfg.R
    worst = 0.0
    for step in range(cfg.steps):
        if fill == cfg.R:
            qm, km, vm = draw(cfg.t, cfg.q_scale), draw(cfg.t, cfg.kv_scale), draw(cfg.t, cfg.kv_scale)
            out = loma.loma_compress_step(qm, km, vm, st["k_read"], st["v_read"], st["k_mem"], st["v_mem"],
                                          cfg.t, cfg.c, n_mem, cfg.scale)
            ref = orc.compress(pick(qm), pick(km), pick(vm))
            mx, _ = check(to_host_f64(out.view(nbh, cfg.t, cfg.d)[tsel]), ref, cfg.dtype, "compress")
            worst = max(worst, mx)
            n_mem, fill = n_mem + 1, 0
        q, kn, vn = draw(1, cfg.q_scale), draw(1, cfg.kv_scale), draw(1, cfg.kv_scale)
        out = loma.loma_decode_attn(q, kn, vn, st["k_mem"], st["v_mem"], st["k_read"], st["v_read"],
                                    cfg.t, cfg.c, n_mem, fill, cfg.scale, workspace=ws)
        ref = orc.decode(pick(q), pick(kn), pick(vn))
        fill += 1
        mx, _ = check(to_host_f64(out.view(nbh, 1, cfg.d)[tsel]), ref, cfg.dtype, f"decode step {step}")
        worst = max(worst, mx)
        if step % 32 == 0:
            print(f"[progress] config 5 step {step} worst {worst:.3e}", flush=True)
            assert torch.isfinite(out.float()).all()
    print(f"[result] config 5: {cfg.steps} steps, {sel.size} sampled (b,h): worst max abs {worst:.3e}", flush=True)
