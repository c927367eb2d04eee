"""The decode entry point that allocates nothing (loma_decode_attn_static) against loma_decode_attn.

Both run the same kernels; the only difference is where the split-K partial results live (a fixed array inside
the library's device image instead of the caller's workspace), so the outputs and the appended K/V rows must be
bit-identical.  Two calls in a row, the second on a smaller input, share the array; shapes are chosen so that
several workgroups split every (b,h) pair's keys, i.e. the array is really used.
"""
import numpy as np
import pytest
import torch

from gpu_util import check, to_dev, to_host_f64
from paper_2401_09486_amd import workloads as wl

pytestmark = pytest.mark.gpu


def gen_cfg(name, B, H, d, t, c, prior, steps):
    return wl.GenConfig(2, name, B, H, d, t, c, prior, steps, "bf16", 1.0, 1.0)


def one_call(loma, c_oracle, cfg, fill):
    """A decode step at reading-zone fill `fill` through both entry points; returns the split count used."""
    print(f"[case] static-scratch decode {cfg} fill={fill}", flush=True)
    st = wl.gen_initial_state(cfg)
    q, kn, vn = wl.gen_step_inputs(cfg, 0)
    n_mem = cfg.prior_chunks
    need = loma.loma_decode_workspace_bytes(cfg.B, cfg.H, cfg.d, cfg.t, cfg.c, n_mem)
    assert 0 < need <= loma.decode_static_scratch_bytes()
    outs, caches = [], []
    for which in ("workspace", "static"):
        dev = {k: to_dev(v) for k, v in st.items()}
        if which == "workspace":
            ws = torch.empty(need, dtype=torch.uint8, device="cuda")
            out = loma.loma_decode_attn(to_dev(q), to_dev(kn), to_dev(vn), dev["k_mem"], dev["v_mem"], dev["k_read"],
                                        dev["v_read"], cfg.t, cfg.c, n_mem, fill, cfg.scale, workspace=ws)
        else:
            out = loma.loma_decode_attn_static(to_dev(q), to_dev(kn), to_dev(vn), dev["k_mem"], dev["v_mem"],
                                               dev["k_read"], dev["v_read"], cfg.t, cfg.c, n_mem, fill, cfg.scale)
        torch.cuda.synchronize()
        outs.append(out)
        caches.append((dev["k_read"], dev["v_read"]))
    assert torch.equal(outs[0].view(torch.int16), outs[1].view(torch.int16)), "outputs differ"
    for a, b in zip(caches[0], caches[1]):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16)), "appended rows differ"
    # and both are right: the oracle's decode step on the same state
    orc = c_oracle.GenerationCache(st["k_mem"].copy(), st["v_mem"].copy(), n_mem, st["k_read"].copy(),
                                   st["v_read"].copy(), fill, cfg.t, cfg.c, cfg.scale)
    ref = orc.decode(q, kn, vn).reshape(cfg.B, cfg.H, 1, cfg.d)
    check(to_host_f64(outs[1]), ref, "bf16", f"{cfg.name} static")


def test_static_scratch_decode_matches_workspace_decode(c_oracle):
    assert torch.cuda.is_available()
    from paper_2401_09486_amd import loma
    # 8 (b,h) pairs x 4800 memory keys: up to 32 splits per pair; then a smaller call (4 pairs, 1600 keys)
    one_call(loma, c_oracle, gen_cfg("static_big", 1, 8, 128, 16, 4, 300, 1), 17)
    one_call(loma, c_oracle, gen_cfg("static_small", 1, 4, 128, 16, 4, 100, 1), 3)
    # back to the large shape: what the smaller call left in the array does not matter
    one_call(loma, c_oracle, gen_cfg("static_big_again", 1, 8, 128, 16, 4, 300, 1), 63)


def test_static_scratch_decode_rejects_what_does_not_fit():
    from paper_2401_09486_amd import loma
    B, H, d, t, c = 4095, 1, 128, 16, 4       # 2 splits x 4095 pairs x 130 floats: just above the array
    assert loma.loma_decode_workspace_bytes(B, H, d, t, c, 4) > loma.decode_static_scratch_bytes()
    q = torch.zeros((B, H, 1, d), dtype=torch.bfloat16, device="cuda")
    mem = torch.zeros((B, H, 64, d), dtype=torch.bfloat16, device="cuda")
    rd = torch.zeros((B, H, t * c, d), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(loma.LomaError) as e:
        loma.loma_decode_attn_static(q, q, q, mem, mem, rd, rd, t, c, 4, 0, 0.1)
    assert e.value.status == loma.ERR_UNSUPPORTED
