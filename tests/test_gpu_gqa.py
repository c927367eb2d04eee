"""Grouped-query decode (loma_decode_attn_gqa): H query heads over H_kv shared key/value heads.  The expected output
is the oracle's plain decode on a cache whose KV heads are written out once per query head (np.repeat), which
is what head sharing means; the appended K/V rows are compared bit for bit, and with H == H_kv the call must agree
with loma_decode_attn."""
import numpy as np
import pytest
import torch

from gpu_util import check, host_bits, to_dev, to_host_f64
from paper_2401_09486_amd import workloads as wl

pytestmark = pytest.mark.gpu


def gqa_case(c_oracle, loma, B, Hq, Hkv, d, t, c, prior, fill, with_new, seed=0):
    G = Hq // Hkv
    kv_cfg = wl.GenConfig(40 + seed, "gqa_kv", B, Hkv, d, t, c, prior, 1, "bf16", 1.0, 1.0)
    q_cfg = wl.GenConfig(41 + seed, "gqa_q", B, Hq, d, t, c, prior, 1, "bf16", 1.0, 1.0)
    st = wl.gen_initial_state(kv_cfg)
    _, kn, vn = wl.gen_step_inputs(kv_cfg, fill)
    q, _, _ = wl.gen_step_inputs(q_cfg, fill)
    dev = {k: to_dev(v) for k, v in st.items()}
    cap = st["k_mem"].shape[2]
    ws = torch.empty(max(loma.loma_decode_gqa_workspace_bytes(B, Hq, Hkv, d), 16), dtype=torch.uint8, device="cuda")
    out = loma.loma_decode_attn_gqa(to_dev(q), to_dev(kn) if with_new else None, to_dev(vn) if with_new else None,
                                    dev["k_mem"] if prior > 0 else None, dev["v_mem"] if prior > 0 else None,
                                    dev["k_read"], dev["v_read"], t, c, prior, fill, kv_cfg.scale, workspace=ws)
    torch.cuda.synchronize()
    rep = lambda a: np.repeat(a, G, axis=1)
    if with_new:
        orc = c_oracle.GenerationCache(rep(st["k_mem"]), rep(st["v_mem"]), prior, rep(st["k_read"]), rep(st["v_read"]),
                                       fill, t, c, kv_cfg.scale)
        ref = orc.decode(q, rep(kn), rep(vn)).reshape(B, Hq, 1, d)
        # the new token's K/V joined the reading zone of every KV head, bits unchanged
        assert np.array_equal(host_bits(dev["k_read"][:, :, fill]), kn[:, :, 0])
        assert np.array_equal(host_bits(dev["v_read"][:, :, fill]), vn[:, :, 0])
    else:
        ref = c_oracle.attend_segments(q, rep(st["k_mem"]), rep(st["v_mem"]), prior * t, rep(st["k_read"]), rep(st["v_read"]),
                                       fill, kv_cfg.scale).reshape(B, Hq, 1, d)
        assert np.array_equal(host_bits(dev["k_read"]), st["k_read"])
    assert np.array_equal(host_bits(dev["k_read"][:, :, :fill]), st["k_read"][:, :, :fill])
    assert np.array_equal(host_bits(dev["k_mem"]), st["k_mem"])
    return out, ref, (st, q, kn, vn, dev)


@pytest.mark.parametrize("shape,fills", [
    ((2, 8, 2, 128, 16, 4, 12), (0, 17, 63)),      # G = 4
    ((1, 16, 2, 64, 8, 4, 30), (0, 5, 31)),        # G = 8, head_dim 64
    ((8, 32, 8, 128, 16, 4, 65), (11,)),           # the generation shape with 8 KV heads
    ((1, 4, 2, 128, 16, 4, 0), (0, 9)),            # G = 2, no memory yet: the cache pointers may be NULL
    ((3, 6, 6, 128, 16, 2, 7), (3,)),              # G = 1
], ids=["g4", "g8_d64", "c3_shape_8kv", "g2_empty_memory", "g1"])
def test_gqa_decode_matches_oracle(c_oracle, shape, fills):
    from paper_2401_09486_amd import loma
    B, Hq, Hkv, d, t, c, prior = shape
    for fill in fills:
        print(f"[case] gqa decode {shape} fill={fill}", flush=True)
        out, ref, _ = gqa_case(c_oracle, loma, B, Hq, Hkv, d, t, c, prior, fill, True)
        mx, mean = check(to_host_f64(out), ref, "bf16", f"gqa decode {shape} fill={fill}")
        print(f"       max {mx:.2e} mean {mean:.2e}", flush=True)


def test_gqa_decode_without_a_new_token(c_oracle):
    from paper_2401_09486_amd import loma
    B, Hq, Hkv, d, t, c, prior, fill = 2, 8, 4, 128, 16, 4, 9, 40
    out, ref, _ = gqa_case(c_oracle, loma, B, Hq, Hkv, d, t, c, prior, fill, False)
    check(to_host_f64(out), ref, "bf16", "gqa decode, cache read only")


def test_gqa_with_one_group_agrees_with_plain_decode_and_repeats_bit_exactly(c_oracle):
    from paper_2401_09486_amd import loma
    B, H, d, t, c, prior, fill = 2, 8, 128, 16, 4, 20, 13
    out, ref, (st, q, kn, vn, _) = gqa_case(c_oracle, loma, B, H, H, d, t, c, prior, fill, True)
    dev2 = {k: to_dev(v) for k, v in st.items()}
    ws = torch.empty(max(loma.loma_decode_workspace_bytes(B, H, d, t, c, prior), 16), dtype=torch.uint8, device="cuda")
    plain = loma.loma_decode_attn(to_dev(q), to_dev(kn), to_dev(vn), dev2["k_mem"], dev2["v_mem"], dev2["k_read"],
                                  dev2["v_read"], t, c, prior, fill, wl.GenConfig(40, "x", B, H, d, t, c, prior, 1, "bf16", 1.0, 1.0).scale, workspace=ws)
    # different split plans, same arithmetic per key: the two agree far inside the parity bar
    assert np.abs(to_host_f64(out) - to_host_f64(plain)).max() <= 4e-3
    out2, _, _ = gqa_case(c_oracle, loma, B, H, H, d, t, c, prior, fill, True)
    assert np.array_equal(host_bits(out), host_bits(out2))


def test_gqa_rejects_what_it_cannot_do():
    from paper_2401_09486_amd import loma
    B, d, t, c = 1, 128, 16, 4
    q = torch.zeros((B, 6, 1, d), dtype=torch.bfloat16, device="cuda")
    kr = torch.zeros((B, 2, t * c, d), dtype=torch.bfloat16, device="cuda")
    kn = torch.zeros((B, 2, 1, d), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(loma.LomaError) as e:      # three query heads per KV head
        loma.loma_decode_attn_gqa(q, kn, kn.clone(), None, None, kr, kr.clone(), t, c, 0, 0, 0.1)
    assert e.value.status == loma.ERR_UNSUPPORTED
    q5 = torch.zeros((B, 5, 1, d), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(loma.LomaError) as e:      # not a multiple at all
        loma.loma_decode_attn_gqa(q5, kn, kn.clone(), None, None, kr, kr.clone(), t, c, 0, 0, 0.1)
    assert e.value.status == loma.ERR_INVALID_ARG
