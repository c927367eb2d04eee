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


def test_gqa_decode_high_ratio_shape_full_size(c_oracle):
    """The launch configuration the benchmark times: B64, 32 query heads over 8 KV heads, 8208 memory KVs plus a
    part-filled reading zone, tensors filled on the device from a host-drawn pool.  The oracle follows 12 sampled
    (b, KV head) pairs with their four query heads each through 6 steps on the same bits."""
    from paper_2401_09486_amd import loma
    c5 = wl.CONFIGS[4]
    B, Hq, Hkv, d, t, c = c5.B, c5.H, 8, c5.d, c5.t, c5.c
    G = Hq // Hkv
    n_mem, cap = c5.prior_chunks + 1, c5.mem_capacity
    pool = wl.TiledPool(c5.seed + 7)
    st = {"k_mem": pool.tensor((B, Hkv, cap, d)), "v_mem": pool.tensor((B, Hkv, cap, d)),
          "k_read": pool.tensor((B, Hkv, t * c, d)), "v_read": pool.tensor((B, Hkv, t * c, d))}
    nkv = B * Hkv
    sel = np.array(sorted(set(np.linspace(0, nkv - 1, 12).astype(int))), dtype=np.int64)
    tsel = torch.from_numpy(sel).cuda()
    qsel = (tsel[:, None] * G + torch.arange(G, device="cuda")[None, :]).reshape(-1)     # their query heads

    def pick_kv(x):   # [B, Hkv, L, d] device -> [1, nsel * G, L, d] host bits, every KV head once per query head
        flat = x.view(nkv, x.shape[2], x.shape[3])
        return np.repeat(host_bits(flat[tsel].contiguous()), G, axis=0)[None]

    fill0 = 37
    orc = c_oracle.GenerationCache(pick_kv(st["k_mem"]), pick_kv(st["v_mem"]), n_mem, pick_kv(st["k_read"]),
                                   pick_kv(st["v_read"]), fill0, t, c, c5.scale)
    ws = torch.empty(max(loma.loma_decode_gqa_workspace_bytes(B, Hq, Hkv, d), 16), dtype=torch.uint8, device="cuda")
    worst = 0.0
    for step in range(6):
        fill = fill0 + step
        print(f"[case] gqa high-ratio shape step {step} fill {fill}", flush=True)
        q = pool.tensor((B, Hq, 1, d), c5.q_scale)
        kn, vn = pool.tensor((B, Hkv, 1, d)), pool.tensor((B, Hkv, 1, d))
        out = loma.loma_decode_attn_gqa(q, kn, vn, st["k_mem"], st["v_mem"], st["k_read"], st["v_read"], t, c, n_mem, fill,
                                        c5.scale, workspace=ws)
        qh = host_bits(q.view(B * Hq, 1, d)[qsel].contiguous())[None]
        ref = orc.decode(qh, pick_kv(kn), pick_kv(vn))
        mx, _ = check(to_host_f64(out.view(B * Hq, 1, d)[qsel]), ref.reshape(-1, 1, d), "bf16", f"gqa full-size step {step}")
        worst = max(worst, mx)
        assert torch.equal(st["k_read"][:, :, fill], kn[:, :, 0]) and torch.equal(st["v_read"][:, :, fill], vn[:, :, 0])
    assert torch.isfinite(out.float()).all()
    print(f"[result] gqa high-ratio shape: worst max abs {worst:.3e}", flush=True)


@pytest.mark.parametrize("shape,fill,with_new", [
    ((2, 8, 2, 128, 16, 4, 12), 17, True),       # G = 4, keys split over workgroups, combine kernel
    ((8, 32, 8, 128, 16, 4, 20), 5, True),       # 64 KV heads per layer
    ((1, 16, 2, 64, 8, 4, 9), 3, True),          # G = 8 (4-wave workgroups), head_dim 64
    ((1, 4, 2, 128, 16, 4, 0), 7, True),         # no memory yet: the cache tables may be NULL
    ((1, 8, 4, 128, 16, 4, 30), 40, False),      # no new token
], ids=["g4_splitk", "kv64", "g8_d64", "empty_memory", "no_new_token"])
def test_gqa_layered_decode_is_the_single_layer_call_per_layer(c_oracle, shape, fill, with_new):
    """loma_decode_attn_gqa_layers: every layer's output and cache rows bit for bit what loma_decode_attn_gqa gives
    on that layer's tensors (which the tests above hold against the oracle)."""
    from paper_2401_09486_amd import loma
    B, Hq, Hkv, d, t, c, prior = shape
    L = 3
    print(f"[case] layered gqa decode {shape} fill={fill} new={with_new}", flush=True)
    layers = []
    for l in range(L):
        kv_cfg = wl.GenConfig(60 + 2 * l, "gqa_layers_kv", B, Hkv, d, t, c, prior, 1, "bf16", 1.0, 1.0)
        q_cfg = wl.GenConfig(61 + 2 * l, "gqa_layers_q", B, Hq, d, t, c, prior, 1, "bf16", 1.0, 1.0)
        st = wl.gen_initial_state(kv_cfg)
        _, kn, vn = wl.gen_step_inputs(kv_cfg, fill)
        q, _, _ = wl.gen_step_inputs(q_cfg, fill)
        layers.append({"st": {k: to_dev(v) for k, v in st.items()}, "single": {k: to_dev(v) for k, v in st.items()},
                       "q": to_dev(q), "kn": to_dev(kn), "vn": to_dev(vn), "scale": kv_cfg.scale})
    cap = layers[0]["st"]["k_mem"].shape[2]
    outs = [torch.empty_like(x["q"]) for x in layers]
    tab = loma.pointer_table
    ws = torch.empty(max(L * loma.loma_decode_gqa_workspace_bytes(B, Hq, Hkv, d), 16), dtype=torch.uint8, device="cuda")
    loma.loma_decode_attn_gqa_layers(
        tab([x["q"] for x in layers]), tab([x["kn"] for x in layers]) if with_new else None,
        tab([x["vn"] for x in layers]) if with_new else None,
        tab([x["st"]["k_mem"] for x in layers]) if prior > 0 else None, tab([x["st"]["v_mem"] for x in layers]) if prior > 0 else None,
        tab([x["st"]["k_read"] for x in layers]), tab([x["st"]["v_read"] for x in layers]), tab(outs),
        L, B, Hq, Hkv, d, t, c, prior, cap, fill, layers[0]["scale"], workspace=ws)
    torch.cuda.synchronize()
    ws1 = torch.empty(max(loma.loma_decode_gqa_workspace_bytes(B, Hq, Hkv, d), 16), dtype=torch.uint8, device="cuda")
    for l, x in enumerate(layers):
        s1 = x["single"]
        ref = loma.loma_decode_attn_gqa(x["q"], x["kn"] if with_new else None, x["vn"] if with_new else None,
                                        s1["k_mem"] if prior > 0 else None, s1["v_mem"] if prior > 0 else None,
                                        s1["k_read"], s1["v_read"], t, c, prior, fill, x["scale"], workspace=ws1)
        torch.cuda.synchronize()
        assert torch.equal(outs[l], ref), f"layer {l}: output differs from the single-layer call"
        assert torch.equal(x["st"]["k_read"], s1["k_read"]) and torch.equal(x["st"]["v_read"], s1["v_read"])
        assert torch.equal(x["st"]["k_mem"], s1["k_mem"])
