"""One decode step on several layers' caches in one launch (loma_decode_attn_layers): each layer's output and
appended K/V row against the oracle (an independent cache per layer) and, bit for bit, against a single-layer
call on the same tensors."""
import numpy as np
import pytest
import torch

from gpu_util import check, host_bits, to_dev, to_host_f64
from paper_2401_09486_amd import workloads as wl

pytestmark = pytest.mark.gpu


def layer_cfg(base, layer):
    """Layer `layer` of a stack: same shape, its own seeded tensors."""
    return wl.GenConfig(base.index + 100 * (layer + 1), f"{base.name}_layer{layer}", base.B, base.H, base.d, base.t,
                        base.c, base.prior_chunks, base.steps, base.dtype, base.kv_scale, base.q_scale)


@pytest.mark.parametrize("shape,fills,with_new", [
    ((1, 8, 128, 16, 4, 300), (0, 17, 63), True),      # few (b,h) pairs: keys split over workgroups, combine kernel
    ((8, 32, 128, 16, 4, 20), (5,), True),             # 256 pairs: one 16-wave workgroup per pair and layer
    ((2, 3, 64, 8, 4, 9), (0, 31), True),              # head_dim 64
    ((1, 4, 128, 16, 4, 0), (7,), True),               # no memory yet: the cache tables may be NULL
    ((1, 8, 128, 16, 4, 40), (1, 64), False),          # no new token: cache read only
], ids=["splitk", "c3_shape", "d64", "empty_memory", "no_new_token"])
def test_layered_decode(c_oracle, shape, fills, with_new):
    from paper_2401_09486_amd import loma
    B, H, d, t, c, prior = shape
    L = 5
    base = wl.GenConfig(2, "layers", B, H, d, t, c, prior, 1, "bf16", 1.0, 1.0)
    cfgs = [layer_cfg(base, l) for l in range(L)]
    for fill in fills:
        print(f"[case] layered decode {shape} fill={fill} new={with_new}", flush=True)
        host = [wl.gen_initial_state(cf) for cf in cfgs]
        toks = [wl.gen_step_inputs(cf, fill) for cf in cfgs]
        dev = [{k: to_dev(v) for k, v in st.items()} for st in host]
        single = [{k: v.clone() for k, v in dl.items()} for dl in dev]
        dq = [to_dev(tk[0]) for tk in toks]
        dkn = [to_dev(tk[1]) for tk in toks]
        dvn = [to_dev(tk[2]) for tk in toks]
        outs = [torch.empty_like(x) for x in dq]
        cap = host[0]["k_mem"].shape[2]
        tab = loma.pointer_table
        nws = loma.loma_decode_layers_workspace_bytes(L, B, H, d, t, c, prior)
        ws = torch.empty(max(nws, 16), dtype=torch.uint8, device="cuda")
        loma.loma_decode_attn_layers(
            tab(dq), tab(dkn) if with_new else None, tab(dvn) if with_new else None,
            tab([x["k_mem"] for x in dev]) if prior > 0 else None, tab([x["v_mem"] for x in dev]) if prior > 0 else None,
            tab([x["k_read"] for x in dev]), tab([x["v_read"] for x in dev]), tab(outs),
            L, B, H, d, t, c, prior, cap, fill, base.scale, workspace=ws)
        torch.cuda.synchronize()
        ws1 = torch.empty(max(loma.loma_decode_workspace_bytes(B, H, d, t, c, prior), 16), dtype=torch.uint8, device="cuda")
        for l in range(L):
            st, (q, kn, vn) = host[l], toks[l]
            if with_new:
                orc = c_oracle.GenerationCache(st["k_mem"].copy(), st["v_mem"].copy(), prior, st["k_read"].copy(),
                                               st["v_read"].copy(), fill, t, c, base.scale)
                ref = orc.decode(q, kn, vn).reshape(B, H, 1, d)
                assert np.array_equal(host_bits(dev[l]["k_read"][:, :, :fill + 1]), orc.k_read[:, :, :fill + 1])
                assert np.array_equal(host_bits(dev[l]["v_read"][:, :, :fill + 1]), orc.v_read[:, :, :fill + 1])
            else:
                ref = c_oracle.attend_segments(q, st["k_mem"], st["v_mem"], prior * t, st["k_read"], st["v_read"], fill,
                                               base.scale).reshape(B, H, 1, d)
            check(to_host_f64(outs[l]), ref, "bf16", f"layer {l}")
            one = loma.loma_decode_attn(dq[l], dkn[l] if with_new else None, dvn[l] if with_new else None,
                                        single[l]["k_mem"] if prior > 0 else None, single[l]["v_mem"] if prior > 0 else None,
                                        single[l]["k_read"], single[l]["v_read"], t, c, prior, fill, base.scale, workspace=ws1)
            torch.cuda.synchronize()
            assert torch.equal(one.view(torch.int16), outs[l].view(torch.int16)), f"layer {l}: differs from a single call"
            assert torch.equal(single[l]["k_read"].view(torch.int16), dev[l]["k_read"].view(torch.int16))
            assert torch.equal(single[l]["v_read"].view(torch.int16), dev[l]["v_read"].view(torch.int16))


def test_layered_decode_rejects_bad_arguments():
    from paper_2401_09486_amd import loma
    z = torch.zeros(3, dtype=torch.int64, device="cuda")
    with pytest.raises(loma.LomaError) as e:      # f32 data: no layered kernel
        loma.loma_decode_attn_layers(z, z, z, z, z, z, z, z, 3, 1, 8, 128, 16, 4, 4, 64, 0, 0.1, dtype=torch.float32)
    assert e.value.status == loma.ERR_UNSUPPORTED
    with pytest.raises(loma.LomaError) as e:      # split-K without its workspace
        loma.loma_decode_attn_layers(z, z, z, z, z, z, z, z, 3, 1, 8, 128, 16, 4, 4, 64, 0, 0.1)
    assert e.value.status == loma.ERR_WORKSPACE
    with pytest.raises(loma.LomaError) as e:      # reading zone already full
        loma.loma_decode_attn_layers(z, z, z, z, z, z, z, z, 3, 1, 8, 128, 16, 4, 4, 64, 64, 0.1)
    assert e.value.status == loma.ERR_INVALID_ARG
