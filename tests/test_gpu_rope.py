"""Rotary embedding on load (loma_decode_attn_rope, loma_compress_step_rope) against oracle rotate-then-attend.

The GPU gets UNROTATED q / k_new / q_mem / k_mem plus position ids; the oracle rotates the same rows in fp64
(oracle/loma_positions.py), rounds them to bf16 -- the type the rotated rows are held in -- and feeds its ordinary
generation routine.  Outputs are held to the usual bar.  The K rows the kernels leave in the caches are rotated
values rounded from fp32 arithmetic, the oracle's from fp64: they may differ by one bf16 unit in the last place
where the exact value lies within ~1e-7 of a rounding boundary, nowhere else.
"""
import numpy as np
import pytest
import torch

from gpu_util import check, host_bits, to_dev, to_host_f64
from paper_2401_09486_amd import workloads as wl

pytestmark = pytest.mark.gpu


def rotated_bits(lp, x_bits, pos, theta):
    return lp.round_to(lp.rope_rotate(wl.bf16_bits_to_f32(x_bits).astype(np.float64), pos, theta), "bf16")


def same_up_to_one_ulp(got_bits, want_bits, what):
    """bf16 bit patterns equal, except for rare elements (counted by the caller: about one in a thousand, where the
    exact value lies within the fp32 error, ~4e-7 of the operands, of a rounding boundary), which differ by one unit
    in the last place -- or, for results below 1e-4 in magnitude (a cancellation in x cos - y sin, where the fp32 error of
    the terms, ~1e-7, spans several of the result's tiny units), by at most 1e-6 in value."""
    got, want = wl.bf16_bits_to_f32(got_bits).astype(np.float64), wl.bf16_bits_to_f32(want_bits).astype(np.float64)
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(want), 1e-30))) - 7)
    err = np.abs(got - want)
    assert np.all(err <= np.maximum(ulp, 1e-6)), f"{what}: rotated rows off by {float((err / ulp).max()):.1f} units in the last place"
    return int((got_bits != want_bits).sum()), int(got_bits.size)


@pytest.mark.parametrize("shape,ptype,theta,cursor0", [
    ((2, 4, 128, 16, 4, 8, 140), "intermittent", 10000.0, 8 * 64),     # keys split over workgroups; 3 compressions
    ((8, 32, 128, 16, 4, 20, 70), "contiguous", 10000.0, 20 * 64),     # 256 pairs: one workgroup each
    ((1, 3, 64, 8, 4, 5, 70), "intermittent", 500000.0, 100000),       # head_dim 64, other base, large positions
    ((1, 2, 128, 40, 2, 3, 90), "contiguous", 10000.0, 3 * 80),        # compression on 2 waves
    ((1, 1, 128, 100, 1, 2, 110), "intermittent", 10000.0, 200),       # compression on 4 waves
], ids=["splitk_intermittent", "c3_shape_contiguous", "d64_far", "t40", "t100"])
def test_generation_with_rope_on_load(c_oracle, shape, ptype, theta, cursor0):
    from oracle import loma_positions as lp
    from paper_2401_09486_amd import loma
    B, H, d, t, c, prior, steps = shape
    cfg = wl.GenConfig(2, "rope", B, H, d, t, c, prior, steps, "bf16", 1.0, 1.0)
    print(f"[case] generation with rope on load {cfg} {ptype} theta={theta} cursor={cursor0}", flush=True)
    code = loma.POS_INTERMITTENT if ptype == "intermittent" else loma.POS_CONTIGUOUS
    st = wl.gen_initial_state(cfg)           # the caches hold (already rotated) K: any values will do
    dev = {k: to_dev(v) for k, v in st.items()}
    orc = c_oracle.GenerationCache(st["k_mem"].copy(), st["v_mem"].copy(), prior, st["k_read"].copy(),
                                   st["v_read"].copy(), cfg.R, t, c, cfg.scale)
    ws = torch.empty(max(loma.loma_decode_workspace_bytes(B, H, d, t, c, prior + cfg.n_compress), 16), dtype=torch.uint8,
                     device="cuda")
    n_mem, fill, events, cursor = prior, cfg.R, 0, cursor0      # cursor: real tokens fed so far; a full reading zone is pending
    worst, mismatch = 0.0, np.zeros(2, dtype=np.int64)
    for step in range(steps):
        if fill == cfg.R:
            qm, km, vm = wl.gen_compress_inputs(cfg, events)
            ids = lp.compress_position_ids(cursor, t, c, n_mem, ptype)
            assert ids.tolist() == [ids[0] + j * (ids[1] - ids[0] if t > 1 else 0) for j in range(t)]
            stride = int(ids[1] - ids[0]) if t > 1 else 1
            out = loma.loma_compress_step_rope(to_dev(qm), to_dev(km), to_dev(vm), dev["k_read"], dev["v_read"],
                                               dev["k_mem"], dev["v_mem"], t, c, n_mem, cfg.scale, int(ids[0]), stride, theta)
            km_rot = rotated_bits(lp, km, ids, theta)
            ref = orc.compress(rotated_bits(lp, qm, ids, theta), km_rot, vm).reshape(B, H, t, d)
            mx, _ = check(to_host_f64(out), ref, "bf16", f"compress event {events}")
            worst = max(worst, mx)
            lo_, hi_ = n_mem * t, (n_mem + 1) * t
            mismatch += same_up_to_one_ulp(host_bits(dev["k_mem"][:, :, lo_:hi_]), km_rot, "spliced K")
            assert np.array_equal(host_bits(dev["v_mem"][:, :, lo_:hi_]), vm)
            n_mem, fill, events = n_mem + 1, 0, events + 1
        q, kn, vn = wl.gen_step_inputs(cfg, step)
        out = loma.loma_decode_attn_rope(to_dev(q), to_dev(kn), to_dev(vn), dev["k_mem"], dev["v_mem"], dev["k_read"],
                                         dev["v_read"], t, c, n_mem, fill, cfg.scale, cursor, theta, workspace=ws)
        pos = lp.generation_position_ids(cursor, 1)
        kn_rot = rotated_bits(lp, kn, pos, theta)
        ref = orc.decode(rotated_bits(lp, q, pos, theta), kn_rot, vn).reshape(B, H, 1, d)
        mx, _ = check(to_host_f64(out), ref, "bf16", f"decode step {step}")
        worst = max(worst, mx)
        mismatch += same_up_to_one_ulp(host_bits(dev["k_read"][:, :, fill:fill + 1]), kn_rot, "appended K")
        assert np.array_equal(host_bits(dev["v_read"][:, :, fill:fill + 1]), vn)
        fill += 1
        cursor += 1
    print(f"[result] rope on load {shape} {ptype}: worst max abs {worst:.3e}; rotated K elements off by one ulp: "
          f"{mismatch[0]} of {mismatch[1]}", flush=True)
    assert mismatch[0] <= 5e-4 * mismatch[1] + 2, "too many rotated elements differ from the fp64 rotation"


def test_rope_at_position_zero_is_the_plain_step():
    """Position 0 turns nothing: the rope entry points return the bits of the plain ones."""
    from paper_2401_09486_amd import loma
    cfg = wl.GenConfig(2, "rope0", 1, 4, 128, 16, 4, 6, 4, "bf16", 1.0, 1.0)
    st = wl.gen_initial_state(cfg)
    q, kn, vn = (to_dev(x) for x in wl.gen_step_inputs(cfg, 0))
    qm, km, vm = (to_dev(x) for x in wl.gen_compress_inputs(cfg, 0))
    ws = torch.empty(max(loma.loma_decode_workspace_bytes(1, 4, 128, 16, 4, 7), 16), dtype=torch.uint8, device="cuda")
    res = []
    for rope in (False, True):
        dev = {k: to_dev(v) for k, v in st.items()}
        if rope:
            o1 = loma.loma_compress_step_rope(qm, km, vm, dev["k_read"], dev["v_read"], dev["k_mem"], dev["v_mem"], 16, 4, 6,
                                              cfg.scale, 0, 0)
            o2 = loma.loma_decode_attn_rope(q, kn, vn, dev["k_mem"], dev["v_mem"], dev["k_read"], dev["v_read"], 16, 4, 7, 0,
                                            cfg.scale, 0, workspace=ws)
        else:
            o1 = loma.loma_compress_step(qm, km, vm, dev["k_read"], dev["v_read"], dev["k_mem"], dev["v_mem"], 16, 4, 6, cfg.scale)
            o2 = loma.loma_decode_attn(q, kn, vn, dev["k_mem"], dev["v_mem"], dev["k_read"], dev["v_read"], 16, 4, 7, 0,
                                       cfg.scale, workspace=ws)
        torch.cuda.synchronize()
        res.append((o1, o2, dev["k_mem"], dev["v_mem"], dev["k_read"], dev["v_read"]))
    for a, b in zip(*res):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
