"""Host-side checks of the C ABI: exported symbols, argument validation, tile schedule.

No kernel is launched here: every call below is rejected by the host-side checks (or is
host-only arithmetic), so the tests run without a GPU.
"""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "loma.h")
LIB = os.path.join(ROOT, "paper_2401_09486_amd", "libloma.so")

pytestmark = pytest.mark.skipif(not os.path.exists(LIB), reason="libloma.so not built (python -m paper_2401_09486_amd.build)")

OK, EINVAL, EUNSUP, EWS, ELAUNCH = 0, -1, -2, -3, -4
F32, BF16 = 0, 1
P = 0x10000  # a non-null, 16-byte aligned fake device address; never dereferenced on the host


@pytest.fixture(scope="module")
def lib():
    from paper_2401_09486_amd import loma
    return loma.lib


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(loma_[a-z_0-9]+)\s*\(", src)))


def test_every_declared_symbol_is_exported():
    names = declared_functions()
    assert {"loma_mask_attn_fwd", "loma_compress_step", "loma_decode_attn",
            "loma_decode_workspace_bytes", "loma_status_string"} <= set(names)
    raw = ctypes.CDLL(LIB)
    for n in names:
        assert hasattr(raw, n), f"{n} declared in loma.h but not exported"


def test_status_strings(lib):
    from paper_2401_09486_amd import loma
    assert loma.status_string(OK) == "ok"
    for code in (EINVAL, EUNSUP, EWS, ELAUNCH, -99):
        assert loma.status_string(code)
    assert loma.abi_version() >= 1


def mask_call(lib, **kw):
    a = dict(q=P, k=P, v=P, out=P, lse=None, B=1, H=1, d=128, t=16, c=4, n=2, scale=0.1, dtype=BF16)
    a.update(kw)
    return lib.loma_mask_attn_fwd(a["q"], a["k"], a["v"], a["out"], a["lse"], a["B"], a["H"], a["d"], a["t"], a["c"],
                                  a["n"], a["scale"], a["dtype"], None)


def test_mask_attn_rejects_bad_arguments(lib):
    assert mask_call(lib, q=None) == EINVAL
    assert mask_call(lib, out=None) == EINVAL
    assert mask_call(lib, k=P + 2) == EINVAL          # misaligned
    assert mask_call(lib, t=0) == EINVAL
    assert mask_call(lib, c=-1) == EINVAL
    assert mask_call(lib, n=0) == EINVAL
    assert mask_call(lib, B=0) == EINVAL
    assert mask_call(lib, scale=0.0) == EINVAL
    assert mask_call(lib, scale=float("nan")) == EINVAL
    assert mask_call(lib, scale=float("inf")) == EINVAL
    assert mask_call(lib, dtype=7) == EUNSUP
    assert mask_call(lib, d=100) == EUNSUP            # not a multiple of 8
    assert mask_call(lib, d=512) == EUNSUP
    assert mask_call(lib, n=1 << 28) == EUNSUP        # sequence too long


def compress_call(lib, **kw):
    a = dict(qm=P, km=P, vm=P, kr=P, vr=P, kc=P, vc=P, out=P, B=1, H=1, d=128, t=16, c=4, nmem=2, cap=64,
             scale=0.1, dtype=BF16)
    a.update(kw)
    return lib.loma_compress_step(a["qm"], a["km"], a["vm"], a["kr"], a["vr"], a["kc"], a["vc"], a["out"], a["B"],
                                  a["H"], a["d"], a["t"], a["c"], a["nmem"], a["cap"], a["scale"], a["dtype"], None)


def test_compress_rejects_bad_arguments(lib):
    assert compress_call(lib, kc=None) == EINVAL
    assert compress_call(lib, vr=P + 8) == EINVAL
    assert compress_call(lib, nmem=-1) == EINVAL
    assert compress_call(lib, nmem=4, cap=64) == EINVAL    # (4+1)*16 > 64: cache full
    assert compress_call(lib, nmem=3, cap=63) == EINVAL
    assert compress_call(lib, t=0) == EINVAL
    assert compress_call(lib, dtype=2) == EUNSUP
    assert compress_call(lib, d=4) == EUNSUP


def decode_call(lib, **kw):
    a = dict(q=P, kn=P, vn=P, kc=P, vc=P, kr=P, vr=P, out=P, B=8, H=32, d=128, t=16, c=4, nmem=4, cap=64, fill=3,
             scale=0.1, dtype=BF16, ws=P, wsb=1 << 30)
    a.update(kw)
    return lib.loma_decode_attn(a["q"], a["kn"], a["vn"], a["kc"], a["vc"], a["kr"], a["vr"], a["out"], a["B"], a["H"],
                                a["d"], a["t"], a["c"], a["nmem"], a["cap"], a["fill"], a["scale"], a["dtype"],
                                a["ws"], a["wsb"], None)


def test_decode_rejects_bad_arguments(lib):
    assert decode_call(lib, q=None) == EINVAL
    assert decode_call(lib, kn=None) == EINVAL                    # k_new without v_new
    assert decode_call(lib, fill=64) == EINVAL                    # reading zone full, token cannot be appended
    assert decode_call(lib, fill=65, kn=None, vn=None) == EINVAL  # longer than t*c
    assert decode_call(lib, fill=-1) == EINVAL
    assert decode_call(lib, nmem=5) == EINVAL                     # 80 memory rows > capacity 64
    assert decode_call(lib, kc=None) == EINVAL                    # memory rows but no cache
    assert decode_call(lib, nmem=0, fill=0, kn=None, vn=None) == EINVAL   # nothing to attend to
    assert decode_call(lib, kr=P + 4) == EINVAL
    assert decode_call(lib, dtype=-1) == EUNSUP
    # split-K (few (b,h) pairs) needs its workspace
    need = lib.loma_decode_workspace_bytes(1, 8, 128, 16, 4, 4, BF16)
    assert need > 0
    assert decode_call(lib, B=1, H=8, ws=None) == EWS
    assert decode_call(lib, B=1, H=8, wsb=need - 1) == EWS


def test_prefill_rejects_bad_arguments(lib):
    def call(q=P, kn=P, vn=P, km=P, vm=P, kr=P, vr=P, out=P, lse=None, B=2, H=4, d=128, t=16, c=4, nm=3, cap=64, fill=10,
             n_new=20, scale=0.1, dtype=BF16):
        return lib.loma_prefill_attn(q, kn, vn, km, vm, kr, vr, out, lse, B, H, d, t, c, nm, cap, fill, n_new, scale, dtype, None)
    assert call(n_new=0) == EINVAL
    assert call(fill=50, n_new=15) == EINVAL            # 65 > t*c = 64
    assert call(fill=-1) == EINVAL
    assert call(nm=5, cap=64) == EINVAL                 # 80 memory rows do not fit the cache
    assert call(kn=None) == EINVAL and call(vn=None) == EINVAL
    assert call(q=P + 8) == EINVAL                      # misaligned
    assert call(km=None) == EINVAL and call(vm=None) == EINVAL
    assert call(lse=P + 2) == EINVAL
    assert call(d=100) == EUNSUP and call(dtype=7) == EUNSUP
    assert call(scale=0.0) == EINVAL


def test_mask_bwd_rejects_bad_arguments(lib):
    # distinct fake addresses: the outputs may not alias an input or each other
    A = [P + 0x1000 * i for i in range(9)]

    def call(q=A[0], k=A[1], v=A[2], out=A[3], lse=A[4], dout=A[5], dq=A[6], dk=A[7], dv=A[8], B=1, H=2, d=128, t=16,
             c=4, n=2, scale=0.1, dtype=BF16, ws=P, wsb=0):
        return lib.loma_mask_attn_bwd(q, k, v, out, lse, dout, dq, dk, dv, B, H, d, t, c, n, scale, dtype, ws, wsb, None)
    need = lib.loma_mask_attn_bwd_workspace_bytes(1, 2, 128, 16, 4, 2, BF16)
    assert need == 2 * 4 * 2 * 2 * 16 * 9            # two floats per row
    # every call below keeps the workspace too small, so even a call with good pointers stops at the host
    assert call(wsb=need - 1) == EWS
    assert call(ws=None, wsb=need) == EWS
    assert call(lse=None, wsb=need) == EINVAL
    assert call(dout=None, wsb=need) == EINVAL
    assert call(dq=A[0], wsb=need) == EINVAL            # aliases q
    assert call(dk=A[8], wsb=need) == EINVAL            # aliases dv
    assert call(dv=A[5], wsb=need) == EINVAL            # aliases dout
    assert call(k=A[1] + 2, wsb=need) == EINVAL
    assert call(n=0, wsb=need) == EINVAL
    assert call(scale=-1.0, wsb=need) == EINVAL
    assert call(d=100, wsb=need) == EUNSUP and call(dtype=3, wsb=need) == EUNSUP
    # the Llama-shaped training configuration shares its memory-key streams out over two workgroups and needs room
    # for their fp32 partial sums; the long-context one is balanced without and needs the two floats per row only
    rows2, rows4 = 2 * 32 * 28 * 16 * 9, 32 * 60 * 32 * 17
    assert lib.loma_mask_attn_bwd_workspace_bytes(2, 32, 128, 16, 4, 28, BF16) == 8 * rows2 + 4 * (64 * 2 * 2 * 28 * 16 * 128)
    assert lib.loma_mask_attn_bwd_workspace_bytes(1, 32, 128, 32, 8, 60, BF16) == 8 * rows4
    assert lib.loma_mask_attn_bwd_workspace_bytes(2, 32, 128, 16, 4, 28, F32) == 8 * rows2     # generic kernels
    assert lib.loma_mask_attn_bwd_workspace_bytes(1, 2, 128, 16, 4, 0, BF16) == 0
    assert lib.loma_mask_attn_bwd_workspace_bytes(1, 2, 100, 16, 4, 2, BF16) == 0


def test_decode_workspace_bytes(lib):
    f = lib.loma_decode_workspace_bytes
    assert f(0, 32, 128, 16, 4, 4, BF16) == 0
    assert f(8, 32, 100, 16, 4, 4, BF16) == 0
    assert f(8, 32, 128, 16, 4, -1, BF16) == 0
    a = f(1, 32, 128, 16, 4, 64, BF16)
    assert a > 0 and a % 4 == 0
    # one workgroup per (b,h) already fills the chip: no split, no workspace
    assert f(8, 32, 128, 16, 4, 64, BF16) == 0
    assert f(64, 64, 128, 16, 16, 512, BF16) == 0


@pytest.mark.parametrize("B,H,d,t,c,n", [(1, 1, 128, 16, 4, 3), (2, 4, 128, 32, 8, 5), (1, 3, 64, 4, 4, 4),
                                         (1, 2, 128, 5, 7, 3), (1, 8, 128, 48, 3, 2), (1, 1, 128, 200, 1, 2)])
def test_mask_schedule_covers_every_row_once(B, H, d, t, c, n):
    from paper_2401_09486_amd import loma
    import torch
    items = loma.mask_schedule(B, H, d, t, c, n, torch.bfloat16)
    R = t * c
    nbh = B * H
    seen = {}
    for blk, (bh, y, zone, o0, rows, keys) in enumerate(items):
        if nbh % 8 == 0:
            assert bh % 8 == blk % 8                # a (b,h) stays on one XCD (workgroups go round-robin over 8)
        assert 0 <= bh < nbh and 0 <= y < n and zone in (0, 1, 2) and rows >= 1
        zlen = t if zone == 1 else R
        assert 0 <= o0 and o0 + rows <= zlen
        if zone == 0:
            assert keys == y * t + o0 + rows        # earlier memory zones + causal prefix up to the last row
        elif zone == 1:
            assert keys == R + t
        else:
            assert keys == t
        for r in range(o0, o0 + rows):
            key = (bh, y, zone, r)
            assert key not in seen
            seen[key] = blk
    assert len(seen) == nbh * n * (2 * R + t)
    # longest first: a (b,h) runs from its last chunk (most earlier memory zones) to its first
    chunks = [y for (bh, y, z, o0, rows, k) in items if bh == 0]
    assert chunks == sorted(chunks, reverse=True)


def test_schedule_size_zero_for_shapes_on_the_generic_path(lib):
    assert lib.loma_mask_schedule_size(1, 1, 64, 4, 4, 4, F32) == 0
    assert lib.loma_mask_schedule_size(1, 1, 96, 4, 4, 4, BF16) == 0
    assert lib.loma_mask_schedule_size(2, 32, 128, 16, 4, 28, BF16) == 2 * 32 * 28 * 3


def test_mask_pass_dispatch_respects_the_division_bound(lib):
    """The MFMA kernels divide a memory-key index by t with a multiply-high that is exact while
    (n_chunks - 1) * t * t < 2^32; a longer sample must not take them (it takes the generic kernels)."""
    assert lib.loma_mask_schedule_size(1, 1, 128, 4096, 1, 256, BF16) > 0     # 255 * 4096^2 < 2^32
    assert lib.loma_mask_schedule_size(1, 1, 128, 4096, 1, 258, BF16) == 0    # 257 * 4096^2 >= 2^32, S = 3.2M still allowed


def test_new_decode_forms_reject_bad_arguments(lib):
    # static-scratch form: same state checks as loma_decode_attn, and a size limit instead of a workspace check
    def static_call(**kw):
        a = dict(q=P, kn=P, vn=P, kc=P, vc=P, kr=P, vr=P, out=P, B=1, H=8, d=128, t=16, c=4, nmem=4, cap=64, fill=3,
                 scale=0.1, dtype=BF16)
        a.update(kw)
        return lib.loma_decode_attn_static(a["q"], a["kn"], a["vn"], a["kc"], a["vc"], a["kr"], a["vr"], a["out"], a["B"],
                                           a["H"], a["d"], a["t"], a["c"], a["nmem"], a["cap"], a["fill"], a["scale"],
                                           a["dtype"], None)
    assert static_call(q=None) == EINVAL
    assert static_call(fill=64) == EINVAL
    assert static_call(nmem=5) == EINVAL
    assert static_call(dtype=9) == EUNSUP
    assert lib.loma_decode_static_scratch_bytes() == 4 << 20
    # 4095 pairs x 2 splits x 130 floats do not fit the fixed array
    assert lib.loma_decode_workspace_bytes(4095, 1, 128, 16, 4, 4, BF16) > lib.loma_decode_static_scratch_bytes()
    assert static_call(B=4095, H=1) == EUNSUP

    def layers_call(**kw):
        a = dict(q=P, kn=P, vn=P, kc=P, vc=P, kr=P, vr=P, out=P, L=4, B=1, H=8, d=128, t=16, c=4, nmem=4, cap=64,
                 fill=3, scale=0.1, dtype=BF16, ws=P, wsb=1 << 30)
        a.update(kw)
        return lib.loma_decode_attn_layers(a["q"], a["kn"], a["vn"], a["kc"], a["vc"], a["kr"], a["vr"], a["out"], a["L"],
                                           a["B"], a["H"], a["d"], a["t"], a["c"], a["nmem"], a["cap"], a["fill"],
                                           a["scale"], a["dtype"], a["ws"], a["wsb"], None)
    assert layers_call(L=0) == EINVAL
    assert layers_call(q=None) == EINVAL
    assert layers_call(kr=P + 4) == EINVAL            # a pointer table must be 8-byte aligned
    assert layers_call(kn=None) == EINVAL             # k_new without v_new
    assert layers_call(kc=None) == EINVAL             # memory rows but no cache table
    assert layers_call(fill=64) == EINVAL
    assert layers_call(dtype=F32) == EUNSUP
    assert layers_call(d=96) == EUNSUP
    need = lib.loma_decode_layers_workspace_bytes(4, 1, 8, 128, 16, 4, 4, BF16)
    assert need == 4 * lib.loma_decode_workspace_bytes(1, 8, 128, 16, 4, 4, BF16) > 0
    assert layers_call(ws=None) == EWS
    assert layers_call(wsb=need - 1) == EWS


def test_grouped_query_decode_rejects_bad_arguments(lib):
    def call(**kw):
        a = dict(q=P, kn=P, vn=P, kc=P, vc=P, kr=P, vr=P, out=P, B=1, H=8, Hkv=2, d=128, t=16, c=4, nmem=4, cap=64,
                 fill=3, scale=0.1, dtype=BF16, ws=P, wsb=1 << 30)
        a.update(kw)
        return lib.loma_decode_attn_gqa(a["q"], a["kn"], a["vn"], a["kc"], a["vc"], a["kr"], a["vr"], a["out"], a["B"],
                                        a["H"], a["Hkv"], a["d"], a["t"], a["c"], a["nmem"], a["cap"], a["fill"],
                                        a["scale"], a["dtype"], a["ws"], a["wsb"], None)
    assert call(q=None) == EINVAL
    assert call(Hkv=3) == EINVAL                  # query heads not a multiple of the KV heads
    assert call(Hkv=0) == EINVAL
    assert call(H=6) == EUNSUP                    # three query heads per KV head
    assert call(H=32, Hkv=2) == EUNSUP            # sixteen
    assert call(kn=None) == EINVAL                # k_new without v_new
    assert call(kc=None) == EINVAL                # memory rows but no cache
    assert call(fill=64) == EINVAL
    assert call(nmem=5) == EINVAL
    assert call(dtype=F32) == EUNSUP
    assert call(d=96) == EUNSUP
    need = lib.loma_decode_gqa_workspace_bytes(1, 8, 2, 128, BF16)
    # partial results per QUERY head: four times what the two KV heads alone would need at the same split plan
    assert need > 0 and need % (8 * 130 * 4) == 0
    assert call(ws=None) == EWS
    assert call(wsb=need - 1) == EWS
    assert lib.loma_decode_gqa_workspace_bytes(1, 8, 3, 128, BF16) == 0
    assert lib.loma_decode_gqa_workspace_bytes(1, 8, 2, 128, F32) == 0


def test_layered_grouped_query_decode_rejects_bad_arguments(lib):
    def call(**kw):
        a = dict(q=P, kn=P, vn=P, kc=P, vc=P, kr=P, vr=P, out=P, L=3, B=1, H=8, Hkv=2, d=128, t=16, c=4, nmem=4, cap=64,
                 fill=3, scale=0.1, dtype=BF16, ws=P, wsb=1 << 30)
        a.update(kw)
        return lib.loma_decode_attn_gqa_layers(a["q"], a["kn"], a["vn"], a["kc"], a["vc"], a["kr"], a["vr"], a["out"], a["L"],
                                               a["B"], a["H"], a["Hkv"], a["d"], a["t"], a["c"], a["nmem"], a["cap"],
                                               a["fill"], a["scale"], a["dtype"], a["ws"], a["wsb"], None)
    assert call(L=0) == EINVAL
    assert call(out=None) == EINVAL
    assert call(kr=P + 4) == EINVAL               # a pointer table must be 8-byte aligned
    assert call(Hkv=3) == EINVAL
    assert call(H=6) == EUNSUP
    assert call(vn=None) == EINVAL                # k_new without v_new
    assert call(fill=64) == EINVAL
    assert call(dtype=F32) == EUNSUP
    need = 3 * lib.loma_decode_gqa_workspace_bytes(1, 8, 2, 128, BF16)
    assert call(ws=None) == EWS
    assert call(wsb=need - 1) == EWS
