"""Thin Python binding over libloma.so (include/loma.h): argument marshalling only.

Every function takes torch tensors that already live on the GPU (PyTorch is used for
device memory and streams, nothing else), checks shapes and dtypes, and passes raw
pointers to the C ABI.  All arithmetic runs in the HIP kernels.  If the shared library
is missing the import fails: there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libloma.so")

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_LAUNCH = 0, -1, -2, -3, -4
F32, BF16 = 0, 1
POS_INTERMITTENT, POS_CONTIGUOUS = 0, 1


class LomaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} not found: build it with `python -m paper_2401_09486_amd.build` "
            "(the HIP library is the only implementation; there is no fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, I, F, Z, LL = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t, ctypes.c_longlong
    lib.loma_status_string.argtypes = [I]
    lib.loma_status_string.restype = ctypes.c_char_p
    lib.loma_abi_version.argtypes = []
    lib.loma_abi_version.restype = I
    lib.loma_mask_attn_fwd.argtypes = [vp, vp, vp, vp, vp, I, I, I, I, I, I, F, I, vp]
    lib.loma_mask_attn_fwd.restype = I
    lib.loma_mask_attn_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, I, I, I, I, I, I, F, I, vp, Z, vp]
    lib.loma_mask_attn_bwd.restype = I
    lib.loma_mask_attn_bwd_workspace_bytes.argtypes = [I, I, I, I, I, I, I]
    lib.loma_mask_attn_bwd_workspace_bytes.restype = Z
    lib.loma_compress_step.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, I, I, I, I, I, I, I, F, I, vp]
    lib.loma_compress_step.restype = I
    lib.loma_decode_attn.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, I, I, I, I, I, I, I, I, F, I, vp, Z, vp]
    lib.loma_decode_attn.restype = I
    lib.loma_decode_attn_static.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, I, I, I, I, I, I, I, I, F, I, vp]
    lib.loma_decode_attn_static.restype = I
    lib.loma_decode_static_scratch_bytes.argtypes = []
    lib.loma_decode_static_scratch_bytes.restype = Z
    lib.loma_decode_attn_layers.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, I, I, I, I, I, I, I, I, I, F, I, vp, Z, vp]
    lib.loma_decode_attn_layers.restype = I
    lib.loma_decode_layers_workspace_bytes.argtypes = [I, I, I, I, I, I, I, I]
    lib.loma_decode_layers_workspace_bytes.restype = Z
    lib.loma_decode_attn_gqa.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, I, I, I, I, I, I, I, I, I, F, I, vp, Z, vp]
    lib.loma_decode_attn_gqa.restype = I
    lib.loma_decode_attn_gqa_layers.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, I, I, I, I, I, I, I, I, I, I, F, I, vp, Z, vp]
    lib.loma_decode_attn_gqa_layers.restype = I
    lib.loma_decode_gqa_workspace_bytes.argtypes = [I, I, I, I, I]
    lib.loma_decode_gqa_workspace_bytes.restype = Z
    lib.loma_decode_attn_rope.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, I, I, I, I, I, I, I, I, F, I, I, F, vp, Z, vp]
    lib.loma_decode_attn_rope.restype = I
    lib.loma_compress_step_rope.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, I, I, I, I, I, I, I, F, I, I, I, F, vp]
    lib.loma_compress_step_rope.restype = I
    lib.loma_memory_position_ids.argtypes = [I, I, I, I, ctypes.POINTER(I)]
    lib.loma_memory_position_ids.restype = I
    lib.loma_sample_position_ids.argtypes = [I, I, I, I, ctypes.POINTER(I)]
    lib.loma_sample_position_ids.restype = I
    lib.loma_prefill_attn.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, I, I, I, I, I, I, I, I, I, F, I, vp]
    lib.loma_prefill_attn.restype = I
    lib.loma_decode_workspace_bytes.argtypes = [I, I, I, I, I, I, I]
    lib.loma_decode_workspace_bytes.restype = Z
    lib.loma_mask_schedule_size.argtypes = [I, I, I, I, I, I, I]
    lib.loma_mask_schedule_size.restype = LL
    lib.loma_mask_schedule_item.argtypes = [I, I, I, I, I, I, I, LL, ctypes.POINTER(I * 6)]
    lib.loma_mask_schedule_item.restype = I
    return lib


lib = _load()


def status_string(status: int) -> str:
    return lib.loma_status_string(int(status)).decode()


def abi_version() -> int:
    return int(lib.loma_abi_version())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def _dev(t, name, shape=None, dtype=None):
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a GPU tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} has shape {tuple(t.shape)}, expected {tuple(shape)}")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} has dtype {t.dtype}, expected {dtype}")
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def loma_mask_attn_fwd(q, k, v, t, c, n_chunks, scale, out=None, lse=None, stream=None):
    """Training / compression-pass form.  q, k, v: [B, H, n_chunks*t*(2c+1), d].  Returns out."""
    B, H, S, d = q.shape
    if out is None:
        out = torch.empty_like(q)
    pq = _dev(q, "q")
    pk, pv = _dev(k, "k", q.shape, q.dtype), _dev(v, "v", q.shape, q.dtype)
    po = _dev(out, "out", q.shape, q.dtype)
    pl = None if lse is None else _dev(lse, "lse", (B, H, S), torch.float32)
    if S != n_chunks * t * (2 * c + 1):
        raise ValueError("sequence length must be n_chunks * t * (2c + 1)")
    rc = lib.loma_mask_attn_fwd(pq, pk, pv, po, pl, B, H, d, t, c, n_chunks, float(scale), _dtype_code(q),
                                _stream(stream))
    if rc != OK:
        raise LomaError(rc, "loma_mask_attn_fwd")
    return out


def loma_mask_attn_bwd_workspace_bytes(B, H, d, t, c, n_chunks, dtype=torch.bfloat16) -> int:
    code = F32 if dtype == torch.float32 else BF16
    return int(lib.loma_mask_attn_bwd_workspace_bytes(B, H, d, t, c, n_chunks, code))


def loma_mask_attn_bwd(q, k, v, out, lse, dout, t, c, n_chunks, scale, dq=None, dk=None, dv=None, workspace=None,
                       stream=None):
    """Gradients of the training form for the upstream gradient dout; out and lse come from
    loma_mask_attn_fwd on the same inputs.  Returns (dq, dk, dv)."""
    B, H, S, d = q.shape
    if S != n_chunks * t * (2 * c + 1):
        raise ValueError("sequence length must be n_chunks * t * (2c + 1)")
    dt = q.dtype
    dq = torch.empty_like(q) if dq is None else dq
    dk = torch.empty_like(q) if dk is None else dk
    dv = torch.empty_like(q) if dv is None else dv
    if workspace is None:
        need = loma_mask_attn_bwd_workspace_bytes(B, H, d, t, c, n_chunks, dt)
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    ptrs = [_dev(q, "q")] + [_dev(x, n, q.shape, dt) for x, n in ((k, "k"), (v, "v"), (out, "out"))]
    ptrs.append(_dev(lse, "lse", (B, H, S), torch.float32))
    ptrs += [_dev(x, n, q.shape, dt) for x, n in ((dout, "dout"), (dq, "dq"), (dk, "dk"), (dv, "dv"))]
    rc = lib.loma_mask_attn_bwd(*ptrs, B, H, d, t, c, n_chunks, float(scale), _dtype_code(q),
                                _dev(workspace, "workspace"), workspace.numel() * workspace.element_size(),
                                _stream(stream))
    if rc != OK:
        raise LomaError(rc, "loma_mask_attn_bwd")
    return dq, dk, dv


def loma_compress_step(q_mem, k_mem, v_mem, k_read, v_read, k_memcache, v_memcache, t, c, n_mem_chunks, scale,
                       out=None, stream=None):
    """Compression boundary: t <m> queries over [reading zone || own K/V], then splice into the cache."""
    B, H, tt, d = q_mem.shape
    if tt != t:
        raise ValueError("q_mem must have t rows")
    if out is None:
        out = torch.empty_like(q_mem)
    dt = q_mem.dtype
    cap = k_memcache.shape[2]
    args = [_dev(q_mem, "q_mem"), _dev(k_mem, "k_mem", q_mem.shape, dt), _dev(v_mem, "v_mem", q_mem.shape, dt),
            _dev(k_read, "k_read", (B, H, t * c, d), dt), _dev(v_read, "v_read", (B, H, t * c, d), dt),
            _dev(k_memcache, "k_memcache", (B, H, cap, d), dt), _dev(v_memcache, "v_memcache", (B, H, cap, d), dt),
            _dev(out, "out", q_mem.shape, dt)]
    rc = lib.loma_compress_step(*args, B, H, d, t, c, n_mem_chunks, cap, float(scale), _dtype_code(q_mem),
                                _stream(stream))
    if rc != OK:
        raise LomaError(rc, "loma_compress_step")
    return out


def loma_compress_step_rope(q_mem, k_mem, v_mem, k_read, v_read, k_memcache, v_memcache, t, c, n_mem_chunks, scale,
                            pos_first, pos_stride, rope_theta=10000.0, out=None, stream=None):
    """loma_compress_step with q_mem and k_mem rotated on load by the ids pos_first + j * pos_stride."""
    B, H, tt, d = q_mem.shape
    if tt != t:
        raise ValueError("q_mem must have t rows")
    if out is None:
        out = torch.empty_like(q_mem)
    dt = q_mem.dtype
    cap = k_memcache.shape[2]
    args = [_dev(q_mem, "q_mem"), _dev(k_mem, "k_mem", q_mem.shape, dt), _dev(v_mem, "v_mem", q_mem.shape, dt),
            _dev(k_read, "k_read", (B, H, t * c, d), dt), _dev(v_read, "v_read", (B, H, t * c, d), dt),
            _dev(k_memcache, "k_memcache", (B, H, cap, d), dt), _dev(v_memcache, "v_memcache", (B, H, cap, d), dt),
            _dev(out, "out", q_mem.shape, dt)]
    rc = lib.loma_compress_step_rope(*args, B, H, d, t, c, n_mem_chunks, cap, float(scale), _dtype_code(q_mem),
                                     int(pos_first), int(pos_stride), float(rope_theta), _stream(stream))
    if rc != OK:
        raise LomaError(rc, "loma_compress_step_rope")
    return out


def memory_position_ids(t, c, chunk, position_type=POS_INTERMITTENT):
    """Ids of the t memory tokens of chunk `chunk` (host list)."""
    buf = (ctypes.c_int * t)()
    rc = lib.loma_memory_position_ids(t, c, chunk, position_type, buf)
    if rc != OK:
        raise LomaError(rc, "loma_memory_position_ids")
    return list(buf)


def sample_position_ids(t, c, n_chunks, position_type=POS_INTERMITTENT):
    """Ids of every row of a restructured sample (host list of n_chunks * t * (2c + 1) ints)."""
    n = n_chunks * t * (2 * c + 1)
    buf = (ctypes.c_int * n)()
    rc = lib.loma_sample_position_ids(t, c, n_chunks, position_type, buf)
    if rc != OK:
        raise LomaError(rc, "loma_sample_position_ids")
    return list(buf)


def loma_decode_workspace_bytes(B, H, d, t, c, n_mem_chunks, dtype=torch.bfloat16) -> int:
    code = F32 if dtype == torch.float32 else BF16
    return int(lib.loma_decode_workspace_bytes(B, H, d, t, c, n_mem_chunks, code))


def loma_decode_attn(q, k_new, v_new, k_memcache, v_memcache, k_read, v_read, t, c, n_mem_chunks, read_fill, scale,
                     out=None, workspace=None, stream=None):
    """One new token per sequence against [memory cache || reading zone (|| new token)]."""
    B, H, one, d = q.shape
    if one != 1:
        raise ValueError("q must be [B, H, 1, d]")
    if out is None:
        out = torch.empty_like(q)
    dt = q.dtype
    pkn = None if k_new is None else _dev(k_new, "k_new", q.shape, dt)
    pvn = None if v_new is None else _dev(v_new, "v_new", q.shape, dt)
    cap = 0 if k_memcache is None else k_memcache.shape[2]
    pkm = None if k_memcache is None else _dev(k_memcache, "k_memcache", (B, H, cap, d), dt)
    pvm = None if v_memcache is None else _dev(v_memcache, "v_memcache", (B, H, cap, d), dt)
    pkr = _dev(k_read, "k_read", (B, H, t * c, d), dt)
    pvr = _dev(v_read, "v_read", (B, H, t * c, d), dt)
    pws, nws = None, 0
    if workspace is not None:
        pws, nws = _dev(workspace, "workspace"), workspace.numel() * workspace.element_size()
    rc = lib.loma_decode_attn(_dev(q, "q"), pkn, pvn, pkm, pvm, pkr, pvr, _dev(out, "out", q.shape, dt),
                              B, H, d, t, c, n_mem_chunks, cap, read_fill, float(scale), _dtype_code(q),
                              pws, nws, _stream(stream))
    if rc != OK:
        raise LomaError(rc, "loma_decode_attn")
    return out


def loma_decode_gqa_workspace_bytes(B, H, H_kv, d, dtype=torch.bfloat16) -> int:
    code = F32 if dtype == torch.float32 else BF16
    return int(lib.loma_decode_gqa_workspace_bytes(B, H, H_kv, d, code))


def loma_decode_attn_gqa(q, k_new, v_new, k_memcache, v_memcache, k_read, v_read, t, c, n_mem_chunks, read_fill, scale,
                         out=None, workspace=None, stream=None):
    """loma_decode_attn with H query heads (q, out: [B, H, 1, d]) over H_kv shared key/value heads (every other
    tensor: [B, H_kv, ...]); query head h reads KV head h // (H // H_kv)."""
    B, H, one, d = q.shape
    if one != 1:
        raise ValueError("q must be [B, H, 1, d]")
    H_kv = k_read.shape[1]
    if out is None:
        out = torch.empty_like(q)
    dt = q.dtype
    pkn = None if k_new is None else _dev(k_new, "k_new", (B, H_kv, 1, d), dt)
    pvn = None if v_new is None else _dev(v_new, "v_new", (B, H_kv, 1, d), dt)
    cap = 0 if k_memcache is None else k_memcache.shape[2]
    pkm = None if k_memcache is None else _dev(k_memcache, "k_memcache", (B, H_kv, cap, d), dt)
    pvm = None if v_memcache is None else _dev(v_memcache, "v_memcache", (B, H_kv, cap, d), dt)
    pkr = _dev(k_read, "k_read", (B, H_kv, t * c, d), dt)
    pvr = _dev(v_read, "v_read", (B, H_kv, t * c, d), dt)
    pws, nws = None, 0
    if workspace is not None:
        pws, nws = _dev(workspace, "workspace"), workspace.numel() * workspace.element_size()
    rc = lib.loma_decode_attn_gqa(_dev(q, "q"), pkn, pvn, pkm, pvm, pkr, pvr, _dev(out, "out", q.shape, dt),
                                  B, H, H_kv, d, t, c, n_mem_chunks, cap, read_fill, float(scale), _dtype_code(q),
                                  pws, nws, _stream(stream))
    if rc != OK:
        raise LomaError(rc, "loma_decode_attn_gqa")
    return out


def loma_decode_attn_rope(q, k_new, v_new, k_memcache, v_memcache, k_read, v_read, t, c, n_mem_chunks, read_fill, scale,
                          pos, rope_theta=10000.0, out=None, workspace=None, stream=None):
    """loma_decode_attn with q and k_new rotated on load by the new token's position id `pos`."""
    B, H, one, d = q.shape
    if one != 1:
        raise ValueError("q must be [B, H, 1, d]")
    if out is None:
        out = torch.empty_like(q)
    dt = q.dtype
    pkn = None if k_new is None else _dev(k_new, "k_new", q.shape, dt)
    pvn = None if v_new is None else _dev(v_new, "v_new", q.shape, dt)
    cap = 0 if k_memcache is None else k_memcache.shape[2]
    pkm = None if k_memcache is None else _dev(k_memcache, "k_memcache", (B, H, cap, d), dt)
    pvm = None if v_memcache is None else _dev(v_memcache, "v_memcache", (B, H, cap, d), dt)
    pws, nws = None, 0
    if workspace is not None:
        pws, nws = _dev(workspace, "workspace"), workspace.numel() * workspace.element_size()
    rc = lib.loma_decode_attn_rope(_dev(q, "q"), pkn, pvn, pkm, pvm, _dev(k_read, "k_read", (B, H, t * c, d), dt),
                                   _dev(v_read, "v_read", (B, H, t * c, d), dt), _dev(out, "out", q.shape, dt),
                                   B, H, d, t, c, n_mem_chunks, cap, read_fill, float(scale), _dtype_code(q),
                                   int(pos), float(rope_theta), pws, nws, _stream(stream))
    if rc != OK:
        raise LomaError(rc, "loma_decode_attn_rope")
    return out


def loma_decode_attn_static(q, k_new, v_new, k_memcache, v_memcache, k_read, v_read, t, c, n_mem_chunks, read_fill, scale,
                            out=None, stream=None):
    """loma_decode_attn without a workspace: the split-K partials live in a fixed array inside the library."""
    B, H, one, d = q.shape
    if one != 1:
        raise ValueError("q must be [B, H, 1, d]")
    if out is None:
        out = torch.empty_like(q)
    dt = q.dtype
    pkn = None if k_new is None else _dev(k_new, "k_new", q.shape, dt)
    pvn = None if v_new is None else _dev(v_new, "v_new", q.shape, dt)
    cap = 0 if k_memcache is None else k_memcache.shape[2]
    pkm = None if k_memcache is None else _dev(k_memcache, "k_memcache", (B, H, cap, d), dt)
    pvm = None if v_memcache is None else _dev(v_memcache, "v_memcache", (B, H, cap, d), dt)
    rc = lib.loma_decode_attn_static(_dev(q, "q"), pkn, pvn, pkm, pvm, _dev(k_read, "k_read", (B, H, t * c, d), dt),
                                     _dev(v_read, "v_read", (B, H, t * c, d), dt), _dev(out, "out", q.shape, dt),
                                     B, H, d, t, c, n_mem_chunks, cap, read_fill, float(scale), _dtype_code(q),
                                     _stream(stream))
    if rc != OK:
        raise LomaError(rc, "loma_decode_attn_static")
    return out


def decode_static_scratch_bytes() -> int:
    return int(lib.loma_decode_static_scratch_bytes())


def pointer_table(tensors) -> torch.Tensor:
    """Device array of the tensors' device addresses (what the layered entry points take per argument)."""
    for x in tensors:
        if not x.is_cuda or not x.is_contiguous():
            raise ValueError("layer tensors must be contiguous GPU tensors")
    return torch.tensor([x.data_ptr() for x in tensors], dtype=torch.int64, device=tensors[0].device)


def loma_decode_layers_workspace_bytes(n_layers, B, H, d, t, c, n_mem_chunks, dtype=torch.bfloat16) -> int:
    code = F32 if dtype == torch.float32 else BF16
    return int(lib.loma_decode_layers_workspace_bytes(n_layers, B, H, d, t, c, n_mem_chunks, code))


def loma_decode_attn_layers(q, k_new, v_new, k_memcache, v_memcache, k_read, v_read, out, n_layers, B, H, d, t, c,
                            n_mem_chunks, mem_capacity, read_fill, scale, dtype=torch.bfloat16, workspace=None,
                            stream=None):
    """One decode step on n_layers caches in one launch.  The first eight arguments are pointer tables
    (pointer_table(list of that argument's per-layer tensors), or None where loma_decode_attn allows it)."""
    tabs = []
    for name, tab in (("q", q), ("k_new", k_new), ("v_new", v_new), ("k_memcache", k_memcache),
                      ("v_memcache", v_memcache), ("k_read", k_read), ("v_read", v_read), ("out", out)):
        tabs.append(None if tab is None else _dev(tab, name, (n_layers,), torch.int64))
    pws, nws = None, 0
    if workspace is not None:
        pws, nws = _dev(workspace, "workspace"), workspace.numel() * workspace.element_size()
    code = F32 if dtype == torch.float32 else BF16
    rc = lib.loma_decode_attn_layers(*tabs, n_layers, B, H, d, t, c, n_mem_chunks, mem_capacity, read_fill,
                                     float(scale), code, pws, nws, _stream(stream))
    if rc != OK:
        raise LomaError(rc, "loma_decode_attn_layers")


def loma_decode_attn_gqa_layers(q, k_new, v_new, k_memcache, v_memcache, k_read, v_read, out, n_layers, B, H, H_kv, d, t, c,
                                n_mem_chunks, mem_capacity, read_fill, scale, dtype=torch.bfloat16, workspace=None,
                                stream=None):
    """loma_decode_attn_gqa on n_layers caches in one launch (pointer tables as for loma_decode_attn_layers)."""
    tabs = []
    for name, tab in (("q", q), ("k_new", k_new), ("v_new", v_new), ("k_memcache", k_memcache),
                      ("v_memcache", v_memcache), ("k_read", k_read), ("v_read", v_read), ("out", out)):
        tabs.append(None if tab is None else _dev(tab, name, (n_layers,), torch.int64))
    pws, nws = None, 0
    if workspace is not None:
        pws, nws = _dev(workspace, "workspace"), workspace.numel() * workspace.element_size()
    code = F32 if dtype == torch.float32 else BF16
    rc = lib.loma_decode_attn_gqa_layers(*tabs, n_layers, B, H, H_kv, d, t, c, n_mem_chunks, mem_capacity, read_fill,
                                         float(scale), code, pws, nws, _stream(stream))
    if rc != OK:
        raise LomaError(rc, "loma_decode_attn_gqa_layers")


def loma_prefill_attn(q, k_new, v_new, k_memcache, v_memcache, k_read, v_read, t, c, n_mem_chunks, read_fill, scale,
                      out=None, lse=None, stream=None):
    """n_new tokens per sequence at once against [memory cache || reading zone], causal among themselves."""
    B, H, n_new, d = q.shape
    if out is None:
        out = torch.empty_like(q)
    dt = q.dtype
    cap = 0 if k_memcache is None else k_memcache.shape[2]
    pkm = None if k_memcache is None else _dev(k_memcache, "k_memcache", (B, H, cap, d), dt)
    pvm = None if v_memcache is None else _dev(v_memcache, "v_memcache", (B, H, cap, d), dt)
    plse = None if lse is None else _dev(lse, "lse", (B, H, n_new), torch.float32)
    rc = lib.loma_prefill_attn(_dev(q, "q"), _dev(k_new, "k_new", q.shape, dt), _dev(v_new, "v_new", q.shape, dt),
                               pkm, pvm, _dev(k_read, "k_read", (B, H, t * c, d), dt),
                               _dev(v_read, "v_read", (B, H, t * c, d), dt), _dev(out, "out", q.shape, dt), plse,
                               B, H, d, t, c, n_mem_chunks, cap, read_fill, n_new, float(scale), _dtype_code(q),
                               _stream(stream))
    if rc != OK:
        raise LomaError(rc, "loma_prefill_attn")
    return out


def mask_schedule(B, H, d, t, c, n_chunks, dtype=torch.bfloat16):
    """Host-only view of the mask pass's work list: list of (bh, chunk, zone, row0, rows, keys)."""
    code = F32 if dtype == torch.float32 else BF16
    n = int(lib.loma_mask_schedule_size(B, H, d, t, c, n_chunks, code))
    items = []
    buf = (ctypes.c_int * 6)()
    for blk in range(n):
        rc = lib.loma_mask_schedule_item(B, H, d, t, c, n_chunks, code, blk, ctypes.byref(buf))
        if rc < 0:
            raise LomaError(rc, "loma_mask_schedule_item")
        if rc == 1:
            items.append(tuple(buf))
    return items
