"""ctypes front end of oracle/loma_oracle.c -- TEST INFRASTRUCTURE, not a product path.

`build()` compiles the C file with gcc (fp64, OpenMP); the wrappers marshal numpy
arrays only.  Inputs may be float32 arrays or uint16 arrays of bf16 bit patterns.
Nothing here imports or is imported by the HIP library's package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "loma_oracle.c")
_LIB = os.path.join(_HERE, "libloma_oracle.so")
_lib = None

F32, BF16 = 0, 1


def build(force: bool = False) -> str:
    """Compile the C oracle next to its source.  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        vp, ip, dp = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p
        I, D, L = ctypes.c_int, ctypes.c_double, ctypes.c_long
        lib.loma_oracle_mask_attn.argtypes = [vp, vp, vp, dp, dp, I, I, I, I, I, I, D, I, ip, I, I]
        lib.loma_oracle_mask_attn.restype = I
        lib.loma_oracle_attend_segments.argtypes = [vp, I, vp, vp, L, I, vp, vp, L, I, dp, dp,
                                                    I, I, I, D, I, ip, I, I]
        lib.loma_oracle_attend_segments.restype = I
        lib.loma_oracle_mask_attn_bwd.argtypes = [vp, vp, vp, vp, dp, dp, dp, I, I, I, I, I, I, D, I, I]
        lib.loma_oracle_mask_attn_bwd.restype = I
        lib.loma_oracle_num_threads.restype = I
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().loma_oracle_num_threads())


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError("oracle inputs must be float32 or uint16 (bf16 bits)")


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def mask_attn(q, k, v, t, c, n_chunks, scale, rows=None, return_lse=False, nthreads=0):
    """Mask pass (Eq. 1-3, 5-7).  q, k, v: [B, H, S, d] float32 or uint16(bf16).
    rows: optional 1-D int array of query rows to compute.  Returns fp64 [B, H, nrows, d]."""
    q, k, v = (np.ascontiguousarray(x) for x in (q, k, v))
    code = _dtype_code(q)
    assert _dtype_code(k) == code and _dtype_code(v) == code
    B, H, S, d = q.shape
    assert k.shape == q.shape and v.shape == q.shape
    assert S == n_chunks * t * (2 * c + 1)
    rows_arr = None
    nrows = S
    if rows is not None:
        rows_arr = np.ascontiguousarray(rows, dtype=np.int32)
        nrows = rows_arr.size
    out = np.empty((B, H, nrows, d), dtype=np.float64)
    lse = np.empty((B, H, nrows), dtype=np.float64) if return_lse else None
    rc = _load().loma_oracle_mask_attn(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), B, H, d, t, c,
                                       n_chunks, float(scale), code, _ptr(rows_arr), nrows, nthreads)
    if rc != 0:
        raise RuntimeError("loma_oracle_mask_attn failed")
    return (out, lse) if return_lse else out


def mask_attn_bwd(q, k, v, dout, t, c, n_chunks, scale, nthreads=0):
    """Gradients (dq, dk, dv), fp64 [B, H, S, d], of the mask pass for the upstream gradient dout."""
    q, k, v, dout = (np.ascontiguousarray(x) for x in (q, k, v, dout))
    code = _dtype_code(q)
    assert all(_dtype_code(x) == code and x.shape == q.shape for x in (k, v, dout))
    B, H, S, d = q.shape
    assert S == n_chunks * t * (2 * c + 1)
    dq, dk, dv = (np.empty((B, H, S, d), dtype=np.float64) for _ in range(3))
    rc = _load().loma_oracle_mask_attn_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(dout), _ptr(dq), _ptr(dk), _ptr(dv),
                                           B, H, d, t, c, n_chunks, float(scale), code, nthreads)
    if rc != 0:
        raise RuntimeError("loma_oracle_mask_attn_bwd failed")
    return dq, dk, dv


def attend_segments(q, k1, v1, n1, k2, v2, n2, scale, bh_list=None, nthreads=0, return_lse=False):
    """All-visible attention of q [B, H, Lq, d] over rows [0, n1) of k1/v1 [B, H, cap1, d]
    followed by rows [0, n2) of k2/v2 [B, H, cap2, d].  Returns fp64 [nbh, Lq, d] (and, with
    return_lse, the log-sum-exp of the scaled scores, fp64 [nbh, Lq])."""
    q = np.ascontiguousarray(q)
    code = _dtype_code(q)
    B, H, Lq, d = q.shape
    arrs = []
    for a, nseg in ((k1, n1), (v1, n1), (k2, n2), (v2, n2)):
        if nseg > 0:
            a = np.ascontiguousarray(a)
            assert _dtype_code(a) == code and a.shape[0] == B and a.shape[1] == H and a.shape[3] == d
        arrs.append(a)
    k1, v1, k2, v2 = arrs
    s1 = k1.shape[2] if n1 > 0 else 0
    s2 = k2.shape[2] if n2 > 0 else 0
    bh_arr = None
    nbh = B * H
    if bh_list is not None:
        bh_arr = np.ascontiguousarray(bh_list, dtype=np.int32)
        nbh = bh_arr.size
    out = np.empty((nbh, Lq, d), dtype=np.float64)
    lse = np.empty((nbh, Lq), dtype=np.float64) if return_lse else None
    rc = _load().loma_oracle_attend_segments(
        _ptr(q), Lq, _ptr(k1) if n1 > 0 else None, _ptr(v1) if n1 > 0 else None, s1, n1,
        _ptr(k2) if n2 > 0 else None, _ptr(v2) if n2 > 0 else None, s2, n2,
        _ptr(out), _ptr(lse), B, H, d, float(scale), code, _ptr(bh_arr), nbh, nthreads)
    if rc != 0:
        raise RuntimeError("loma_oracle_attend_segments failed")
    return (out, lse) if return_lse else out


class GenerationCache:
    """Generation form (Sec. 3.1 steps 1-3, Appendix A) over explicit host buffers.

    State: k_mem/v_mem [B, H, mem_capacity, d] with n_mem_chunks*t valid rows and
    k_read/v_read [B, H, t*c, d] with read_fill valid rows; dtype float32 or uint16(bf16).
    """

    def __init__(self, k_mem, v_mem, n_mem_chunks, k_read, v_read, read_fill, t, c, scale):
        self.k_mem, self.v_mem, self.k_read, self.v_read = k_mem, v_mem, k_read, v_read
        self.n_mem_chunks, self.read_fill = int(n_mem_chunks), int(read_fill)
        self.t, self.c, self.R, self.scale = t, c, t * c, float(scale)
        assert k_read.shape[2] == self.R and 0 <= self.read_fill <= self.R
        assert self.n_mem_chunks * t <= k_mem.shape[2]

    def decode(self, q, k_new, v_new, bh_list=None):
        """Append (k_new, v_new) [B, H, 1, d] to the reading zone, attend over the whole cache."""
        if self.read_fill >= self.R:
            raise ValueError("reading zone full: compress first")
        self.k_read[:, :, self.read_fill] = k_new[:, :, 0]
        self.v_read[:, :, self.read_fill] = v_new[:, :, 0]
        self.read_fill += 1
        out, self.last_lse = attend_segments(q, self.k_mem, self.v_mem, self.n_mem_chunks * self.t,
                                             self.k_read, self.v_read, self.read_fill, self.scale, bh_list,
                                             return_lse=True)
        return out

    def prefill(self, q, k_new, v_new, bh_list=None):
        """l tokens at once (Appendix A, several input tokens): token i sees the cache and new tokens
        0..i -- written out as l single-token steps, the plain meaning of the shifted lower triangle."""
        l = q.shape[2]
        if l < 1 or self.read_fill + l > self.R:
            raise ValueError("the new tokens must fit the reading zone")
        outs, lses = [], []
        for i in range(l):
            outs.append(self.decode(q[:, :, i:i + 1], k_new[:, :, i:i + 1], v_new[:, :, i:i + 1], bh_list))
            lses.append(self.last_lse)
        self.last_lse = np.concatenate(lses, axis=1)      # [nbh, l]: one value per new token
        return np.concatenate(outs, axis=2)

    def compress(self, q_m, k_m, v_m, bh_list=None):
        """t <m> queries over [reading zone || own K/V]; then splice the t new KVs into the memory."""
        if self.read_fill != self.R:
            raise ValueError("compression needs a full reading zone")
        lo = self.n_mem_chunks * self.t
        if lo + self.t > self.k_mem.shape[2]:
            raise ValueError("memory cache full")
        out = attend_segments(q_m, self.k_read, self.v_read, self.R, k_m, v_m, self.t, self.scale, bh_list)
        self.k_mem[:, :, lo:lo + self.t] = k_m
        self.v_mem[:, :, lo:lo + self.t] = v_m
        self.n_mem_chunks += 1
        self.read_fill = 0
        return out
