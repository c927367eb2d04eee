"""Seeded synthetic workloads shaped like the paper's Llama-2-7B settings (Sec. 5.1).

This module only draws random numbers and rounds them to the storage type; it
holds none of the attention arithmetic.  Both the HIP path's tests and the CPU
checker are fed from here, so they see identical bits.

The five configurations (seed = 9486 + index):
  0  tiny mask pass, fp32      B1  H1  d64  t4  c4   4 chunks   N(0,1)
  1  mask pass, bf16           B2  H32 d128 t16 c4   28 chunks  0.5*N(0,1)
  2  generation, bf16          B8  H32 d128 t16 c4   64 prior chunks, 256 decode steps
  3  long mask pass, bf16      B1  H32 d128 t32 c8   60 chunks  0.5*N(0,1)
  4  high-ratio decode, bf16   B64 H32 d128 t16 c16  512 prior chunks, 128 decode steps
The generation configurations start with a FULL reading zone, i.e. at the instant
the appendix's driver loop is about to compress; compression then recurs every
t*c decode steps.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

SEED_BASE = 9486


@dataclass(frozen=True)
class MaskConfig:
    index: int
    name: str
    B: int
    H: int
    d: int
    t: int
    c: int
    n_chunks: int
    dtype: str          # "f32" | "bf16"
    value_scale: float  # inputs are value_scale * N(0,1)

    @property
    def R(self):
        return self.t * self.c

    @property
    def s(self):
        return self.t * (2 * self.c + 1)

    @property
    def S(self):
        return self.n_chunks * self.s

    @property
    def scale(self):
        return 1.0 / float(np.sqrt(self.d))

    @property
    def seed(self):
        return SEED_BASE + self.index


@dataclass(frozen=True)
class GenConfig:
    index: int
    name: str
    B: int
    H: int
    d: int
    t: int
    c: int
    prior_chunks: int   # chunks already compressed when the run starts
    steps: int          # decode steps (one query per sequence each)
    dtype: str
    kv_scale: float
    q_scale: float

    @property
    def R(self):
        return self.t * self.c

    @property
    def scale(self):
        return 1.0 / float(np.sqrt(self.d))

    @property
    def seed(self):
        return SEED_BASE + self.index

    @property
    def n_compress(self):
        """Compressions in the run: one pending at step 0, then one per R decoded tokens."""
        return 1 + (self.steps - 1) // self.R if self.steps > 0 else 1

    @property
    def mem_capacity(self):
        return (self.prior_chunks + self.n_compress) * self.t


CONFIGS = (
    MaskConfig(0, "c1_tiny_mask_f32", 1, 1, 64, 4, 4, 4, "f32", 1.0),
    MaskConfig(1, "c2_llama7b_mask_bf16", 2, 32, 128, 16, 4, 28, "bf16", 0.5),
    GenConfig(2, "c3_generation_bf16", 8, 32, 128, 16, 4, 64, 256, "bf16", 1.0, 1.0),
    MaskConfig(3, "c4_long_mask_bf16", 1, 32, 128, 32, 8, 60, "bf16", 0.5),
    GenConfig(4, "c5_highratio_decode_bf16", 64, 32, 128, 16, 16, 512, 128, "bf16", 1.0, 0.5),
)


def shrink(cfg, **kw):
    """A smaller variant of a configuration (same seed and distribution)."""
    return replace(cfg, **kw)


# ---- storage rounding ------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bf16 bit patterns (uint16).  Finite inputs only."""
    bits = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = bits + np.uint32(0x7FFF) + ((bits >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _draw(rng, shape, value_scale, dtype):
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if value_scale != 1.0:
        x *= np.float32(value_scale)
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    return x


# ---- mask-pass inputs --------------------------------------------------------
def mask_inputs(cfg: MaskConfig):
    """q, k, v of shape [B, H, S, d]: float32 arrays (f32 configs) or uint16 bf16 bits."""
    rng = np.random.default_rng(cfg.seed)
    shape = (cfg.B, cfg.H, cfg.S, cfg.d)
    return tuple(_draw(rng, shape, cfg.value_scale, cfg.dtype) for _ in range(3))


def mask_grad_input(cfg: MaskConfig):
    """Upstream gradient of the mask pass's output, [B, H, S, d], unit normal, in the config's dtype
    (a stream of its own, so q, k, v of mask_inputs are unchanged by drawing it)."""
    rng = np.random.default_rng(cfg.seed + 500_000)
    return _draw(rng, (cfg.B, cfg.H, cfg.S, cfg.d), 1.0, cfg.dtype)


# ---- generation inputs ---------------------------------------------------------
def gen_initial_state(cfg: GenConfig):
    """Cache at the start of the run: prior_chunks*t memory rows in buffers of
    mem_capacity rows, and a full reading zone of t*c rows."""
    rng = np.random.default_rng(cfg.seed)
    Lm = cfg.prior_chunks * cfg.t
    out = {}
    for name in ("k_mem", "v_mem"):
        buf = np.zeros((cfg.B, cfg.H, cfg.mem_capacity, cfg.d),
                       dtype=np.uint16 if cfg.dtype == "bf16" else np.float32)
        buf[:, :, :Lm] = _draw(rng, (cfg.B, cfg.H, Lm, cfg.d), cfg.kv_scale, cfg.dtype)
        out[name] = buf
    for name in ("k_read", "v_read"):
        out[name] = _draw(rng, (cfg.B, cfg.H, cfg.R, cfg.d), cfg.kv_scale, cfg.dtype)
    return out


def gen_step_inputs(cfg: GenConfig, step: int):
    """(q, k_new, v_new), each [B, H, 1, d], for decode step `step`."""
    rng = np.random.default_rng([cfg.seed, 1, step])
    shape = (cfg.B, cfg.H, 1, cfg.d)
    q = _draw(rng, shape, cfg.q_scale, cfg.dtype)
    k = _draw(rng, shape, cfg.kv_scale, cfg.dtype)
    v = _draw(rng, shape, cfg.kv_scale, cfg.dtype)
    return q, k, v


def gen_compress_inputs(cfg: GenConfig, event: int):
    """(q_mem, k_mem, v_mem), each [B, H, t, d], for the event-th compression."""
    rng = np.random.default_rng([cfg.seed, 2, event])
    shape = (cfg.B, cfg.H, cfg.t, cfg.d)
    q = _draw(rng, shape, cfg.q_scale, cfg.dtype)
    k = _draw(rng, shape, cfg.kv_scale, cfg.dtype)
    v = _draw(rng, shape, cfg.kv_scale, cfg.dtype)
    return q, k, v


# ---- work and traffic accounting (counting only) -----------------------------------
def visible_pairs(t: int, c: int, n: int) -> int:
    """Ones in the whole-sample mask per (b, h), from the block sizes of the chunk and
    cross-chunk masks: earlier memory zones for reading rows, the causal triangle, the
    memory rows, and the repetition rows (memory zone + self)."""
    R = t * c
    return R * t * n * (n - 1) // 2 + n * (R * (R + 1) // 2 + t * (R + t) + R * (t + 1))


def mask_pass_useful_flops(cfg: MaskConfig) -> int:
    return 4 * cfg.d * visible_pairs(cfg.t, cfg.c, cfg.n_chunks) * cfg.B * cfg.H


def elem_bytes(dtype: str) -> int:
    return 2 if dtype == "bf16" else 4


def mask_pass_bytes(cfg: MaskConfig) -> int:
    """q, k, v read once and out written once."""
    return 4 * cfg.B * cfg.H * cfg.S * cfg.d * elem_bytes(cfg.dtype)


def decode_bytes(B, H, d, n_keys, dtype) -> int:
    """K and V of every visible key read once, plus q, k_new, v_new in and out."""
    return B * H * (2 * n_keys * d + 4 * d) * elem_bytes(dtype)


def compress_bytes(B, H, d, t, c, dtype) -> int:
    """reading zone + <m> K/V read, q in, out, and the splice write."""
    R = t * c
    return B * H * (2 * (R + t) * d + 2 * t * d + 2 * t * d) * elem_bytes(dtype)


def compress_useful_flops(B, H, d, t, c) -> int:
    return 4 * d * t * (t * c + t) * B * H


# ---- device-side tensors for the large configurations ---------------------------------------
class TiledPool:
    """Seeded unit-normal bf16 values drawn once on the host (numpy default_rng); device tensors are filled with
    runs of the pool at offsets the same host generator picks.  Stands in for fresh draws where a tensor set is too
    large for a trip through host memory (the 9 GB caches of the largest generation configuration, the rotating
    tensor sets of the benchmark); no GPU random-number kernel is involved.  Scales are powers of two (exact)."""

    def __init__(self, seed, n=1 << 23, device="cuda"):
        import torch
        rng = np.random.default_rng(seed)
        bits = f32_to_bf16_bits(rng.standard_normal(n, dtype=np.float32))
        self.torch = torch
        self.unit = torch.from_numpy(bits.view(np.int16)).to(device).view(torch.bfloat16)
        self.scaled = {1.0: self.unit}
        self.rng = rng
        self.n = n
        self.device = device

    def tensor(self, shape, scale=1.0):
        torch = self.torch
        if scale not in self.scaled:
            assert np.log2(scale) == int(np.log2(scale)), "scales are powers of two"
            self.scaled[scale] = (self.unit.float() * scale).to(torch.bfloat16)
        src = self.scaled[scale]
        out = torch.empty(shape, dtype=torch.bfloat16, device=self.device)
        flat = out.view(-1)
        piece = self.n // 2
        for i in range(0, flat.numel(), piece):
            m = min(piece, flat.numel() - i)
            off = int(self.rng.integers(0, self.n - m + 1))
            flat[i:i + m] = src[off:off + m]
        return out


def gen_initial_state_device(cfg: GenConfig, device="cuda", pool=None):
    """Same layout as gen_initial_state, filled on the GPU from a TiledPool seeded with cfg.seed (bf16 only).
    Returns torch tensors in the storage dtype."""
    import torch
    assert cfg.dtype == "bf16"
    pool = pool or TiledPool(cfg.seed, device=device)
    Lm = cfg.prior_chunks * cfg.t
    state = {}
    for name in ("k_mem", "v_mem"):
        buf = torch.zeros((cfg.B, cfg.H, cfg.mem_capacity, cfg.d), dtype=torch.bfloat16, device=device)
        buf[:, :, :Lm] = pool.tensor((cfg.B, cfg.H, Lm, cfg.d), cfg.kv_scale)
        state[name] = buf
    for name in ("k_read", "v_read"):
        state[name] = pool.tensor((cfg.B, cfg.H, cfg.R, cfg.d), cfg.kv_scale)
    return state
