"""CPU fp64 oracle for LoMA's position ids and for rotary position embedding -- TEST INFRASTRUCTURE.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module.  It shares no code
with the HIP library and never imports it.

Position ids (Sec. 4.5, Eq. 14; Appendix A, compress_last_chunk with both position types):
  * the text is cut into chunks of t*c tokens (the reading zones); reading token j of chunk i keeps its
    original position i*tc + j (first stated purpose of the design);
  * the t memory tokens of chunk i take, with position type "intermittent", the ids of every c-th reading
    token counted from the end of each group of c: i*tc + c-1, i*tc + 2c-1, ..., i*tc + tc-1 (Eq. 14, read
    with chunk length tc and chunk start i*tc: the printed "length t, start it" cannot produce a last id of
    it + tc - 1 inside the chunk, and the appendix computes range(cursor - tc + c - 1, cursor, c)); the last
    of them is one below the next chunk's first reading id (second stated purpose);
  * with position type "contiguous" (the appendix's other branch) they take mem_cursor .. mem_cursor + t-1,
    where mem_cursor = (chunks compressed so far) * t is the length of the compressed cache;
  * repetition tokens: the paper gives no ids for them.  Reading taken here: repetition token j of chunk i
    carries the id of the reading token it reproduces, i*tc + j, so that its distance to the memory token
    that covers position j is the same as the reading token's.
Generation (Appendix A): `cursor` counts the real tokens fed so far; new tokens take cursor, cursor+1, ...;
memory tokens do not advance it.

Rotary embedding: the paper fine-tunes Llama-2, whose attention rotates q and k by their position id before
the scores are taken.  Convention: the one of the public Llama-2 code in its widely used "rotate-half" form --
head-dim element i (i < d/2) pairs with element i + d/2, the pair turns by the angle pos * theta^(-2i/d):
    y[i]       = x[i] cos(a_i) - x[i + d/2] sin(a_i)
    y[i + d/2] = x[i + d/2] cos(a_i) + x[i] sin(a_i),        a_i = pos * theta^(-2i/d).
All arithmetic here is fp64; `round_to` rounds a result to the storage type the way a model running in that
type would hold it (the kernels keep rotated q and k in the storage type too).
"""
from __future__ import annotations

import numpy as np

INTERMITTENT, CONTIGUOUS = "intermittent", "contiguous"


def memory_position_ids(chunk: int, t: int, c: int, position_type: str = INTERMITTENT) -> np.ndarray:
    """Ids of the t memory tokens of chunk `chunk` (= number of chunks compressed before it)."""
    if position_type == INTERMITTENT:
        return np.array([chunk * t * c + (j + 1) * c - 1 for j in range(t)], dtype=np.int64)   # Eq. 14
    if position_type == CONTIGUOUS:
        return np.array([chunk * t + j for j in range(t)], dtype=np.int64)                      # mem_cursor + j
    raise ValueError(f"unknown position type {position_type!r}")


def sample_position_ids(t: int, c: int, n: int, position_type: str = INTERMITTENT) -> np.ndarray:
    """Ids of every row of a restructured training sample of n chunks [reading | memory | repetition]."""
    R = t * c
    ids = []
    for i in range(n):
        reading = [i * R + j for j in range(R)]
        ids += reading                                               # original positions, preserved
        ids += memory_position_ids(i, t, c, position_type).tolist()
        ids += reading                                               # each <r> token: the token it reproduces
    return np.array(ids, dtype=np.int64)


def generation_position_ids(cursor: int, n_new: int) -> np.ndarray:
    """Ids of n_new real tokens fed when `cursor` real tokens have been fed before (Appendix A)."""
    return np.arange(cursor, cursor + n_new, dtype=np.int64)


def compress_position_ids(cursor: int, t: int, c: int, compressed_chunks: int, position_type: str = INTERMITTENT):
    """Ids of the t memory tokens at a compression boundary of the generation loop: the reading zone that was
    just filled holds the tokens cursor - tc .. cursor - 1."""
    R = t * c
    if cursor < R:
        raise ValueError("a full reading zone has been fed before any compression")
    if position_type == INTERMITTENT:
        first_of_zone = cursor - R
        return np.array([first_of_zone + (j + 1) * c - 1 for j in range(t)], dtype=np.int64)
    if position_type == CONTIGUOUS:
        return np.array([compressed_chunks * t + j for j in range(t)], dtype=np.int64)
    raise ValueError(f"unknown position type {position_type!r}")


def rope_angles(pos, d: int, theta: float = 10000.0) -> np.ndarray:
    """[len(pos), d/2] angles pos * theta^(-2i/d), fp64."""
    if d % 2:
        raise ValueError("head_dim must be even")
    pos = np.asarray(pos, dtype=np.float64).reshape(-1)
    inv_freq = np.float64(theta) ** (-2.0 * np.arange(d // 2, dtype=np.float64) / d)
    return pos[:, None] * inv_freq[None, :]


def rope_rotate(x, pos, theta: float = 10000.0) -> np.ndarray:
    """Rotate rows of x [..., L, d] by their position ids pos [L]; returns fp64."""
    x = np.asarray(x, dtype=np.float64)
    L, d = x.shape[-2], x.shape[-1]
    a = rope_angles(pos, d, theta)
    if a.shape[0] != L:
        raise ValueError("one position id per row")
    cos, sin = np.cos(a), np.sin(a)
    lo, hi = x[..., : d // 2], x[..., d // 2:]
    return np.concatenate([lo * cos - hi * sin, hi * cos + lo * sin], axis=-1)


def round_to(x: np.ndarray, dtype: str) -> np.ndarray:
    """fp64 -> the storage type's value set (round to nearest even), returned as float32 values ("f32") or as
    bf16 bit patterns in uint16 ("bf16"): what a tensor of that type holds after the rotation."""
    x32 = np.asarray(x, dtype=np.float64).astype(np.float32)
    if dtype == "f32":
        return x32
    if dtype != "bf16":
        raise ValueError(dtype)
    # fp64 -> bf16 in one rounding: round the fp64 value's 53-bit significand to 8 bits directly
    m, e = np.frexp(np.asarray(x, dtype=np.float64))        # x = m * 2^e, 0.5 <= |m| < 1
    q = np.rint(m * 256.0) / 256.0                           # 8 significant bits, ties to even
    y = np.ldexp(q, e).astype(np.float32)                    # exact: 8 bits fit fp32
    bits = y.view(np.uint32)
    assert not np.any(bits & np.uint32(0xFFFF)), "value not representable in bf16"
    return (bits >> np.uint32(16)).astype(np.uint16)
