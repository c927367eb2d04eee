"""CPU fp64 oracle for LoMA attention -- TEST INFRASTRUCTURE, not a product path.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
module.  It shares no code with the HIP library and never imports it.

What it computes (LoMA paper):
  * the explicit 0/1 attention mask of a restructured training sample, built two
    independent ways: block assembly of Eq. 1, Eq. 2, Eq. 3 (Sec. 4.3) and an
    element-wise predicate written from the three mask criteria of Sec. 4.3
    plus the "token itself" clause of the Introduction;
  * masked scaled-dot-product attention O = Softmax(A) V, Eq. 5-7 (Sec. 4.4),
    where a 0 in the mask removes the pair from the softmax;
  * the generation form of Sec. 3.1 (steps 1-3) and Appendix A: a query over
    [memory-zone KVs of earlier chunks || live reading zone] and the periodic
    compression pass of t <m> queries over [reading zone || their own KVs].

Everything is dense numpy in float64; there is no blocking, fusion or skipping.
Inputs are taken as exact fp64 images of whatever (fp32 / bf16-rounded) values
the caller passes.

Pins (tests/test_oracle_*.py): the hand-written Fig. 1 mask, closed-form counts,
Q = 0 / constant-V closed forms, reduction of each zone to a library SDPA call,
brute-force enumeration on tiny inputs, visibility (perturbation) invariance and
generation-form == mask-pass rows.
"""
from __future__ import annotations

import numpy as np

READ, MEM, REP = 0, 1, 2


# --------------------------------------------------------------------------
# Mask, builder 1: block assembly, Eq. 1 (M), Eq. 3 (S), Eq. 2 (whole sample)
# --------------------------------------------------------------------------
def chunk_mask_M(t: int, c: int) -> np.ndarray:
    """Eq. 1: the s x s mask of one training chunk, s = t(2c+1)."""
    R = t * c
    L = np.tril(np.ones((R, R), dtype=np.uint8))          # causal, diagonal included
    one = lambda a, b: np.ones((a, b), dtype=np.uint8)
    zero = lambda a, b: np.zeros((a, b), dtype=np.uint8)
    eye = np.eye(R, dtype=np.uint8)
    return np.block([
        [L,          zero(R, t), zero(R, R)],
        [one(t, R),  one(t, t),  zero(t, R)],
        [zero(R, R), one(R, t),  eye],
    ])


def cross_mask_S(t: int, c: int) -> np.ndarray:
    """Eq. 3: what a chunk sees of an EARLIER chunk: reading rows x memory columns."""
    R = t * c
    s = 2 * R + t
    S = np.zeros((s, s), dtype=np.uint8)
    S[0:R, R:R + t] = 1
    return S


def mask_from_blocks(t: int, c: int, n: int) -> np.ndarray:
    """Eq. 2: M on the diagonal, S everywhere below it, 0 above."""
    M, S = chunk_mask_M(t, c), cross_mask_S(t, c)
    Z = np.zeros_like(M)
    rows = [[M if j == i else (S if j < i else Z) for j in range(n)] for i in range(n)]
    return np.block(rows)


# --------------------------------------------------------------------------
# Mask, builder 2: the three criteria of Sec. 4.3, one (row, column) at a time
# --------------------------------------------------------------------------
def zone_of(offset: int, t: int, c: int) -> int:
    R = t * c
    if offset < R:
        return READ
    if offset < R + t:
        return MEM
    return REP


def visible(p: int, q: int, t: int, c: int) -> bool:
    """May the token at row p attend to the token at column q?"""
    s = t * (2 * c + 1)
    yp, op = divmod(p, s)
    yq, oq = divmod(q, s)
    zp, zq = zone_of(op, t, c), zone_of(oq, t, c)
    if zp == READ:
        # criterion 1: every preceding memory zone; causal inside its own reading zone
        if yq < yp:
            return zq == MEM
        return yq == yp and zq == READ and oq <= op
    if zp == MEM:
        # criterion 2: bidirectional inside the memory zone + the adjacent reading zone, nothing else
        return yq == yp and zq in (READ, MEM)
    # criterion 3 (+ Introduction): the memory zone right before it, and the token itself
    return yq == yp and (zq == MEM or q == p)


def mask_from_rules(t: int, c: int, n: int) -> np.ndarray:
    S = n * t * (2 * c + 1)
    out = np.zeros((S, S), dtype=np.uint8)
    for p in range(S):
        for q in range(S):
            out[p, q] = 1 if visible(p, q, t, c) else 0
    return out


# --------------------------------------------------------------------------
# Masked attention, Eq. 5-7
# --------------------------------------------------------------------------
def masked_softmax_attention(q, k, v, mask, scale):
    """One head.  q: [Lq, d]; k, v: [Lk, d]; mask: [Lq, Lk] of 0/1.

    A = scale * q k^T (Eq. 5); pairs with mask 0 are removed from the softmax;
    O_i = E_i * sum_j exp(A_ij) v_j with E_i = 1 / sum_j exp(A_ij) (Eq. 7).
    Returns (O [Lq, d], LSE [Lq], W [Lq, Lk]) with W the attention weights.
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    keep = np.asarray(mask).astype(bool)
    if not keep.any(axis=1).all():
        raise ValueError("a query row has no visible key")
    A = (q @ k.T) * float(scale)
    A = np.where(keep, A, -np.inf)
    row_max = A.max(axis=1, keepdims=True)
    e = np.where(keep, np.exp(A - row_max), 0.0)
    denom = e.sum(axis=1, keepdims=True)
    W = e / denom
    # masked V rows must not leak NaN/Inf through 0 * x: multiply only visible pairs
    O = np.zeros((q.shape[0], v.shape[1]), dtype=np.float64)
    for i in range(q.shape[0]):
        idx = np.nonzero(keep[i])[0]
        O[i] = W[i, idx] @ v[idx]
    lse = (row_max + np.log(denom))[:, 0]
    return O, lse, W


def mask_attn_fwd(q, k, v, t, c, n_chunks, scale, return_lse=False):
    """Training / compression-pass form.  q, k, v: [B, H, S, d], S = n_chunks * t(2c+1)."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    B, H, S, d = q.shape
    if S != n_chunks * t * (2 * c + 1):
        raise ValueError("sequence length is not n_chunks * t(2c+1)")
    mask = mask_from_blocks(t, c, n_chunks)
    out = np.empty((B, H, S, d), dtype=np.float64)
    lse = np.empty((B, H, S), dtype=np.float64)
    for b in range(B):
        for h in range(H):
            out[b, h], lse[b, h], _ = masked_softmax_attention(q[b, h], k[b, h], v[b, h], mask, scale)
    return (out, lse) if return_lse else out


def mask_attn_bwd(q, k, v, dout, t, c, n_chunks, scale):
    """Gradients of the mask pass (Sec. 4.4: O = softmax(A + log M) V, Eq. 5-7) for an upstream
    gradient dout of O.  With W the attention weights (0 on masked pairs):
        dV = W^T dO;   dW = dO V^T;   dA = W * (dW - rowsum(dO * O));   dQ = scale dA K;   dK = scale dA^T Q.
    A masked pair has W = 0, so nothing flows through it: a repetition row sends gradient only to its
    chunk's memory K/V and to its own K/V (the path that trains the memory tokens, Sec. 4.2).
    Returns (dq, dk, dv), fp64, shaped like q."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    dout = np.asarray(dout, dtype=np.float64)
    B, H, S, d = q.shape
    if S != n_chunks * t * (2 * c + 1):
        raise ValueError("sequence length is not n_chunks * t(2c+1)")
    mask = mask_from_blocks(t, c, n_chunks)
    dq, dk, dv = np.empty_like(q), np.empty_like(q), np.empty_like(q)
    for b in range(B):
        for h in range(H):
            O, _, W = masked_softmax_attention(q[b, h], k[b, h], v[b, h], mask, scale)
            dO = dout[b, h]
            dv[b, h] = W.T @ dO
            dW = dO @ v[b, h].T
            delta = (dO * O).sum(axis=1, keepdims=True)
            dA = W * (dW - delta)
            dq[b, h] = float(scale) * (dA @ k[b, h])
            dk[b, h] = float(scale) * (dA.T @ q[b, h])
    return dq, dk, dv


# --------------------------------------------------------------------------
# Generation form: Sec. 3.1 steps 1-3, Appendix A
# --------------------------------------------------------------------------
class GenerationCache:
    """Explicit KV cache of one attention layer: [mem_0 .. mem_{y-1} || live reading zone].

    decode():   append the new token's (k, v) to the reading zone, then attend over
                the whole cache (the appendix mask for one new token is all ones over
                cache + itself).
    compress(): needs a full reading zone (t*c tokens).  The t <m> queries attend,
                unmasked, over [reading zone || their own t KVs] -- NOT over older
                memory zones (the appendix slices the last t*c cache rows only).
                Then the reading zone is dropped and the t new KVs join the memory.
    """

    def __init__(self, B, H, d, t, c, scale):
        self.B, self.H, self.d, self.t, self.c = B, H, d, t, c
        self.R = t * c
        self.scale = float(scale)
        self.k_mem = np.zeros((B, H, 0, d))
        self.v_mem = np.zeros((B, H, 0, d))
        self.k_read = np.zeros((B, H, 0, d))
        self.v_read = np.zeros((B, H, 0, d))
        self.n_mem_chunks = 0

    @property
    def read_fill(self):
        return self.k_read.shape[2]

    def load_state(self, k_mem, v_mem, k_read, v_read):
        k_mem = np.asarray(k_mem, dtype=np.float64)
        if k_mem.shape[2] % self.t:
            raise ValueError("memory length must be a multiple of t")
        if np.asarray(k_read).shape[2] > self.R:
            raise ValueError("reading zone longer than t*c")
        self.k_mem, self.v_mem = k_mem, np.asarray(v_mem, dtype=np.float64)
        self.k_read, self.v_read = np.asarray(k_read, dtype=np.float64), np.asarray(v_read, dtype=np.float64)
        self.n_mem_chunks = k_mem.shape[2] // self.t

    def _attend(self, q, k, v):
        Lq, Lk = q.shape[2], k.shape[2]
        ones = np.ones((Lq, Lk), dtype=np.uint8)
        out = np.empty(q.shape, dtype=np.float64)
        for b in range(self.B):
            for h in range(self.H):
                out[b, h], _, _ = masked_softmax_attention(q[b, h], k[b, h], v[b, h], ones, self.scale)
        return out

    def decode(self, q, k_new, v_new):
        """q, k_new, v_new: [B, H, 1, d]."""
        if self.read_fill >= self.R:
            raise ValueError("reading zone is full: compress first (Appendix A keeps it < t*c at rest)")
        self.k_read = np.concatenate([self.k_read, np.asarray(k_new, dtype=np.float64)], axis=2)
        self.v_read = np.concatenate([self.v_read, np.asarray(v_new, dtype=np.float64)], axis=2)
        k = np.concatenate([self.k_mem, self.k_read], axis=2)
        v = np.concatenate([self.v_mem, self.v_read], axis=2)
        return self._attend(np.asarray(q, dtype=np.float64), k, v)

    def decode_gqa(self, q, k_new, v_new):
        """Grouped-query decode: this cache holds H = H_kv key/value heads; q is [B, Hq, 1, d] with Hq a multiple
        of H, k_new, v_new are [B, H, 1, d].  Query head h reads KV head h // (Hq // H); otherwise decode()
        (Appendix A with one input token; the head sharing is the cache layout of grouped-query models, not the
        paper's Llama-2-7B)."""
        q = np.asarray(q, dtype=np.float64)
        Hq = q.shape[1]
        if Hq % self.H:
            raise ValueError("query heads must be a multiple of the cache's heads")
        G = Hq // self.H
        if self.read_fill >= self.R:
            raise ValueError("reading zone is full: compress first")
        self.k_read = np.concatenate([self.k_read, np.asarray(k_new, dtype=np.float64)], axis=2)
        self.v_read = np.concatenate([self.v_read, np.asarray(v_new, dtype=np.float64)], axis=2)
        k = np.concatenate([self.k_mem, self.k_read], axis=2)
        v = np.concatenate([self.v_mem, self.v_read], axis=2)
        ones = np.ones((1, k.shape[2]), dtype=np.uint8)
        out = np.empty(q.shape, dtype=np.float64)
        for b in range(self.B):
            for h in range(Hq):
                out[b, h], _, _ = masked_softmax_attention(q[b, h], k[b, h // G], v[b, h // G], ones, self.scale)
        return out

    def prefill(self, q, k_new, v_new):
        """q, k_new, v_new: [B, H, l, d] -- l tokens fed at once (Appendix A, inference_input with
        several input tokens).  The l rows are appended to the reading zone; the mask over
        [memory || reading zone incl. the new rows] is the lower triangle shifted by the
        number of cached rows: new token i sees every cached row and new tokens 0..i."""
        q = np.asarray(q, dtype=np.float64)
        l = q.shape[2]
        if l < 1 or self.read_fill + l > self.R:
            raise ValueError("the new tokens must fit the reading zone (feed a longer prompt in pieces)")
        cached = self.k_mem.shape[2] + self.read_fill
        self.k_read = np.concatenate([self.k_read, np.asarray(k_new, dtype=np.float64)], axis=2)
        self.v_read = np.concatenate([self.v_read, np.asarray(v_new, dtype=np.float64)], axis=2)
        k = np.concatenate([self.k_mem, self.k_read], axis=2)
        v = np.concatenate([self.v_mem, self.v_read], axis=2)
        mask = np.tril(np.ones((l, cached + l), dtype=np.uint8), k=cached)
        out = np.empty(q.shape, dtype=np.float64)
        lse = np.empty(q.shape[:3], dtype=np.float64)
        for b in range(self.B):
            for h in range(self.H):
                out[b, h], lse[b, h], _ = masked_softmax_attention(q[b, h], k[b, h], v[b, h], mask, self.scale)
        self.last_lse = lse
        return out

    def compress(self, q_m, k_m, v_m):
        """q_m, k_m, v_m: [B, H, t, d] -- the t <m> tokens."""
        if self.read_fill != self.R:
            raise ValueError("compression needs a full reading zone")
        k_m = np.asarray(k_m, dtype=np.float64)
        v_m = np.asarray(v_m, dtype=np.float64)
        k = np.concatenate([self.k_read, k_m], axis=2)
        v = np.concatenate([self.v_read, v_m], axis=2)
        out = self._attend(np.asarray(q_m, dtype=np.float64), k, v)
        self.k_mem = np.concatenate([self.k_mem, k_m], axis=2)
        self.v_mem = np.concatenate([self.v_mem, v_m], axis=2)
        self.k_read = self.k_read[:, :, :0]
        self.v_read = self.v_read[:, :, :0]
        self.n_mem_chunks += 1
        return out
