// dK/dV pass of the mask pass's gradients on the matrix cores (engine and notation: loma_bwd_engine.h), the sum of
// shared blocks' partial results, and the entry that runs the passes.
#include "loma_bwd_engine.h"

namespace loma {
namespace {

// dK/dV pass: per (b,h) the blocks of memory keys (longest first: the first block is seen by every later
// chunk; each streams the later chunks' reading rows from the last chunk backwards), then the reading-zone key
// blocks of every chunk.  Repetition-zone keys belong to the dQ pass.
// With P.split == 2 every block of memory keys is worked on by two workgroups: the first takes the block's own
// memory and repetition rows and the reading rows of the nearer later chunks, the second the reading rows of
// the farther ones (about half the rows each); both leave fp32 partial sums that bwd_reduce_kernel adds.
// the job of workgroup `id` of the dK/dV pass and the (b,h) pair it belongs to
template <int D>
__device__ __forceinline__ int dkv_job_of(const BwdParams& P, long long id, BwdJob& J) {
    const int nmk = P.n * P.t;
    const int nMK = (nmk + P.bm - 1) / P.bm;          // blocks of memory keys
    const int nRB = (P.R + P.bm - 1) / P.bm;          // reading-zone key blocks per chunk
    int bh, u;
    split_block(id, P.nbh, nMK * P.split + P.n * nRB, nMK * P.split, bh, u);
    J.rep = 0; J.t = P.t; J.magic_t = magic_of(P.t); J.z0 = J.z1 = 0; J.cb = 0;
    J.part_k = J.part_v = nullptr;
    J.pipe0 = J.pipe1 = J.pipe_end = 0;
    if (u < nMK * P.split) {
        const int part = u % P.split;
        const int mk0 = (u / P.split) * P.bm;
        J.vis = VIS_MEMKEYS;
        J.ooff = mk0; J.orows = min(P.bm, nmk - mk0);
        J.own = owner_range(P.R);
        J.own.slab0 = P.t; J.own.stride0 = P.s; J.own.magic0 = J.magic_t;
        const int y_first = mk0 / P.t, y_last = (mk0 + J.orows - 1) / P.t;
        const int nslabs = P.n - 1 - y_first;                        // later chunks: their reading rows see the block
        const int own_rows = (y_last - y_first + 1) * (P.s - P.R);    // memory and repetition rows of the block's chunks
        int a_lo = 0, a_hi = nslabs;
        if (P.split == 2) {
            const int a_mid = min(nslabs, max(0, (nslabs * P.R - own_rows) / (2 * P.R)));
            if (part == 0) a_hi = a_mid; else a_lo = a_mid;
            float* base = P.partials + ((long)(bh * P.split + part) * 2) * nmk * D;
            J.part_k = base; J.part_v = base + (long)nmk * D;
        }
        // reading rows of the later chunks, the farthest chunk first: the blocks of one (b,h) that run side by side
        // then stream the same rows at about the same time, and the tiles every key of the block sees come first
        J.z0 = y_first + a_hi; J.z1 = y_first;
        J.str.base0 = (y_first + a_hi) * P.s; J.str.n0 = (a_hi - a_lo) * P.R;
        J.str.slab0 = P.R; J.str.stride0 = -P.s; J.str.magic0 = magic_of(P.R);
        J.str.base1 = y_first * P.s + P.R; J.str.n1 = part == 0 ? own_rows : 0;
        J.str.slab1 = P.s - P.R; J.str.stride1 = P.s; J.str.magic1 = magic_of(P.s - P.R);
        if (P.R % 32 == 0) {
            J.pipe1 = min(a_hi - a_lo, max(0, J.z0 - y_last)) * (P.R / 32);   // chunks past the block's last one
            // whole tiles of one chunk: the reading rows, and the memory and repetition rows too when their slabs are tiled
            J.pipe_end = J.str.n0 / 32 + ((P.s - P.R) % 32 == 0 ? J.str.n1 / 32 : 0);
        }
    } else {
        u -= nMK * P.split;
        const int y = u / nRB, o0 = (u % nRB) * P.bm;
        J.vis = VIS_FROM_ROW;
        J.ooff = 0; J.orows = min(P.bm, P.R - o0);
        J.own = owner_range(y * P.s + o0);
        J.str = one_range(y * P.s + o0, P.R + P.t - o0);
        J.pipe0 = (J.orows + 30) / 32; J.pipe1 = (P.R + P.t - o0) / 32;   // rows from the block's last one on, whole tiles
        J.pipe_end = J.pipe1;
        J.pipe0 = min(J.pipe0, J.pipe1);
    }
    J.nstr = J.str.n0 + J.str.n1;
    return bh;
}

template <int D, int NW>
__global__ __launch_bounds__(64 * NW) void bwd_dkv_kernel(BwdParams P) {
    extern __shared__ __align__(16) bf16_t smem[];
    BwdJob J;
    const int bh = dkv_job_of<D>(P, blockIdx.x, J);
    const BwdTensors T = at_sequence(P.T, (long)bh * P.n * P.s, D);
    bwd_job<D, NW, PASS_DKV>(J, T, P.scale, P.sc, smem);
}

// dk, dv of the memory-zone keys = the partial sums of the workgroups that shared their streams, added in a
// fixed order (one thread per 8 head-dim columns of a key)
template <int D>
__global__ __launch_bounds__(256) void bwd_reduce_kernel(BwdParams P) {
    constexpr int CPR = D / 8;
    const int nmk = P.n * P.t;
    const long id = (long)blockIdx.x * 256 + threadIdx.x;
    const long key = id / CPR;                 // over nbh * nmk
    const int pc = (int)(id % CPR);
    if (key >= (long)P.nbh * nmk) return;
    const int bh = (int)(key / nmk), mk = (int)(key % nmk);
    const long row = (long)bh * P.n * P.s + (long)(mk / P.t) * P.s + P.R + mk % P.t;
    float sk[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, sv[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int part = 0; part < P.split; ++part) {
        const float* pk = P.partials + (((long)(bh * P.split + part) * 2) * nmk + mk) * D + pc * 8;
        const float* pv = pk + (long)nmk * D;
#pragma unroll
        for (int e = 0; e < 8; ++e) { sk[e] += pk[e]; sv[e] += pv[e]; }
    }
    uint4 ok, ov;
    ok.x = pack_bf16(sk[0], sk[1]); ok.y = pack_bf16(sk[2], sk[3]); ok.z = pack_bf16(sk[4], sk[5]); ok.w = pack_bf16(sk[6], sk[7]);
    ov.x = pack_bf16(sv[0], sv[1]); ov.y = pack_bf16(sv[2], sv[3]); ov.z = pack_bf16(sv[4], sv[5]); ov.w = pack_bf16(sv[6], sv[7]);
    *reinterpret_cast<uint4*>(P.T.dk + row * D + pc * 8) = ok;
    *reinterpret_cast<uint4*>(P.T.dv + row * D + pc * 8) = ov;
}

template <int D>
int launch_dkv(const BwdParams& P, hipStream_t st) {
    const long long nmk = (long long)P.n * P.t;
    const long long nMK = (nmk + P.bm - 1) / P.bm, nRB = (P.R + P.bm - 1) / P.bm;
    const long long grid = (long long)P.nbh * (nMK * P.split + (long long)P.n * nRB);
    int rc;
    if (P.bm == 128) rc = launch(bwd_dkv_kernel<D, 4>, grid, 256, BCfg<D>::smem_bytes(4, Stages<PASS_DKV, 4>::NS), P, st);
    else if (P.bm == 64) rc = launch(bwd_dkv_kernel<D, 2>, grid, 128, BCfg<D>::smem_bytes(2, Stages<PASS_DKV, 2>::NS), P, st);
    else rc = launch(bwd_dkv_kernel<D, 1>, grid, 64, BCfg<D>::smem_bytes(1, Stages<PASS_DKV, 1>::NS), P, st);
    if (rc != LOMA_OK || P.split == 1) return rc;
    return launch(bwd_reduce_kernel<D>, ((long long)P.nbh * nmk * (D / 8) + 255) / 256, 256, 0, P, st);
}

}  // namespace

int launch_bwd_dkv_pass(const BwdParams& P, int D, hipStream_t st) {
    return D == 128 ? launch_dkv<128>(P, st) : launch_dkv<64>(P, st);
}

bool mask_attn_bwd_mfma_fits(const Geometry& g) {
    // the slab divisions by multiplication are exact while (list index) * (slab length) < 2^32
    return (long long)g.S * g.s < (1LL << 32);
}

// Workgroups per block of memory keys in the dK/dV pass.  The first block streams the reading rows of every
// later chunk; when that one list is longer than what an average workgroup slot of the chip carries in the
// whole pass, the pass takes as long as that block, and the lists are shared out over two workgroups.
int mask_attn_bwd_stream_split(int nbh, const Geometry& g) {
    const int bm = mask_bwd_block_rows(g.R), nw = bm / 32;
    const long long slots = 256LL * (nw == 4 ? 1 : (nw == 2 ? 2 : 4));   // one wave per SIMD
    const long long nmk = (long long)g.n * g.t, nMK = (nmk + bm - 1) / bm;
    long long mem_tiles = 0, longest = 0;
    for (long long b = 0; b < nMK; ++b) {
        const long long mk0 = b * bm, rows = nmk - mk0 < bm ? nmk - mk0 : bm;
        const long long y_first = mk0 / g.t, y_last = (mk0 + rows - 1) / g.t;
        const long long tiles = ((g.n - 1 - y_first) * g.R + (y_last - y_first + 1) * (g.s - g.R) + 31) / 32;
        mem_tiles += tiles;
        if (tiles > longest) longest = tiles;
    }
    long long read_tiles = 0;
    for (int o0 = 0; o0 < g.R; o0 += bm) read_tiles += (g.R + g.t - o0 + 31) / 32;
    const long long total = (long long)nbh * (mem_tiles + g.n * read_tiles);
    return (g.n >= 4 && longest * slots * 100 > total * 115) ? 2 : 1;
}

// floats ahead of the partial sums: two per row, rounded up so that the partial sums start 16-byte aligned
inline size_t per_row_floats(size_t rows) { return (2 * rows + 3) / 4 * 4; }

size_t mask_attn_bwd_mfma_workspace_floats(int nbh, int D, const Geometry& g) {
    const size_t rows = (size_t)nbh * g.S;
    const int split = mask_attn_bwd_stream_split(nbh, g);
    return split > 1 ? per_row_floats(rows) + (size_t)nbh * split * 2 * (size_t)g.n * g.t * D : 2 * rows;
}

int launch_mask_attn_bwd_mfma(const void* q, const void* k, const void* v, const void* out, const float* lse,
                              const void* dout, void* dq, void* dk, void* dv, float* workspace,
                              int nbh, int D, const Geometry& g, float scale, hipStream_t st) {
    BwdParams P;
    P.T.q = (const bf16_t*)q; P.T.k = (const bf16_t*)k; P.T.v = (const bf16_t*)v; P.T.dout = (const bf16_t*)dout;
    P.T.out = (const bf16_t*)out; P.T.lse = lse;
    P.T.dq = (bf16_t*)dq; P.T.dk = (bf16_t*)dk; P.T.dv = (bf16_t*)dv;
    P.nbh = nbh; P.n = g.n; P.t = g.t; P.R = g.R; P.s = g.s;
    P.bm = mask_bwd_block_rows(g.R);
    P.scale = scale; P.sc = scale * LOG2E;
    const long long rows = (long long)nbh * g.S;
    P.T.delta = workspace; P.T.nl = workspace + rows;   // two floats per row, then the partial sums
    P.split = mask_attn_bwd_stream_split(nbh, g);
    P.partials = workspace + per_row_floats((size_t)rows);
    if (int rc = launch_bwd_dq_pass(P, D, st)) return rc;
    return launch_bwd_dkv_pass(P, D, st);
}

}  // namespace loma
