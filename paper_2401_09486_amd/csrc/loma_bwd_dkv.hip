// dK/dV pass of the mask pass's gradients on the matrix cores (engine and notation: loma_bwd_engine.h),
// the per-row delta that both passes read, and the entry that runs all three.
#include "loma_bwd_engine.h"

namespace loma {
namespace {

// dK/dV pass: per (b,h) the blocks of memory keys (longest first: the first block is seen by every later
// chunk), then the reading-zone key blocks of every chunk.  Repetition-zone keys belong to the dQ pass.
template <int D, int NW>
__global__ __launch_bounds__(64 * NW) void bwd_dkv_kernel(BwdParams P) {
    extern __shared__ __align__(16) bf16_t smem[];
    const int nMK = (P.n * P.t + P.bm - 1) / P.bm;    // blocks of memory keys
    const int nRB = (P.R + P.bm - 1) / P.bm;          // reading-zone key blocks per chunk
    int bh, u;
    split_block(blockIdx.x, P.nbh, nMK + P.n * nRB, bh, u);
    BwdJob J;
    J.rep = 0; J.t = P.t; J.magic_t = magic_of(P.t); J.y_first = 0; J.cb = 0;
    if (u < nMK) {
        const int mk0 = u * P.bm;
        J.vis = VIS_MEMKEYS;
        J.ooff = mk0; J.orows = min(P.bm, P.n * P.t - mk0);
        J.own = owner_range(P.R);
        J.own.slab0 = P.t; J.own.stride0 = P.s; J.own.magic0 = J.magic_t;
        const int y_first = mk0 / P.t, y_last = (mk0 + J.orows - 1) / P.t;
        J.y_first = y_first;
        J.str.base0 = (y_first + 1) * P.s; J.str.n0 = (P.n - 1 - y_first) * P.R;
        J.str.slab0 = P.R; J.str.stride0 = P.s; J.str.magic0 = magic_of(P.R);
        J.str.base1 = y_first * P.s + P.R; J.str.n1 = (y_last - y_first + 1) * (P.s - P.R);
        J.str.slab1 = P.s - P.R; J.str.stride1 = P.s; J.str.magic1 = magic_of(P.s - P.R);
    } else {
        u -= nMK;
        const int y = u / nRB, o0 = (u % nRB) * P.bm;
        J.vis = VIS_FROM_ROW;
        J.ooff = 0; J.orows = min(P.bm, P.R - o0);
        J.own = owner_range(y * P.s + o0);
        J.str = one_range(y * P.s + o0, P.R + P.t - o0);
    }
    J.nstr = J.str.n0 + J.str.n1;
    const BwdTensors T = at_sequence(P.T, (long)bh * P.n * P.s, D);
    bwd_job<D, NW, PASS_DKV>(J, T, P.scale, P.sc, smem);
}

// Per row: delta = dout . out and nl = -lse * log2(e) (the form the exp2 of the passes wants); rows in the
// row layout (lane = 16-byte piece).
template <int D>
__global__ __launch_bounds__(256) void bwd_delta_kernel(const bf16_t* out, const bf16_t* dout, const float* lse,
                                                        float* delta, float* nl, long rows) {
    constexpr int CPR = D / 8;
    const long row = ((long)blockIdx.x * 256 + threadIdx.x) / CPR;
    const int pc = threadIdx.x % CPR;
    const long rc = row < rows ? row : rows - 1;
    const u32x4 a = *reinterpret_cast<const u32x4*>(out + rc * D + pc * 8);
    const u32x4 b = *reinterpret_cast<const u32x4*>(dout + rc * D + pc * 8);
    const float s = row_sum<CPR>(dot8(a, b));
    if (pc == 0 && row < rows) {
        delta[row] = s;
        nl[row] = -lse[row] * LOG2E;
    }
}

template <int D>
int launch_dkv(const BwdParams& P, hipStream_t st) {
    const long long nMK = ((long long)P.n * P.t + P.bm - 1) / P.bm, nRB = (P.R + P.bm - 1) / P.bm;
    const long long grid = (long long)P.nbh * (nMK + (long long)P.n * nRB);
    if (P.bm == 128) return launch(bwd_dkv_kernel<D, 4>, grid, 256, BCfg<D>::smem_bytes(4, Stages<PASS_DKV, 4>::NS), P, st);
    if (P.bm == 64) return launch(bwd_dkv_kernel<D, 2>, grid, 128, BCfg<D>::smem_bytes(2, Stages<PASS_DKV, 2>::NS), P, st);
    return launch(bwd_dkv_kernel<D, 1>, grid, 64, BCfg<D>::smem_bytes(1, Stages<PASS_DKV, 1>::NS), P, st);
}

template <int D>
int launch_delta(const void* out, const float* lse, const BwdParams& P, long long rows, hipStream_t st) {
    const long long grid = (rows * (D / 8) + 255) / 256;
    if (grid > 0x7fffffffLL) return LOMA_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(bwd_delta_kernel<D>, dim3((unsigned)grid), dim3(256), 0, st, (const bf16_t*)out, P.T.dout, lse,
                       const_cast<float*>(P.T.delta), const_cast<float*>(P.T.nl), (long)rows);
    return hipGetLastError() == hipSuccess ? LOMA_OK : LOMA_ERR_LAUNCH;
}

}  // namespace

int launch_bwd_dkv_pass(const BwdParams& P, int D, hipStream_t st) {
    return D == 128 ? launch_dkv<128>(P, st) : launch_dkv<64>(P, st);
}

bool mask_attn_bwd_mfma_fits(const Geometry& g) {
    // the slab divisions by multiplication are exact while (list index) * (slab length) < 2^32
    return (long long)g.S * g.s < (1LL << 32);
}

int launch_mask_attn_bwd_mfma(const void* q, const void* k, const void* v, const void* out, const float* lse,
                              const void* dout, void* dq, void* dk, void* dv, float* workspace,
                              int nbh, int D, const Geometry& g, float scale, hipStream_t st) {
    BwdParams P;
    P.T.q = (const bf16_t*)q; P.T.k = (const bf16_t*)k; P.T.v = (const bf16_t*)v; P.T.dout = (const bf16_t*)dout;
    P.T.dq = (bf16_t*)dq; P.T.dk = (bf16_t*)dk; P.T.dv = (bf16_t*)dv;
    P.nbh = nbh; P.n = g.n; P.t = g.t; P.R = g.R; P.s = g.s;
    P.bm = mask_block_rows(g.R);
    P.scale = scale; P.sc = scale * LOG2E;
    const long long rows = (long long)nbh * g.S;
    P.T.delta = workspace; P.T.nl = workspace + rows;   // two floats per row
    if (int rc = D == 128 ? launch_delta<128>(out, lse, P, rows, st) : launch_delta<64>(out, lse, P, rows, st)) return rc;
    if (int rc = launch_bwd_dq_pass(P, D, st)) return rc;
    return launch_bwd_dkv_pass(P, D, st);
}

}  // namespace loma
