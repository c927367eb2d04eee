// Gradients of the mask pass, generic kernels: one wavefront per row, fp32 arithmetic on the
// vector ALU, f32 or bf16 storage, any head_dim that is a multiple of 8 up to 256.
//
// With W the attention weights of Sec. 4.4 (Eq. 5-7; zero on masked pairs), G the gradient of the
// output and delta_i = G_i . O_i:
//     dV_j = sum_i W_ij G_i,   dA_ij = W_ij (G_i . V_j - delta_i),
//     dQ_i = scale sum_j dA_ij K_j,   dK_j = scale sum_i dA_ij Q_i.
// W_ij = exp(scale Q_i.K_j - LSE_i) is rebuilt from the forward pass's log-sum-exp.
// The dQ kernel walks the keys a row sees (the mask of Sec. 4.3, Eq. 1-3, by rows); the dK/dV
// kernel walks the queries that see a key (the same mask by columns):
//     reading-zone key o of chunk y:  reading rows o..R-1 and the memory rows of chunk y;
//     memory-zone key of chunk y:     memory and repetition rows of chunk y, and the reading rows
//                                     of every later chunk;
//     repetition-zone key:            its own row only.
// Every sum has one owner, so there are no atomics and the result is deterministic.
#include "loma_internal.h"

namespace loma {
namespace {

constexpr int MAXD = 256;

template <typename T> __device__ __forceinline__ float ld(const T* p, long i);
template <> __device__ __forceinline__ float ld<float>(const float* p, long i) { return p[i]; }
template <> __device__ __forceinline__ float ld<uint16_t>(const uint16_t* p, long i) {
    return __uint_as_float(((uint32_t)p[i]) << 16);
}
template <typename T> __device__ __forceinline__ void st(T* p, long i, float x);
template <> __device__ __forceinline__ void st<float>(float* p, long i, float x) { p[i] = x; }
template <> __device__ __forceinline__ void st<uint16_t>(uint16_t* p, long i, float x) {
    uint32_t u = __float_as_uint(x);
    u += 0x7fffu + ((u >> 16) & 1u);  // round to nearest even (finite values)
    p[i] = (uint16_t)(u >> 16);
}

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

// delta[row] = dout[row] . out[row]; one wave per row
template <typename T>
__global__ __launch_bounds__(64) void bwd_delta_kernel(const T* out, const T* dout, float* delta, int D) {
    const long row = blockIdx.x;
    float a = 0.f;
    for (int e = threadIdx.x; e < D; e += 64) a = fmaf(ld(out, row * D + e), ld(dout, row * D + e), a);
    a = wave_sum(a);
    if (threadIdx.x == 0) delta[row] = a;
}

// Up to two runs of rows of one sequence: run 0 is `n0` rows in slabs of `slab` rows `stride` rows
// apart starting at row `r0`; run 1 is `n1` consecutive rows from row `r1`.
struct RowRuns {
    long r0, r1;
    int n0, n1, slab;
    long stride;
    __device__ __forceinline__ long row(int j) const {
        if (j < n0) { const int a = j / slab; return r0 + (long)a * stride + (j - a * slab); }
        return r1 + (j - n0);
    }
};

// One wave per query row: dq = scale * sum_j dA_j k_j over the keys the row sees.
template <typename T>
__global__ __launch_bounds__(64) void bwd_dq_rows_kernel(const T* q, const T* k, const T* v, const T* dout,
                                                         const float* lse, const float* delta, T* dq,
                                                         int D, int t, int R, int s, int S, float scale) {
    __shared__ float qs[MAXD], gs[MAXD];
    const long row = blockIdx.x;      // over B*H*S
    const long seq = (row / S) * S;   // first row of this (b,h)
    const int p = (int)(row - seq);
    const int y = p / s, o = p - y * s;
    const long chunk = seq + (long)y * s;
    RowRuns kr;
    kr.r0 = kr.r1 = 0; kr.n0 = kr.n1 = 0; kr.slab = 1; kr.stride = 0;
    bool self = false;
    if (o < R) {             // reading row: earlier memory zones, own causal prefix
        kr.r0 = seq + R; kr.n0 = y * t; kr.slab = t; kr.stride = s;
        kr.r1 = chunk; kr.n1 = o + 1;
    } else if (o < R + t) {  // memory row: own reading and memory zone
        kr.r1 = chunk; kr.n1 = R + t;
    } else {                 // repetition row: own memory zone, then itself
        kr.r1 = chunk + R; kr.n1 = t; self = true;
    }
    const int lane = threadIdx.x;
    for (int e = lane; e < D; e += 64) { qs[e] = ld(q, row * D + e); gs[e] = ld(dout, row * D + e); }
    __syncthreads();
    const float L = lse[row], dl = delta[row];
    const int n = kr.n0 + kr.n1 + (self ? 1 : 0);
    float acc[MAXD / 64] = {0.f, 0.f, 0.f, 0.f};
    for (int base = 0; base < n; base += 64) {
        const int j = base + lane;
        float da = 0.f;
        long krow = 0;
        if (j < n) {
            krow = (self && j == n - 1) ? row : kr.row(j);
            float a = 0.f, dw = 0.f;
            for (int e = 0; e < D; ++e) {
                a = fmaf(qs[e], ld(k, krow * D + e), a);
                dw = fmaf(gs[e], ld(v, krow * D + e), dw);
            }
            da = expf(a * scale - L) * (dw - dl);
        }
        const int cnt = min(64, n - base);
        for (int jj = 0; jj < cnt; ++jj) {
            const float dj = __shfl(da, jj);
            const long rj = __shfl(krow, jj);
#pragma unroll
            for (int i = 0; i < MAXD / 64; ++i) {
                const int e = lane + 64 * i;
                if (e < D) acc[i] = fmaf(dj, ld(k, rj * D + e), acc[i]);
            }
        }
    }
#pragma unroll
    for (int i = 0; i < MAXD / 64; ++i) {
        const int e = lane + 64 * i;
        if (e < D) st(dq, row * D + e, acc[i] * scale);
    }
}

// One wave per key row: dk = scale * sum_i dA_i q_i, dv = sum_i W_i dout_i over the queries that see it.
template <typename T>
__global__ __launch_bounds__(64) void bwd_dkv_rows_kernel(const T* q, const T* k, const T* v, const T* dout,
                                                          const float* lse, const float* delta, T* dk, T* dv,
                                                          int D, int t, int R, int s, int S, int nchunks, float scale) {
    __shared__ float ks[MAXD], vs[MAXD];
    const long row = blockIdx.x;
    const long seq = (row / S) * S;
    const int p = (int)(row - seq);
    const int y = p / s, o = p - y * s;
    const long chunk = seq + (long)y * s;
    RowRuns qr;
    qr.r0 = qr.r1 = 0; qr.n0 = qr.n1 = 0; qr.slab = 1; qr.stride = 0;
    if (o < R) {             // reading-zone key: own reading rows from it on, own memory rows
        qr.r1 = chunk + o; qr.n1 = R + t - o;
    } else if (o < R + t) {  // memory-zone key: reading rows of later chunks; own memory and repetition rows
        qr.r0 = chunk + s; qr.n0 = (nchunks - 1 - y) * R; qr.slab = R; qr.stride = s;
        qr.r1 = chunk + R; qr.n1 = s - R;
    } else {                 // repetition-zone key: itself
        qr.r1 = row; qr.n1 = 1;
    }
    const int lane = threadIdx.x;
    for (int e = lane; e < D; e += 64) { ks[e] = ld(k, row * D + e); vs[e] = ld(v, row * D + e); }
    __syncthreads();
    const int n = qr.n0 + qr.n1;
    float acck[MAXD / 64] = {0.f, 0.f, 0.f, 0.f}, accv[MAXD / 64] = {0.f, 0.f, 0.f, 0.f};
    for (int base = 0; base < n; base += 64) {
        const int i = base + lane;
        float w = 0.f, da = 0.f;
        long qrow = 0;
        if (i < n) {
            qrow = qr.row(i);
            float a = 0.f, dw = 0.f;
            for (int e = 0; e < D; ++e) {
                a = fmaf(ld(q, qrow * D + e), ks[e], a);
                dw = fmaf(ld(dout, qrow * D + e), vs[e], dw);
            }
            w = expf(a * scale - lse[qrow]);
            da = w * (dw - delta[qrow]);
        }
        const int cnt = min(64, n - base);
        for (int ii = 0; ii < cnt; ++ii) {
            const float wi = __shfl(w, ii), di = __shfl(da, ii);
            const long ri = __shfl(qrow, ii);
#pragma unroll
            for (int x = 0; x < MAXD / 64; ++x) {
                const int e = lane + 64 * x;
                if (e < D) {
                    accv[x] = fmaf(wi, ld(dout, ri * D + e), accv[x]);
                    acck[x] = fmaf(di, ld(q, ri * D + e), acck[x]);
                }
            }
        }
    }
#pragma unroll
    for (int x = 0; x < MAXD / 64; ++x) {
        const int e = lane + 64 * x;
        if (e < D) { st(dk, row * D + e, acck[x] * scale); st(dv, row * D + e, accv[x]); }
    }
}

inline int after_launch() { return hipGetLastError() == hipSuccess ? LOMA_OK : LOMA_ERR_LAUNCH; }

template <typename T>
int launch_all(const void* q, const void* k, const void* v, const void* out, const float* lse, const void* dout,
               void* dq, void* dk, void* dv, float* delta, long long rows, int D, const Geometry& g, float scale,
               hipStream_t st) {
    const dim3 grid((unsigned)rows), block(64);
    hipLaunchKernelGGL(bwd_delta_kernel<T>, grid, block, 0, st, (const T*)out, (const T*)dout, delta, D);
    if (int rc = after_launch()) return rc;
    hipLaunchKernelGGL(bwd_dq_rows_kernel<T>, grid, block, 0, st, (const T*)q, (const T*)k, (const T*)v,
                       (const T*)dout, lse, (const float*)delta, (T*)dq, D, g.t, g.R, g.s, g.S, scale);
    if (int rc = after_launch()) return rc;
    hipLaunchKernelGGL(bwd_dkv_rows_kernel<T>, grid, block, 0, st, (const T*)q, (const T*)k, (const T*)v,
                       (const T*)dout, lse, (const float*)delta, (T*)dk, (T*)dv, D, g.t, g.R, g.s, g.S, g.n, scale);
    return after_launch();
}

}  // namespace

int launch_mask_attn_bwd_generic(const void* q, const void* k, const void* v, const void* out, const float* lse,
                                 const void* dout, void* dq, void* dk, void* dv, float* delta,
                                 int nbh, int D, const Geometry& g, float scale, int dtype, hipStream_t st) {
    const long long rows = (long long)nbh * g.S;
    if (rows > 0x7fffffffLL) return LOMA_ERR_UNSUPPORTED;
    if (dtype == LOMA_F32)
        return launch_all<float>(q, k, v, out, lse, dout, dq, dk, dv, delta, rows, D, g, scale, st);
    return launch_all<uint16_t>(q, k, v, out, lse, dout, dq, dk, dv, delta, rows, D, g, scale, st);
}

}  // namespace loma
