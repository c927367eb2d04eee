// Generic kernels: one wavefront per query row, fp32 arithmetic on the vector ALU, any
// head_dim that is a multiple of 8 up to 256, f32 or bf16 storage.  They serve the shapes
// the MFMA kernels do not take (f32 data, unusual head_dim) for all three entry points.
// The visible keys of a row are derived from (chunk, zone) exactly as in the mask of
// Sec. 4.3 (Eq. 1-3); masked keys are never read.  Softmax per Eq. 7, computed online over
// batches of 64 keys (one key per lane for the scores, one head-dim column per lane for PV).
#include "loma_internal.h"

namespace loma {
namespace {

constexpr int MAXD = 256;

struct RowSegs {  // visible keys of one query row: three row ranges, range 0 slab-strided
    const void *k0, *v0, *k1, *v1, *k2, *v2;
    int n0, n1, n2;
    int slab;
    long slab_stride;  // in elements
};

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

template <typename T>
__device__ __forceinline__ void seg_rows(const RowSegs& sg, int j, int D, const T*& kp, const T*& vp) {
    if (j < sg.n0) {
        const int a = j / sg.slab;
        const long off = (long)a * sg.slab_stride + (long)(j - a * sg.slab) * D;
        kp = static_cast<const T*>(sg.k0) + off; vp = static_cast<const T*>(sg.v0) + off;
    } else if (j < sg.n0 + sg.n1) {
        const long off = (long)(j - sg.n0) * D;
        kp = static_cast<const T*>(sg.k1) + off; vp = static_cast<const T*>(sg.v1) + off;
    } else {
        const long off = (long)(j - sg.n0 - sg.n1) * D;
        kp = static_cast<const T*>(sg.k2) + off; vp = static_cast<const T*>(sg.v2) + off;
    }
}

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
    return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

// One wavefront (blockDim.x == 64) computes one output row.
template <typename T>
__device__ void wave_attend(const T* q, const RowSegs& sg, int D, float scale, T* out, float* lse) {
    __shared__ float qs[MAXD];
    const int lane = threadIdx.x;
    for (int e = lane; e < D; e += 64) qs[e] = ld(q, e);
    __syncthreads();
    const int L = sg.n0 + sg.n1 + sg.n2;
    float m = -INFINITY, l = 0.f;
    float acc[MAXD / 64] = {0.f, 0.f, 0.f, 0.f};
    for (int base = 0; base < L; base += 64) {
        const int j = base + lane;
        float s = -INFINITY;
        if (j < L) {
            const T *kp, *vp;
            seg_rows<T>(sg, j, D, kp, vp);
            float a = 0.f;
            for (int e = 0; e < D; ++e) a = fmaf(qs[e], ld(kp, e), a);
            s = a * scale;
        }
        const float mn = fmaxf(m, wave_max(s));  // finite: every batch holds at least key `base`
        const float p = (j < L) ? expf(s - mn) : 0.f;
        const float alpha = expf(m - mn);        // m = -inf on the first batch gives 0
        l = l * alpha + wave_sum(p);
#pragma unroll
        for (int i = 0; i < MAXD / 64; ++i) acc[i] *= alpha;
        const int cnt = min(64, L - base);
        for (int jj = 0; jj < cnt; ++jj) {
            const float pj = __shfl(p, jj);
            const T *kp, *vp;
            seg_rows<T>(sg, base + jj, D, kp, vp);
#pragma unroll
            for (int i = 0; i < MAXD / 64; ++i) {
                const int e = lane + 64 * i;
                if (e < D) acc[i] = fmaf(pj, ld(vp, e), acc[i]);
            }
        }
        m = mn;
    }
#pragma unroll
    for (int i = 0; i < MAXD / 64; ++i) {
        const int e = lane + 64 * i;
        if (e < D) st(out, e, acc[i] / l);
    }
    if (lse != nullptr && lane == 0) *lse = m + logf(l);
}

template <typename T>
__global__ __launch_bounds__(64) void mask_rows_kernel(const T* q, const T* k, const T* v, T* out, float* lse,
                                                       int D, int t, int R, int s, int S, float scale) {
    const long row = blockIdx.x;            // over B*H*S
    const long seq = (row / S) * S;         // first row of this (b,h)
    const int p = (int)(row - seq);
    const int y = p / s, o = p - y * s;
    const long chunk = seq + (long)y * s;
    RowSegs sg;
    sg.k0 = sg.k1 = sg.k2 = k; sg.v0 = sg.v1 = sg.v2 = v;
    sg.n0 = sg.n1 = sg.n2 = 0; sg.slab = 1; sg.slab_stride = 0;
    if (o < R) {                 // reading row: earlier memory zones, then own causal prefix
        sg.k0 = k + (seq + R) * D; sg.v0 = v + (seq + R) * D;
        sg.n0 = y * t; sg.slab = t; sg.slab_stride = (long)s * D;
        sg.k1 = k + chunk * D; sg.v1 = v + chunk * D; sg.n1 = o + 1;
    } else if (o < R + t) {      // memory row: own reading + memory zone
        sg.k1 = k + chunk * D; sg.v1 = v + chunk * D; sg.n1 = R + t;
    } else {                     // repetition row: own memory zone, then itself
        sg.k1 = k + (chunk + R) * D; sg.v1 = v + (chunk + R) * D; sg.n1 = t;
        sg.k2 = k + row * D; sg.v2 = v + row * D; sg.n2 = 1;
    }
    wave_attend<T>(q + row * D, sg, D, scale, out + row * D, lse ? lse + row : nullptr);
}

template <typename T>
__global__ __launch_bounds__(64) void compress_rows_kernel(const T* q_mem, const T* k_mem, const T* v_mem,
                                                           const T* k_read, const T* v_read, T* k_cache, T* v_cache,
                                                           T* out, int D, int t, int R, long cache_row0,
                                                           long cache_rows, float scale) {
    const long row = blockIdx.x;  // over B*H*t
    const long bh = row / t;
    RowSegs sg;
    sg.k0 = sg.v0 = nullptr; sg.n0 = 0; sg.slab = 1; sg.slab_stride = 0;
    sg.k1 = k_read + bh * R * D; sg.v1 = v_read + bh * R * D; sg.n1 = R;
    sg.k2 = k_mem + bh * t * D; sg.v2 = v_mem + bh * t * D; sg.n2 = t;
    wave_attend<T>(q_mem + row * D, sg, D, scale, out + row * D, nullptr);
    // splice this <m> token's K/V into the compressed cache
    const long dst = (bh * cache_rows + cache_row0 + (row - bh * t)) * D;
    for (int e = threadIdx.x; e < D; e += 64) {
        k_cache[dst + e] = k_mem[row * D + e];
        v_cache[dst + e] = v_mem[row * D + e];
    }
}

template <typename T>
__global__ __launch_bounds__(64) void decode_rows_kernel(const T* q, const T* k_new, const T* v_new,
                                                         const T* k_cache, const T* v_cache, T* k_read, T* v_read,
                                                         T* out, int D, int R, int n_mem_keys, long cache_rows,
                                                         int read_fill, float scale) {
    const long bh = blockIdx.x;
    RowSegs sg;
    sg.k0 = k_cache ? k_cache + bh * cache_rows * D : nullptr;
    sg.v0 = v_cache ? v_cache + bh * cache_rows * D : nullptr;
    sg.n0 = n_mem_keys; sg.slab = 1 << 30; sg.slab_stride = 0;
    sg.k1 = k_read + bh * R * D; sg.v1 = v_read + bh * R * D; sg.n1 = read_fill;
    sg.k2 = k_new ? k_new + bh * D : nullptr; sg.v2 = v_new ? v_new + bh * D : nullptr;
    sg.n2 = k_new ? 1 : 0;
    wave_attend<T>(q + bh * D, sg, D, scale, out + bh * D, nullptr);
    if (k_new) {  // the new token joins the reading zone (it was read from k_new above, not from here)
        const long dst = (bh * R + read_fill) * D;
        for (int e = threadIdx.x; e < D; e += 64) {
            k_read[dst + e] = k_new[bh * D + e];
            v_read[dst + e] = v_new[bh * D + e];
        }
    }
}

// one wave per new token: memory keys, live reading rows, new tokens 0..i (read from k_new/v_new);
// the wave also appends its token to the reading zone (rows nobody reads in this launch)
template <typename T>
__global__ __launch_bounds__(64) void prefill_rows_kernel(const T* q, const T* k_new, const T* v_new,
                                                          const T* k_cache, const T* v_cache, T* k_read, T* v_read,
                                                          T* out, float* lse, int D, int R, int n_mem_keys,
                                                          long cache_rows, int read_fill, int n_new, float scale) {
    const long bh = blockIdx.x / n_new;
    const int i = blockIdx.x % n_new;
    RowSegs sg;
    sg.k0 = k_cache ? k_cache + bh * cache_rows * D : nullptr;
    sg.v0 = v_cache ? v_cache + bh * cache_rows * D : nullptr;
    sg.n0 = n_mem_keys; sg.slab = 1 << 30; sg.slab_stride = 0;
    sg.k1 = k_read + bh * R * D; sg.v1 = v_read + bh * R * D; sg.n1 = read_fill;
    sg.k2 = k_new + bh * n_new * D; sg.v2 = v_new + bh * n_new * D; sg.n2 = i + 1;
    const long row = bh * n_new + i;
    wave_attend<T>(q + row * D, sg, D, scale, out + row * D, lse ? lse + row : nullptr);
    const long dst = (bh * R + read_fill + i) * D;
    for (int e = threadIdx.x; e < D; e += 64) {
        k_read[dst + e] = k_new[row * D + e];
        v_read[dst + e] = v_new[row * D + e];
    }
}

inline int check_launch(long long grid) {
    return grid > 0x7fffffffLL ? LOMA_ERR_UNSUPPORTED : LOMA_OK;
}
inline int after_launch() { return hipGetLastError() == hipSuccess ? LOMA_OK : LOMA_ERR_LAUNCH; }

}  // namespace

int launch_mask_attn_generic(const void* q, const void* k, const void* v, void* out, float* lse,
                             int nbh, int D, const Geometry& g, float scale, int dtype, hipStream_t st) {
    const long long grid = (long long)nbh * g.S;
    if (int rc = check_launch(grid)) return rc;
    if (dtype == LOMA_F32)
        hipLaunchKernelGGL(mask_rows_kernel<float>, dim3((unsigned)grid), dim3(64), 0, st,
                           (const float*)q, (const float*)k, (const float*)v, (float*)out, lse,
                           D, g.t, g.R, g.s, g.S, scale);
    else
        hipLaunchKernelGGL(mask_rows_kernel<uint16_t>, dim3((unsigned)grid), dim3(64), 0, st,
                           (const uint16_t*)q, (const uint16_t*)k, (const uint16_t*)v, (uint16_t*)out, lse,
                           D, g.t, g.R, g.s, g.S, scale);
    return after_launch();
}

int launch_compress_generic(const void* q_mem, const void* k_mem, const void* v_mem,
                            const void* k_read, const void* v_read, void* k_memcache, void* v_memcache,
                            void* out, int nbh, int D, int t, int c, int n_mem_chunks, int mem_capacity,
                            float scale, int dtype, hipStream_t st) {
    const long long grid = (long long)nbh * t;
    if (int rc = check_launch(grid)) return rc;
    const long row0 = (long)n_mem_chunks * t;
    if (dtype == LOMA_F32)
        hipLaunchKernelGGL(compress_rows_kernel<float>, dim3((unsigned)grid), dim3(64), 0, st,
                           (const float*)q_mem, (const float*)k_mem, (const float*)v_mem, (const float*)k_read,
                           (const float*)v_read, (float*)k_memcache, (float*)v_memcache, (float*)out,
                           D, t, t * c, row0, (long)mem_capacity, scale);
    else
        hipLaunchKernelGGL(compress_rows_kernel<uint16_t>, dim3((unsigned)grid), dim3(64), 0, st,
                           (const uint16_t*)q_mem, (const uint16_t*)k_mem, (const uint16_t*)v_mem,
                           (const uint16_t*)k_read, (const uint16_t*)v_read, (uint16_t*)k_memcache,
                           (uint16_t*)v_memcache, (uint16_t*)out, D, t, t * c, row0, (long)mem_capacity, scale);
    return after_launch();
}

int launch_decode_generic(const void* q, const void* k_new, const void* v_new,
                          const void* k_memcache, const void* v_memcache, void* k_read, void* v_read,
                          void* out, int nbh, int D, int R, int n_mem_keys, int mem_capacity, int read_fill,
                          float scale, int dtype, hipStream_t st) {
    if (int rc = check_launch(nbh)) return rc;
    if (dtype == LOMA_F32)
        hipLaunchKernelGGL(decode_rows_kernel<float>, dim3((unsigned)nbh), dim3(64), 0, st,
                           (const float*)q, (const float*)k_new, (const float*)v_new, (const float*)k_memcache,
                           (const float*)v_memcache, (float*)k_read, (float*)v_read, (float*)out,
                           D, R, n_mem_keys, (long)mem_capacity, read_fill, scale);
    else
        hipLaunchKernelGGL(decode_rows_kernel<uint16_t>, dim3((unsigned)nbh), dim3(64), 0, st,
                           (const uint16_t*)q, (const uint16_t*)k_new, (const uint16_t*)v_new,
                           (const uint16_t*)k_memcache, (const uint16_t*)v_memcache, (uint16_t*)k_read,
                           (uint16_t*)v_read, (uint16_t*)out, D, R, n_mem_keys, (long)mem_capacity, read_fill, scale);
    return after_launch();
}

int launch_prefill_generic(const void* q, const void* k_new, const void* v_new,
                           const void* k_memcache, const void* v_memcache, void* k_read, void* v_read,
                           void* out, float* lse, int nbh, int D, int R, int n_mem_keys, int mem_capacity,
                           int read_fill, int n_new, float scale, int dtype, hipStream_t st) {
    const long long grid = (long long)nbh * n_new;
    if (int rc = check_launch(grid)) return rc;
    if (dtype == LOMA_F32)
        hipLaunchKernelGGL(prefill_rows_kernel<float>, dim3((unsigned)grid), dim3(64), 0, st,
                           (const float*)q, (const float*)k_new, (const float*)v_new, (const float*)k_memcache,
                           (const float*)v_memcache, (float*)k_read, (float*)v_read, (float*)out, lse,
                           D, R, n_mem_keys, (long)mem_capacity, read_fill, n_new, scale);
    else
        hipLaunchKernelGGL(prefill_rows_kernel<uint16_t>, dim3((unsigned)grid), dim3(64), 0, st,
                           (const uint16_t*)q, (const uint16_t*)k_new, (const uint16_t*)v_new,
                           (const uint16_t*)k_memcache, (const uint16_t*)v_memcache, (uint16_t*)k_read,
                           (uint16_t*)v_read, (uint16_t*)out, lse, D, R, n_mem_keys, (long)mem_capacity, read_fill,
                           n_new, scale);
    return after_launch();
}

}  // namespace loma
