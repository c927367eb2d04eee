// Split-K decode attention for the generation form (Sec. 3.1 steps 1 and 3; Appendix A,
// one new token against the compressed cache).  The query of each (b,h) sees
//     [ n_mem_chunks*t memory-zone KVs | read_fill live reading-zone KVs | the new token ]
// with no mask, so the step is one pass over K and V: HBM-bound (2 flop per byte).
//
// Grid = (key splits, B*H).  A workgroup streams its key range with 16-byte loads: D/8 lanes
// cover one 2*D-byte row, so a wave-wide load instruction fetches 64/(D/8) whole rows, fully
// coalesced; each wave keeps 8 K and 8 V loads in flight.  Scores use packed bf16 dot products
// with fp32 accumulation and a butterfly over the lanes of a row; every lane group carries its
// own online-softmax state (m, l, acc[8]) so the loop needs no cross-group traffic.  The lane
// groups of a wave are merged with lane permutes, the waves through LDS.  Two shapes:
//   few (b,h) pairs (< 1024): 16 waves per workgroup, one workgroup per (b,h) when that already
//       gives one workgroup per CU -- a single launch, no partial results in HBM;
//   many (b,h) pairs: 4 waves per workgroup, thousands of workgroups.
// When one (b,h) is split over several workgroups, the partial (m, l, acc) go to the workspace
// and a second tiny kernel merges them in a fixed order (deterministic, no atomics).  The new
// token's K/V are read from k_new/v_new and appended to the reading zone by split 0 -- no
// workgroup reads the row another one is writing.
#include <mutex>
#include <type_traits>

#include "loma_internal.h"
#include "loma_rope.h"

namespace loma {
namespace {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef uint16_t bf16_t;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

constexpr float LOG2E = 1.4426950408889634f;
constexpr int DEC_UNROLL = 8;          // row-loads in flight per wave, for K and for V
constexpr int DEC_SMALL_NBH = 1024;    // below: 16-wave workgroups, ~1 per CU; from here on: 4-wave workgroups
constexpr int DEC_TARGET_WGS_16 = 256;
constexpr int DEC_TARGET_WGS_4 = 4096;

// Pointer tables of the layered form: one device pointer per layer and tensor, read by the kernel.
struct LayerTables {
    const bf16_t* const* q;
    const bf16_t* const* k_new;
    const bf16_t* const* v_new;
    const bf16_t* const* k_mem;
    const bf16_t* const* v_mem;
    bf16_t* const* k_read;
    bf16_t* const* v_read;
    bf16_t* const* out;
};

struct DecodeParams {
    const bf16_t *q, *k_new, *v_new, *k_mem, *v_mem;
    bf16_t *k_read, *v_read, *out;
    LayerTables tab;     // layered form only
    long ws_layer_floats;   // floats of workspace per layer (layered form)
    float* ws_acc;   // [nbh * nsplit, D]
    float* ws_ml;    // [nbh * nsplit, 2]
    long mem_rows;   // mem_capacity
    int R, n_mem, n_read, has_new, L;
    int nsplit, keys_per_split;
    float sc;        // scale * log2(e)
};

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
// bit pattern of two packed bf16 -> vector operand (taken by value: element references of
// ext-vectors must not be handed to __builtin_bit_cast directly)
__device__ __forceinline__ bf16x2 as_bf16x2(uint32_t w) { return __builtin_bit_cast(bf16x2, w); }
__device__ __forceinline__ uint16_t f32_to_bf16(float x) {
    uint32_t u = __float_as_uint(x);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// sum over the LPR consecutive lanes that share a key row; every lane gets the total.
// DPP lane permutes inside a row of 16 lanes: swap neighbours, swap pairs, mirror 8, mirror 16.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x) {
    const int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false);
    return x + __int_as_float(y);
}
template <int LPR>
__device__ __forceinline__ float row_sum(float x) {
    x = dpp_add<0xB1>(x);   // quad_perm [1,0,3,2]
    x = dpp_add<0x4E>(x);   // quad_perm [2,3,0,1]
    x = dpp_add<0x141>(x);  // row_half_mirror
    if (LPR == 16) x = dpp_add<0x140>(x);  // row_mirror
    return x;
}

// LAYERED: blockIdx.z is a layer; its eight tensors come from the pointer tables, everything else (shapes,
// cache state, split plan) is shared by the layers, so a layer's result is computed exactly as by a call of its own.
// ROPE: q and the new token's K arrive unrotated and are turned by the new token's position id as they are
// loaded (the cache holds rotated K); the appended K row is the rotated one.
struct NoRope {};
template <int D, int DEC_WAVES, bool LAYERED, bool ROPE>
__global__ __launch_bounds__(64 * DEC_WAVES) void decode_split_kernel(DecodeParams P,
                                                                      std::conditional_t<ROPE, RopeTable, NoRope> RT) {
    constexpr int LPR = D / 8;            // lanes per key row
    constexpr int RPL = 64 / LPR;         // rows per wave-wide load
    constexpr int KPW = RPL * DEC_UNROLL; // keys per wave iteration
    __shared__ float sm_acc[DEC_WAVES][D];
    __shared__ float sm_m[DEC_WAVES], sm_l[DEC_WAVES];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int sp = blockIdx.x;
    const long bh = blockIdx.y;
    const int col = lane % LPR, sub = lane / LPR;
    const int kbeg = sp * P.keys_per_split;
    const int kend = min(P.L, kbeg + P.keys_per_split);

    if constexpr (LAYERED) {
        const int layer = blockIdx.z;
        P.q = P.tab.q[layer];
        P.k_new = P.has_new ? P.tab.k_new[layer] : nullptr;
        P.v_new = P.has_new ? P.tab.v_new[layer] : nullptr;
        P.k_mem = P.n_mem > 0 ? P.tab.k_mem[layer] : nullptr;
        P.v_mem = P.n_mem > 0 ? P.tab.v_mem[layer] : nullptr;
        P.k_read = P.tab.k_read[layer];
        P.v_read = P.tab.v_read[layer];
        P.out = P.tab.out[layer];
        if (P.ws_acc != nullptr) { P.ws_acc += layer * P.ws_layer_floats; P.ws_ml += layer * P.ws_layer_floats; }
    }
    const bf16_t* kmem = P.k_mem + bh * P.mem_rows * D;
    const bf16_t* vmem = P.v_mem + bh * P.mem_rows * D;
    const bf16_t* kread = P.k_read + bh * (long)P.R * D;
    const bf16_t* vread = P.v_read + bh * (long)P.R * D;
    const bf16_t* knew = P.k_new + bh * D;
    const bf16_t* vnew = P.v_new + bh * D;

    uint4 qv = *reinterpret_cast<const uint4*>(P.q + bh * D + col * 8);
    if constexpr (ROPE) {
        const u32x4 r = rope::load_rotated_piece<D>(P.q + bh * D, col, RT.pos_first, RT);
        qv = uint4{r[0], r[1], r[2], r[3]};
    }
    const bf16x2 q0 = as_bf16x2(qv.x), q1 = as_bf16x2(qv.y), q2 = as_bf16x2(qv.z), q3 = as_bf16x2(qv.w);

    float m = -INFINITY, l = 0.f;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    for (int base = kbeg + w * KPW; base < kend; base += DEC_WAVES * KPW) {
        u32x4 kk[DEC_UNROLL], vv[DEC_UNROLL];
#pragma unroll
        for (int u = 0; u < DEC_UNROLL; ++u) {
            const int j = base + u * RPL + sub;
            kk[u] = u32x4{0, 0, 0, 0};
            vv[u] = u32x4{0, 0, 0, 0};
            if (j < kend) {
                const bf16_t *kp, *vp;
                if (j < P.n_mem) { kp = kmem + (long)j * D; vp = vmem + (long)j * D; }
                else if (j < P.n_mem + P.n_read) { kp = kread + (long)(j - P.n_mem) * D; vp = vread + (long)(j - P.n_mem) * D; }
                else { kp = knew; vp = vnew; }
                kk[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kp + col * 8));
                vv[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vp + col * 8));
            }
        }
        if constexpr (ROPE) {   // the new token's key (the last key of the list, met by one lane group of one wave)
            if (P.has_new && base + (DEC_UNROLL - 1) * RPL + RPL > P.n_mem + P.n_read) {
#pragma unroll
                for (int u = 0; u < DEC_UNROLL; ++u) {
                    const int j = base + u * RPL + sub;
                    if (j < kend && j >= P.n_mem + P.n_read) kk[u] = rope::load_rotated_piece<D>(knew, col, RT.pos_first, RT);
                }
            }
        }
        float s[DEC_UNROLL];
        float mx = m;
#pragma unroll
        for (int u = 0; u < DEC_UNROLL; ++u) {
            const uint32_t k0 = kk[u][0], k1 = kk[u][1], k2 = kk[u][2], k3 = kk[u][3];
            float a = __builtin_amdgcn_fdot2_f32_bf16(q0, as_bf16x2(k0), 0.f, false);
            a = __builtin_amdgcn_fdot2_f32_bf16(q1, as_bf16x2(k1), a, false);
            a = __builtin_amdgcn_fdot2_f32_bf16(q2, as_bf16x2(k2), a, false);
            a = __builtin_amdgcn_fdot2_f32_bf16(q3, as_bf16x2(k3), a, false);
            a = row_sum<LPR>(a) * P.sc;
            s[u] = (base + u * RPL + sub < kend) ? a : -INFINITY;
            mx = fmaxf(mx, s[u]);
        }
        // mx stays -inf only while this lane group has seen no key at all
        const float alpha = (mx == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f(m - mx);
        float ps = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] *= alpha;
#pragma unroll
        for (int u = 0; u < DEC_UNROLL; ++u) {
            const float p = (s[u] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(s[u] - mx);
            ps += p;
            acc[0] = fmaf(p, bf16_lo(vv[u].x), acc[0]);
            acc[1] = fmaf(p, bf16_hi(vv[u].x), acc[1]);
            acc[2] = fmaf(p, bf16_lo(vv[u].y), acc[2]);
            acc[3] = fmaf(p, bf16_hi(vv[u].y), acc[3]);
            acc[4] = fmaf(p, bf16_lo(vv[u].z), acc[4]);
            acc[5] = fmaf(p, bf16_hi(vv[u].z), acc[5]);
            acc[6] = fmaf(p, bf16_lo(vv[u].w), acc[6]);
            acc[7] = fmaf(p, bf16_hi(vv[u].w), acc[7]);
        }
        l = l * alpha + ps;
        m = mx;
    }

    // merge the lane groups of the wave: partner groups sit 16 and 32 lanes away (and 8 for D = 64)
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) {
        const float m2 = __shfl_xor(m, off), l2 = __shfl_xor(l, off);
        const float M = fmaxf(m, m2);
        const float w1 = (m == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m - M);
        const float w2 = (m2 == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m2 - M);
        l = l * w1 + l2 * w2;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = acc[e] * w1 + __shfl_xor(acc[e], off) * w2;
        m = M;
    }
    // merge the waves of the workgroup
    if (sub == 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) sm_acc[w][col * 8 + e] = acc[e];
        if (col == 0) { sm_m[w] = m; sm_l[w] = l; }
    }
    __syncthreads();
    if (tid < D) {
        float M = -INFINITY;
#pragma unroll
        for (int gidx = 0; gidx < DEC_WAVES; ++gidx) M = fmaxf(M, sm_m[gidx]);
        float Lsum = 0.f, o = 0.f;
#pragma unroll
        for (int gidx = 0; gidx < DEC_WAVES; ++gidx) {
            const float wgt = (sm_m[gidx] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(sm_m[gidx] - M);
            Lsum = fmaf(sm_l[gidx], wgt, Lsum);
            o = fmaf(sm_acc[gidx][tid], wgt, o);
        }
        if (P.nsplit == 1) {
            P.out[bh * D + tid] = f32_to_bf16(o / Lsum);
        } else {
            const long pi = bh * P.nsplit + sp;
            P.ws_acc[pi * D + tid] = o;
            if (tid == 0) { P.ws_ml[pi * 2] = M; P.ws_ml[pi * 2 + 1] = Lsum; }
        }
    }
    // append the new token to the reading zone (Appendix A: the cache grows by the input token)
    if (P.has_new && sp == 0 && tid < 2 * LPR) {
        const int which = tid / LPR, piece = tid % LPR;
        uint4 x = *reinterpret_cast<const uint4*>((which ? vnew : knew) + piece * 8);
        if constexpr (ROPE) {
            if (which == 0) {
                const u32x4 r = rope::load_rotated_piece<D>(knew, piece, RT.pos_first, RT);
                x = uint4{r[0], r[1], r[2], r[3]};
            }
        }
        bf16_t* dst = (which ? P.v_read : P.k_read) + (bh * (long)P.R + P.n_read) * D;
        *reinterpret_cast<uint4*>(dst + piece * 8) = x;
    }
}

// Grouped-query form: G consecutive query heads share one KV head (models other than Llama-2-7B; with G = 1 this is
// the kernel above without its layered and rotary variants).  A workgroup belongs to a KV head and a key split and
// streams that head's K and V ONCE for all G queries: same loads, same lane layout, G online-softmax states per lane
// group, worked through one query after the other while a batch of rows sits in registers (16-wave workgroups hold
// half as many rows at a time: 128 registers per lane).  blockIdx.y = b * H_kv + hk;
// query head (b, hk * G + gq) has index bh * G + gq in q, out and the partial results.
template <int D, int G, int DEC_WAVES, int UNROLL, bool LAYERED>
__global__ __launch_bounds__(64 * DEC_WAVES) void decode_split_gqa_kernel(DecodeParams P) {
    constexpr int LPR = D / 8;
    constexpr int RPL = 64 / LPR;
    constexpr int KPW = RPL * UNROLL;
    __shared__ float sm_acc[DEC_WAVES][D];
    __shared__ float sm_m[DEC_WAVES], sm_l[DEC_WAVES];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int sp = blockIdx.x;
    const long bh = blockIdx.y;
    const int col = lane % LPR, sub = lane / LPR;
    const int kbeg = sp * P.keys_per_split;
    const int kend = min(P.L, kbeg + P.keys_per_split);
    if constexpr (LAYERED) {   // blockIdx.z is a layer: its tensors from the pointer tables, its own block of partial results
        const int layer = blockIdx.z;
        P.q = P.tab.q[layer];
        P.k_new = P.has_new ? P.tab.k_new[layer] : nullptr;
        P.v_new = P.has_new ? P.tab.v_new[layer] : nullptr;
        P.k_mem = P.n_mem > 0 ? P.tab.k_mem[layer] : nullptr;
        P.v_mem = P.n_mem > 0 ? P.tab.v_mem[layer] : nullptr;
        P.k_read = P.tab.k_read[layer];
        P.v_read = P.tab.v_read[layer];
        P.out = P.tab.out[layer];
        if (P.ws_acc != nullptr) { P.ws_acc += layer * P.ws_layer_floats; P.ws_ml += layer * P.ws_layer_floats; }
    }
    const bf16_t* kmem = P.k_mem + bh * P.mem_rows * D;
    const bf16_t* vmem = P.v_mem + bh * P.mem_rows * D;
    const bf16_t* kread = P.k_read + bh * (long)P.R * D;
    const bf16_t* vread = P.v_read + bh * (long)P.R * D;
    const bf16_t* knew = P.k_new + bh * D;
    const bf16_t* vnew = P.v_new + bh * D;

    bf16x2 qq[G][4];
    float m[G], l[G], acc[G][8];
#pragma unroll
    for (int gq = 0; gq < G; ++gq) {
        const uint4 qv = *reinterpret_cast<const uint4*>(P.q + (bh * G + gq) * D + col * 8);
        qq[gq][0] = as_bf16x2(qv.x); qq[gq][1] = as_bf16x2(qv.y); qq[gq][2] = as_bf16x2(qv.z); qq[gq][3] = as_bf16x2(qv.w);
        m[gq] = -INFINITY; l[gq] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[gq][e] = 0.f;
    }

    for (int base = kbeg + w * KPW; base < kend; base += DEC_WAVES * KPW) {
        u32x4 kk[UNROLL], vv[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int j = base + u * RPL + sub;
            kk[u] = u32x4{0, 0, 0, 0};
            vv[u] = u32x4{0, 0, 0, 0};
            if (j < kend) {
                const bf16_t *kp, *vp;
                if (j < P.n_mem) { kp = kmem + (long)j * D; vp = vmem + (long)j * D; }
                else if (j < P.n_mem + P.n_read) { kp = kread + (long)(j - P.n_mem) * D; vp = vread + (long)(j - P.n_mem) * D; }
                else { kp = knew; vp = vnew; }
                kk[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kp + col * 8));
                vv[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vp + col * 8));
            }
        }
#pragma unroll
        for (int gq = 0; gq < G; ++gq) {
            float s[UNROLL];
            float mx = m[gq];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const uint32_t k0 = kk[u][0], k1 = kk[u][1], k2 = kk[u][2], k3 = kk[u][3];
                float a = __builtin_amdgcn_fdot2_f32_bf16(qq[gq][0], as_bf16x2(k0), 0.f, false);
                a = __builtin_amdgcn_fdot2_f32_bf16(qq[gq][1], as_bf16x2(k1), a, false);
                a = __builtin_amdgcn_fdot2_f32_bf16(qq[gq][2], as_bf16x2(k2), a, false);
                a = __builtin_amdgcn_fdot2_f32_bf16(qq[gq][3], as_bf16x2(k3), a, false);
                a = row_sum<LPR>(a) * P.sc;
                s[u] = (base + u * RPL + sub < kend) ? a : -INFINITY;
                mx = fmaxf(mx, s[u]);
            }
            const float alpha = (mx == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f(m[gq] - mx);
            float ps = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[gq][e] *= alpha;
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const float p = (s[u] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(s[u] - mx);
                ps += p;
                acc[gq][0] = fmaf(p, bf16_lo(vv[u].x), acc[gq][0]);
                acc[gq][1] = fmaf(p, bf16_hi(vv[u].x), acc[gq][1]);
                acc[gq][2] = fmaf(p, bf16_lo(vv[u].y), acc[gq][2]);
                acc[gq][3] = fmaf(p, bf16_hi(vv[u].y), acc[gq][3]);
                acc[gq][4] = fmaf(p, bf16_lo(vv[u].z), acc[gq][4]);
                acc[gq][5] = fmaf(p, bf16_hi(vv[u].z), acc[gq][5]);
                acc[gq][6] = fmaf(p, bf16_lo(vv[u].w), acc[gq][6]);
                acc[gq][7] = fmaf(p, bf16_hi(vv[u].w), acc[gq][7]);
            }
            l[gq] = l[gq] * alpha + ps;
            m[gq] = mx;
        }
    }

#pragma unroll
    for (int gq = 0; gq < G; ++gq) {
        float mg = m[gq], lg = l[gq];
        // merge the lane groups of the wave, then the waves of the workgroup, as in the kernel above
#pragma unroll
        for (int off = LPR; off < 64; off <<= 1) {
            const float m2 = __shfl_xor(mg, off), l2 = __shfl_xor(lg, off);
            const float M = fmaxf(mg, m2);
            const float w1 = (mg == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mg - M);
            const float w2 = (m2 == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m2 - M);
            lg = lg * w1 + l2 * w2;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[gq][e] = acc[gq][e] * w1 + __shfl_xor(acc[gq][e], off) * w2;
            mg = M;
        }
        if (gq > 0) __syncthreads();   // the previous query's merge has read the buffers
        if (sub == 0) {
#pragma unroll
            for (int e = 0; e < 8; ++e) sm_acc[w][col * 8 + e] = acc[gq][e];
            if (col == 0) { sm_m[w] = mg; sm_l[w] = lg; }
        }
        __syncthreads();
        if (tid < D) {
            float M = -INFINITY;
#pragma unroll
            for (int gidx = 0; gidx < DEC_WAVES; ++gidx) M = fmaxf(M, sm_m[gidx]);
            float Lsum = 0.f, o = 0.f;
#pragma unroll
            for (int gidx = 0; gidx < DEC_WAVES; ++gidx) {
                const float wgt = (sm_m[gidx] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(sm_m[gidx] - M);
                Lsum = fmaf(sm_l[gidx], wgt, Lsum);
                o = fmaf(sm_acc[gidx][tid], wgt, o);
            }
            const long bhq = bh * G + gq;
            if (P.nsplit == 1) {
                P.out[bhq * D + tid] = f32_to_bf16(o / Lsum);
            } else {
                const long pi = bhq * P.nsplit + sp;
                P.ws_acc[pi * D + tid] = o;
                if (tid == 0) { P.ws_ml[pi * 2] = M; P.ws_ml[pi * 2 + 1] = Lsum; }
            }
        }
    }
    // append the new token to the KV head's reading zone
    if (P.has_new && sp == 0 && tid < 2 * LPR) {
        const int which = tid / LPR, piece = tid % LPR;
        const uint4 x = *reinterpret_cast<const uint4*>((which ? vnew : knew) + piece * 8);
        bf16_t* dst = (which ? P.v_read : P.k_read) + (bh * (long)P.R + P.n_read) * D;
        *reinterpret_cast<uint4*>(dst + piece * 8) = x;
    }
}

template <int D, bool LAYERED>
__global__ __launch_bounds__(D) void decode_combine_kernel(DecodeParams P) {
    const long bh = blockIdx.x;
    const int tid = threadIdx.x;
    if constexpr (LAYERED) {
        const int layer = blockIdx.y;
        P.out = P.tab.out[layer];
        P.ws_acc += layer * P.ws_layer_floats;
        P.ws_ml += layer * P.ws_layer_floats;
    }
    float M = -INFINITY;
    for (int sp = 0; sp < P.nsplit; ++sp) M = fmaxf(M, P.ws_ml[(bh * P.nsplit + sp) * 2]);
    float Lsum = 0.f, o = 0.f;
    for (int sp = 0; sp < P.nsplit; ++sp) {
        const long pi = bh * P.nsplit + sp;
        const float ms = P.ws_ml[pi * 2];
        const float wgt = (ms == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(ms - M);
        Lsum = fmaf(P.ws_ml[pi * 2 + 1], wgt, Lsum);
        o = fmaf(P.ws_acc[pi * D + tid], wgt, o);
    }
    P.out[bh * D + tid] = f32_to_bf16(o / Lsum);
}

inline int wg_waves(int nbh) { return nbh < DEC_SMALL_NBH ? 16 : 4; }
inline int target_splits(int nbh) {
    const int target = nbh < DEC_SMALL_NBH ? DEC_TARGET_WGS_16 : DEC_TARGET_WGS_4;
    return (target + nbh - 1) / nbh;
}

// keys per split: whole workgroup iterations, at most target_splits(nbh) splits
void plan_splits(int nbh, int D, int n_keys, int& nsplit, int& keys_per_split) {
    const int kpi = wg_waves(nbh) * (64 / (D / 8)) * DEC_UNROLL;  // keys per workgroup iteration
    const int units = (n_keys + kpi - 1) / kpi;
    const int tgt = target_splits(nbh);
    const int ups = (units + tgt - 1) / tgt;
    nsplit = (units + ups - 1) / ups;
    keys_per_split = ups * kpi;
}

template <int D, bool LAYERED, bool ROPE = false>
int launch_decode_d(DecodeParams& P, int nbh, int n_layers, void* workspace, hipStream_t st,
                    std::conditional_t<ROPE, RopeTable, NoRope> RT = {}) {
    plan_splits(nbh, D, P.L, P.nsplit, P.keys_per_split);
    P.ws_acc = static_cast<float*>(workspace);
    P.ws_ml = P.ws_acc ? P.ws_acc + (size_t)nbh * target_splits(nbh) * D : nullptr;
    P.ws_layer_floats = (long)nbh * target_splits(nbh) * (D + 2);
    if (nbh > 65535 || n_layers > 65535) return LOMA_ERR_UNSUPPORTED;
    if (wg_waves(nbh) == 16)
        hipLaunchKernelGGL((decode_split_kernel<D, 16, LAYERED, ROPE>), dim3(P.nsplit, nbh, n_layers), dim3(1024), 0, st, P, RT);
    else
        hipLaunchKernelGGL((decode_split_kernel<D, 4, LAYERED, ROPE>), dim3(P.nsplit, nbh, n_layers), dim3(256), 0, st, P, RT);
    if (hipGetLastError() != hipSuccess) return LOMA_ERR_LAUNCH;
    if (P.nsplit > 1) {
        hipLaunchKernelGGL((decode_combine_kernel<D, LAYERED>), dim3(nbh, n_layers), dim3(D), 0, st, P);
        if (hipGetLastError() != hipSuccess) return LOMA_ERR_LAUNCH;
    }
    return LOMA_OK;
}

// Split-K partial results of the entry point that allocates nothing: a fixed array in the library's own
// device image, one copy per GPU, alive until the process ends.  The host never uses this name as an address:
// the per-device address comes from hipGetSymbolAddress (static_scratch_ptr).
constexpr size_t DEC_STATIC_SCRATCH_BYTES = size_t(4) << 20;
static __device__ __align__(256) unsigned char scratch[DEC_STATIC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex scratch_mu;
void* scratch_ptr_of_device[MAX_DEVICES] = {};

}  // namespace

int decode_num_splits(int nbh, int n_keys) {
    int ns, kps;
    plan_splits(nbh, 128, n_keys, ns, kps);
    return ns;
}

size_t decode_workspace_bytes(int nbh, int D, int /*n_keys_max*/) {
    const int tgt = target_splits(nbh);
    if (tgt <= 1) return 0;
    return (size_t)nbh * tgt * (D + 2) * sizeof(float);
}

size_t decode_static_scratch_bytes() { return DEC_STATIC_SCRATCH_BYTES; }

void* decode_static_scratch_ptr() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
    std::lock_guard<std::mutex> lock(scratch_mu);
    if (scratch_ptr_of_device[dev] == nullptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
        scratch_ptr_of_device[dev] = p;
    }
    return scratch_ptr_of_device[dev];
}

int launch_decode_splitk(const void* q, const void* k_new, const void* v_new,
                         const void* k_memcache, const void* v_memcache, void* k_read, void* v_read,
                         void* out, int nbh, int D, int R, int n_mem_keys, int mem_capacity, int read_fill,
                         float scale, void* workspace, hipStream_t st, const RopeTable* rope) {
    DecodeParams P = {};
    P.q = static_cast<const bf16_t*>(q);
    P.k_new = static_cast<const bf16_t*>(k_new); P.v_new = static_cast<const bf16_t*>(v_new);
    P.k_mem = static_cast<const bf16_t*>(k_memcache); P.v_mem = static_cast<const bf16_t*>(v_memcache);
    P.k_read = static_cast<bf16_t*>(k_read); P.v_read = static_cast<bf16_t*>(v_read);
    P.out = static_cast<bf16_t*>(out);
    P.mem_rows = mem_capacity; P.R = R; P.n_mem = n_mem_keys; P.n_read = read_fill;
    P.has_new = k_new != nullptr;
    P.L = n_mem_keys + read_fill + (P.has_new ? 1 : 0);
    P.sc = scale * LOG2E;
    if (rope != nullptr)
        return D == 128 ? launch_decode_d<128, false, true>(P, nbh, 1, workspace, st, *rope)
                        : launch_decode_d<64, false, true>(P, nbh, 1, workspace, st, *rope);
    return D == 128 ? launch_decode_d<128, false>(P, nbh, 1, workspace, st)
                    : launch_decode_d<64, false>(P, nbh, 1, workspace, st);
}

// grouped-query form: split plan from the KV heads as in the plain form (few heads: 16-wave workgroups, about one per
// CU; many: 4-wave workgroups), partial results per query head
namespace {
// eight queries per KV head do not fit the 128 registers a lane of a 16-wave workgroup has: 4-wave workgroups then
inline bool gqa_wide(int nbh_kv, int G) { return wg_waves(nbh_kv) == 16 && G <= 4; }
inline int gqa_target_splits(int nbh_kv, int G) {
    return gqa_wide(nbh_kv, G) ? target_splits(nbh_kv) : (DEC_TARGET_WGS_4 + nbh_kv - 1) / nbh_kv;
}
template <int D, int G, bool LAYERED>
int launch_decode_gqa_dg(DecodeParams& P, int nbh_kv, int n_layers, void* workspace, hipStream_t st) {
    const bool wide = gqa_wide(nbh_kv, G);
    const int kpi = (wide ? 16 * 4 : 4 * DEC_UNROLL) * (64 / (D / 8));   // keys per workgroup iteration
    const int units = (P.L + kpi - 1) / kpi;
    const int tgt = gqa_target_splits(nbh_kv, G);
    const int ups = (units + tgt - 1) / tgt;
    P.nsplit = (units + ups - 1) / ups;
    P.keys_per_split = ups * kpi;
    const long nbh_q = (long)nbh_kv * G;
    P.ws_acc = static_cast<float*>(workspace);
    P.ws_ml = P.ws_acc ? P.ws_acc + (size_t)nbh_q * tgt * D : nullptr;
    P.ws_layer_floats = nbh_q * tgt * (D + 2);
    if (n_layers > 65535) return LOMA_ERR_UNSUPPORTED;
    if constexpr (G <= 4) {
        if (wide) hipLaunchKernelGGL((decode_split_gqa_kernel<D, G, 16, 4, LAYERED>), dim3(P.nsplit, nbh_kv, n_layers), dim3(1024), 0, st, P);
    }
    if (!wide) hipLaunchKernelGGL((decode_split_gqa_kernel<D, G, 4, DEC_UNROLL, LAYERED>), dim3(P.nsplit, nbh_kv, n_layers), dim3(256), 0, st, P);
    if (hipGetLastError() != hipSuccess) return LOMA_ERR_LAUNCH;
    if (P.nsplit > 1) {
        hipLaunchKernelGGL((decode_combine_kernel<D, LAYERED>), dim3((unsigned)nbh_q, n_layers), dim3(D), 0, st, P);
        if (hipGetLastError() != hipSuccess) return LOMA_ERR_LAUNCH;
    }
    return LOMA_OK;
}
template <int D, bool LAYERED>
int launch_decode_gqa_d(DecodeParams& P, int nbh_kv, int G, int n_layers, void* workspace, hipStream_t st) {
    switch (G) {
        case 1: return launch_decode_gqa_dg<D, 1, LAYERED>(P, nbh_kv, n_layers, workspace, st);
        case 2: return launch_decode_gqa_dg<D, 2, LAYERED>(P, nbh_kv, n_layers, workspace, st);
        case 4: return launch_decode_gqa_dg<D, 4, LAYERED>(P, nbh_kv, n_layers, workspace, st);
        case 8: return launch_decode_gqa_dg<D, 8, LAYERED>(P, nbh_kv, n_layers, workspace, st);
        default: return LOMA_ERR_UNSUPPORTED;
    }
}
}  // namespace

size_t decode_gqa_workspace_bytes(int nbh_kv, int G, int D) {
    const int tgt = gqa_target_splits(nbh_kv, G);
    if (tgt <= 1) return 0;
    return (size_t)nbh_kv * G * tgt * (D + 2) * sizeof(float);
}

int launch_decode_gqa(const void* q, const void* k_new, const void* v_new,
                      const void* k_memcache, const void* v_memcache, void* k_read, void* v_read,
                      void* out, int nbh_kv, int G, int D, int R, int n_mem_keys, int mem_capacity, int read_fill,
                      float scale, void* workspace, hipStream_t st) {
    DecodeParams P = {};
    P.q = static_cast<const bf16_t*>(q);
    P.k_new = static_cast<const bf16_t*>(k_new); P.v_new = static_cast<const bf16_t*>(v_new);
    P.k_mem = static_cast<const bf16_t*>(k_memcache); P.v_mem = static_cast<const bf16_t*>(v_memcache);
    P.k_read = static_cast<bf16_t*>(k_read); P.v_read = static_cast<bf16_t*>(v_read);
    P.out = static_cast<bf16_t*>(out);
    P.mem_rows = mem_capacity; P.R = R; P.n_mem = n_mem_keys; P.n_read = read_fill;
    P.has_new = k_new != nullptr;
    P.L = n_mem_keys + read_fill + (P.has_new ? 1 : 0);
    P.sc = scale * LOG2E;
    if (nbh_kv > 65535 || (long long)nbh_kv * G > 0x7fffffffLL) return LOMA_ERR_UNSUPPORTED;
    return D == 128 ? launch_decode_gqa_d<128, false>(P, nbh_kv, G, 1, workspace, st)
                    : launch_decode_gqa_d<64, false>(P, nbh_kv, G, 1, workspace, st);
}

int launch_decode_gqa_layers(const void* const* tables[8], bool has_new, int n_layers, int nbh_kv, int G, int D, int R,
                             int n_mem_keys, int mem_capacity, int read_fill, float scale, void* workspace, hipStream_t st) {
    DecodeParams P = {};
    P.tab.q = reinterpret_cast<const bf16_t* const*>(tables[0]);
    P.tab.k_new = reinterpret_cast<const bf16_t* const*>(tables[1]);
    P.tab.v_new = reinterpret_cast<const bf16_t* const*>(tables[2]);
    P.tab.k_mem = reinterpret_cast<const bf16_t* const*>(tables[3]);
    P.tab.v_mem = reinterpret_cast<const bf16_t* const*>(tables[4]);
    P.tab.k_read = (bf16_t* const*)(tables[5]);
    P.tab.v_read = (bf16_t* const*)(tables[6]);
    P.tab.out = (bf16_t* const*)(tables[7]);
    P.mem_rows = mem_capacity; P.R = R; P.n_mem = n_mem_keys; P.n_read = read_fill;
    P.has_new = has_new;
    P.L = n_mem_keys + read_fill + (has_new ? 1 : 0);
    P.sc = scale * LOG2E;
    if (nbh_kv > 65535 || (long long)nbh_kv * G > 0x7fffffffLL) return LOMA_ERR_UNSUPPORTED;
    return D == 128 ? launch_decode_gqa_d<128, true>(P, nbh_kv, G, n_layers, workspace, st)
                    : launch_decode_gqa_d<64, true>(P, nbh_kv, G, n_layers, workspace, st);
}

int launch_decode_splitk_layers(const void* const* tables[8], bool has_new, int n_layers, int nbh, int D, int R,
                                int n_mem_keys, int mem_capacity, int read_fill, float scale, void* workspace,
                                hipStream_t st) {
    DecodeParams P = {};
    P.tab.q = reinterpret_cast<const bf16_t* const*>(tables[0]);
    P.tab.k_new = reinterpret_cast<const bf16_t* const*>(tables[1]);
    P.tab.v_new = reinterpret_cast<const bf16_t* const*>(tables[2]);
    P.tab.k_mem = reinterpret_cast<const bf16_t* const*>(tables[3]);
    P.tab.v_mem = reinterpret_cast<const bf16_t* const*>(tables[4]);
    P.tab.k_read = (bf16_t* const*)(tables[5]);
    P.tab.v_read = (bf16_t* const*)(tables[6]);
    P.tab.out = (bf16_t* const*)(tables[7]);
    P.mem_rows = mem_capacity; P.R = R; P.n_mem = n_mem_keys; P.n_read = read_fill;
    P.has_new = has_new;
    P.L = n_mem_keys + read_fill + (has_new ? 1 : 0);
    P.sc = scale * LOG2E;
    return D == 128 ? launch_decode_d<128, true>(P, nbh, n_layers, workspace, st)
                    : launch_decode_d<64, true>(P, nbh, n_layers, workspace, st);
}

}  // namespace loma
