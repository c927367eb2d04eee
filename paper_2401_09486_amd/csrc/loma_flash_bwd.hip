// MFMA kernels for the gradients of the mask pass (Sec. 4.3 Eq. 1-3 with Sec. 4.4 Eq. 5-7,
// differentiated) on gfx950, bf16 data with head_dim 64 or 128.
//
// With W_ij = exp(scale q_i.k_j - lse_i) on visible pairs, G the gradient of the output and
// delta_i = G_i . O_i:   dV = W^T G,   dA = W o (G V^T - delta),   dQ = scale dA K,   dK = scale dA^T Q.
// Two passes share one tile engine.  A workgroup OWNS 32 rows per wave (operands in registers)
// and STREAMS the rows that interact with them through LDS, 32 at a time:
//     dQ pass:     owner = a block of query rows (q, G in registers), stream = the keys those rows
//                  see (K, V tiles) -- the same block list as the forward pass;
//     dK/dV pass:  owner = a block of keys (k, v in registers), stream = the queries that see them
//                  (Q, G tiles with their lse and delta) -- the mask read by columns:
//                    reading-zone keys o.. of chunk y: reading rows >= o and the memory rows of y;
//                    memory-zone keys: the memory and repetition rows of their chunk and the
//                    reading rows of every later chunk.  One block owns 32*NW consecutive memory
//                    keys of the sequence, across chunks, so that a streamed query row is used by
//                    as many keys as a reading-zone block offers.
// Per tile, with lane = owner row and the streamed rows down the accumulator registers:
//     S' = X xo^T and dP' = Y yo^T   (X, Y the streamed tiles; plain LDS reads as A operand)
//     P = exp2(S' sc - lse), dS = P (dP' - delta), rounded to bf16 in the B-operand layout
//     acc^T += X^T dS  (and, for keys, accV^T += Y^T P)   (transposing LDS reads as A operand)
// so every MFMA takes one operand from LDS and one from registers.  A tile's rows are stored
// with their 16-byte pieces XOR-permuted such that both the plain and the transposing read are
// free of bank conflicts.  Repetition rows see their own key only through the diagonal: that
// term (for dQ, and the whole of dK/dV of repetition-zone keys) is added on the vector ALU when
// the dQ rows of a repetition block leave.  Every output row has one owner: no atomics.
#include "loma_mfma.h"

namespace loma {
namespace {

using namespace mfma;

enum : int { PASS_DQ = 0, PASS_DKV = 1 };
enum : int { VIS_CAUSAL = 0, VIS_FROM_ROW = 1, VIS_MEMKEYS = 2 };

// Rows of one (b,h) sequence: two ranges walked back to back, each cut into slabs of `slab` rows
// whose starts lie `stride` rows apart.  magic = floor(2^32 / slab) + 1 gives j / slab as
// umulhi(j, magic) while j * slab < 2^32 (checked on the host); slab 1 needs no division.
struct RowList {
    int base0, n0, slab0, stride0;
    unsigned magic0;
    int base1, n1, slab1, stride1;
    unsigned magic1;
};

__host__ __device__ inline unsigned magic_of(int slab) { return slab <= 1 ? 0u : (unsigned)(0x100000000ULL / (unsigned)slab) + 1u; }

__device__ __forceinline__ int div_slab(int j, int slab, unsigned magic) {
    return slab == 1 ? j : (int)__umulhi((unsigned)j, magic);
}
// slab index of list entry j inside its range, and the row it names
__device__ __forceinline__ int list_row(const RowList L, int j, int* slab_index = nullptr) {
    const bool in0 = j < L.n0;
    const int jj = in0 ? j : j - L.n0;
    const int slab = in0 ? L.slab0 : L.slab1;
    const int a = div_slab(jj, slab, in0 ? L.magic0 : L.magic1);
    if (slab_index) *slab_index = a;
    return (in0 ? L.base0 : L.base1) + a * (in0 ? L.stride0 : L.stride1) + (jj - a * slab);
}

struct BwdJob {
    RowList own;   // owner rows: entry `ooff + r` for block row r (range 0 only)
    int ooff, orows;
    RowList str;   // streamed rows, nstr of them
    int nstr;
    int vis;       // which rule decides whether streamed row j and owner row r interact
    int cb;        // VIS_CAUSAL: j <= cb + r.   VIS_FROM_ROW: j >= r.
    // VIS_MEMKEYS: owner r is memory key ooff + r of chunk yk = (ooff + r) / t; streamed row j of range 0
    // is a reading row of chunk y_first + 1 + slab index (visible iff yk < that chunk), of range 1 a memory
    // or repetition row of chunk y_first + slab index (visible iff yk == that chunk)
    int t, y_first;
    unsigned magic_t;
    int rep;       // dQ pass on repetition rows: add the rows' own-key terms when they leave
};

struct BwdTensors {   // all at the first row of the (b,h) sequence
    const bf16_t *q, *k, *v, *dout;
    const float *lse, *delta;
    bf16_t *dq, *dk, *dv;
};

template <int D>
struct BCfg {
    static constexpr int BN = 32;            // streamed rows per tile
    static constexpr int CPR = D / 8;        // 16-byte pieces per row
    static constexpr int RPI = 64 / CPR;     // tile rows one wave-wide direct load covers
    static constexpr int KSTEPS = D / 16;
    static constexpr int DT = D / 32;
    static constexpr int TILE = BN * D;      // elements of one tensor's tile
    static constexpr int STAGE_BYTES = 2 * TILE * 2 + 64 * 4;   // X, Y, then 32 lse and 32 delta values
    static constexpr int NS = 2;
    static constexpr int FSTR = D + 4;       // row stride (floats) of the fp32 staging area rows leave through
    static constexpr int WAVE_STAGING_BYTES = 32 * FSTR * 4;
    static constexpr int smem_bytes(int nw) {
        return NS * STAGE_BYTES > nw * WAVE_STAGING_BYTES ? NS * STAGE_BYTES : nw * WAVE_STAGING_BYTES;
    }
};

// position of 16-byte piece c of tile row r: c ^ swz(r).  16 consecutive rows give 16 different values
// (plain reads: one piece of 16 rows), and the four rows r..r+3 of a transposing read differ in the two
// high bits while rows 4 apart differ in the two low bits.
template <int CPR>
__device__ __forceinline__ int swz(int r) { return (4 * (r & 3) + ((r >> 2) & 3)) % CPR; }

__device__ __forceinline__ void direct_load_4B(const float* src, float* lds_dst) {
    const unsigned dst = __builtin_amdgcn_readfirstlane(
        (unsigned)(size_t)(__attribute__((address_space(3))) float*)lds_dst);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off" ::"s"(dst), "v"(src) : "memory", "m0");
}

// Direct HBM -> LDS copy of streamed tile [j0, j0 + 32): X and Y rows (entries past the list replay its
// last row; the arithmetic masks them) and, for the dK/dV pass, the rows' lse and delta.
template <int D, int NW, int PASS>
__device__ __forceinline__ void request_tile(const BwdJob& J, const bf16_t* X, const bf16_t* Y, const float* lse,
                                             const float* delta, int j0, int w, int lane, bf16_t* stage) {
    using C = BCfg<D>;
    constexpr int IPW = C::BN / C::RPI / NW;
    static_assert(IPW >= 1, "tile rows split over the waves");
    const int p = lane % C::CPR;
    bf16_t* Xs = stage;
    bf16_t* Ys = stage + C::TILE;
#pragma unroll
    for (int i = 0; i < IPW; ++i) {
        const int rbase = (w * IPW + i) * C::RPI;   // wave-uniform
        const int r = rbase + lane / C::CPR;
        const long row = list_row(J.str, min(j0 + r, J.nstr - 1));
        const int c = p ^ swz<C::CPR>(r);
        direct_load_16B(X + row * D + c * 8, Xs + rbase * D);
        direct_load_16B(Y + row * D + c * 8, Ys + rbase * D);
    }
    if constexpr (PASS == PASS_DKV) {
        // every wave writes the same 64 values (keeps the waves' load counts equal)
        const long row = list_row(J.str, min(j0 + (lane & 31), J.nstr - 1));
        direct_load_4B((lane < 32 ? lse : delta) + row, reinterpret_cast<float*>(stage + 2 * C::TILE));
    }
}

// fp32 accumulators (lane = owner row, registers = head-dim) times `mul` into the wave's staging area
template <int D>
__device__ __forceinline__ void stage_acc(const f32x16 (&acc)[BCfg<D>::DT], float mul, float* Of, int lane) {
    using C = BCfg<D>;
    const int g = lane >> 5, l32 = lane & 31;
#pragma unroll
    for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
            float4 x;
            x.x = acc[dt][4 * i4 + 0] * mul; x.y = acc[dt][4 * i4 + 1] * mul;
            x.z = acc[dt][4 * i4 + 2] * mul; x.w = acc[dt][4 * i4 + 3] * mul;
            *reinterpret_cast<float4*>(Of + l32 * C::FSTR + 32 * dt + 8 * i4 + 4 * g) = x;
        }
}

// staged rows -> bf16 rows of `dst` (row layout: lane = 16-byte piece of a row, whole 1 KB runs per store)
template <int D>
__device__ __forceinline__ void store_staged(const float* Of, bf16_t* dst, const BwdJob& J, int row0, int lane) {
    using C = BCfg<D>;
    const int rl = lane / C::CPR, pc = lane % C::CPR;
#pragma unroll
    for (int i = 0; i < 32 / C::RPI; ++i) {
        const int r = i * C::RPI + rl;
        const float4 a = *reinterpret_cast<const float4*>(Of + r * C::FSTR + pc * 8);
        const float4 b = *reinterpret_cast<const float4*>(Of + r * C::FSTR + pc * 8 + 4);
        uint4 o;
        o.x = pack_bf16(a.x, a.y); o.y = pack_bf16(a.z, a.w); o.z = pack_bf16(b.x, b.y); o.w = pack_bf16(b.z, b.w);
        if (row0 + r < J.orows) {
            const long row = list_row(J.own, J.ooff + row0 + r);
            *reinterpret_cast<uint4*>(dst + row * D + pc * 8) = o;
        }
    }
}

__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c) {   // a, b: bf16 pairs
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), c, false);
}
__device__ __forceinline__ float dot8(u32x4 a, u32x4 b) {
    // (elements are copied out first: a bit cast applied to a vector element reads element 0)
    const uint32_t a0 = a.x, a1 = a.y, a2 = a.z, a3 = a.w, b0 = b.x, b1 = b.y, b2 = b.z, b3 = b.w;
    return dot2(a3, b3, dot2(a2, b2, dot2(a1, b1, dot2(a0, b0, 0.f))));
}
// x * a + b on the eight bf16 values of b, result packed to bf16 (b may be all zero)
__device__ __forceinline__ uint4 axpb8(float x, u32x4 a, float4 b0, float4 b1) {
    uint4 o;
    o.x = pack_bf16(fmaf(x, bf16_lo(a.x), b0.x), fmaf(x, bf16_hi(a.x), b0.y));
    o.y = pack_bf16(fmaf(x, bf16_lo(a.y), b0.z), fmaf(x, bf16_hi(a.y), b0.w));
    o.z = pack_bf16(fmaf(x, bf16_lo(a.z), b1.x), fmaf(x, bf16_hi(a.z), b1.y));
    o.w = pack_bf16(fmaf(x, bf16_lo(a.w), b1.z), fmaf(x, bf16_hi(a.w), b1.w));
    return o;
}

// Repetition rows leave: row p also sees its own key (identity block of Eq. 1), and is the only row that
// sees it.  With w = exp(scale q_p.k_p - lse_p) and da = w (G_p.v_p - delta_p):
//     dq_p = staged + scale da k_p,   dk_p = scale da q_p,   dv_p = w G_p.
template <int D>
__device__ __forceinline__ void store_staged_rep(const float* Of, const BwdTensors& T, const BwdJob& J, int row0,
                                                 float scale, float sc, int lane) {
    using C = BCfg<D>;
    const int rl = lane / C::CPR, pc = lane % C::CPR;
#pragma unroll
    for (int i = 0; i < 32 / C::RPI; ++i) {
        const int r = i * C::RPI + rl;
        const bool live = row0 + r < J.orows;
        const long row = list_row(J.own, J.ooff + min(row0 + r, J.orows - 1));   // rows past the block replay its last row
        const long at = row * D + pc * 8;
        const u32x4 qq = *reinterpret_cast<const u32x4*>(T.q + at);
        const u32x4 kk = *reinterpret_cast<const u32x4*>(T.k + at);
        const u32x4 vv = *reinterpret_cast<const u32x4*>(T.v + at);
        const u32x4 gg = *reinterpret_cast<const u32x4*>(T.dout + at);
        const float s = row_sum<C::CPR>(dot8(qq, kk));
        const float dw = row_sum<C::CPR>(dot8(gg, vv));
        const float wgt = __builtin_amdgcn_exp2f(s * sc - T.lse[row] * LOG2E);
        const float da = wgt * (dw - T.delta[row]);
        const float4 a = *reinterpret_cast<const float4*>(Of + r * C::FSTR + pc * 8);
        const float4 b = *reinterpret_cast<const float4*>(Of + r * C::FSTR + pc * 8 + 4);
        const float4 z = {0.f, 0.f, 0.f, 0.f};
        if (live) {
            *reinterpret_cast<uint4*>(T.dq + at) = axpb8(scale * da, kk, a, b);
            *reinterpret_cast<uint4*>(T.dk + at) = axpb8(scale * da, qq, z, z);
            *reinterpret_cast<uint4*>(T.dv + at) = axpb8(wgt, gg, z, z);
        }
    }
}

template <int D, int NW, int PASS>
__device__ __forceinline__ void bwd_job(const BwdJob& J, const BwdTensors& T, float scale, float sc, bf16_t* smem) {
    using C = BCfg<D>;
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 5, l32 = lane & 31;
    // owner operands come from (xo, yo), streamed tiles from (X, Y)
    const bf16_t* Xo = PASS == PASS_DQ ? T.q : T.k;
    const bf16_t* Yo = PASS == PASS_DQ ? T.dout : T.v;
    const bf16_t* X = PASS == PASS_DQ ? T.k : T.q;
    const bf16_t* Y = PASS == PASS_DQ ? T.v : T.dout;

    const int row0 = 32 * w;
    const bool has_rows = row0 < J.orows;
    const int r_hi = min(row0 + 31, J.orows - 1);            // last live row of this wave
    const int r_own = min(row0 + l32, J.orows - 1);          // lanes past the block replay its last row (never stored)
    const long orow = list_row(J.own, J.ooff + r_own);
    const int ntiles = (J.nstr + C::BN - 1) / C::BN;

    if (ntiles > 0) request_tile<D, NW, PASS>(J, X, Y, T.lse, T.delta, 0, w, lane, smem);

    // owner rows as B operands: lane (row l32, half g) holds head-dim 16*ks + 8*g .. +7
    bf16x8 xo[C::KSTEPS], yo[C::KSTEPS];
#pragma unroll
    for (int ks = 0; ks < C::KSTEPS; ++ks) {
        xo[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(Xo + orow * D + 16 * ks + 8 * g));
        yo[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(Yo + orow * D + 16 * ks + 8 * g));
    }
    float nl_own = 0.f, dl_own = 0.f;
    if constexpr (PASS == PASS_DQ) {
        nl_own = -T.lse[orow] * LOG2E;
        dl_own = T.delta[orow];
    }
    // who sees whom: per-lane and per-wave quantities of the job's rule
    const int yk = J.vis == VIS_MEMKEYS ? div_slab(J.ooff + r_own, J.t, J.magic_t) : 0;
    const int yk_lo = J.vis == VIS_MEMKEYS ? div_slab(J.ooff + min(row0, J.orows - 1), J.t, J.magic_t) : 0;
    const int yk_hi = J.vis == VIS_MEMKEYS ? div_slab(J.ooff + r_hi, J.t, J.magic_t) : 0;

    // per-lane LDS offsets (elements) of the operand reads under the tiles' piece permutation
    int poff[C::KSTEPS], toff[2][C::DT];
#pragma unroll
    for (int ks = 0; ks < C::KSTEPS; ++ks) poff[ks] = l32 * D + (((2 * ks + g) ^ swz<C::CPR>(l32)) * 8);
    {
        const int i = lane & 15, q = i >> 2, h = (lane >> 4) & 1;
#pragma unroll
        for (int a = 0; a < 2; ++a) {
            const int r = 8 * a + 4 * g + q;
#pragma unroll
            for (int dt = 0; dt < C::DT; ++dt)
                toff[a][dt] = r * D + (((4 * dt + 2 * h + ((i & 3) >> 1)) ^ swz<C::CPR>(r)) * 8) + 4 * (i & 1);
        }
    }

    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    f32x16 accX[C::DT];                         // dQ^T (dQ pass) or dK^T (dK/dV pass)
    f32x16 accY[PASS == PASS_DKV ? C::DT : 1];  // dV^T
#pragma unroll
    for (int dt = 0; dt < C::DT; ++dt) accX[dt] = zero16;
#pragma unroll
    for (int dt = 0; dt < (PASS == PASS_DKV ? C::DT : 1); ++dt) accY[dt] = zero16;

    wait_direct_loads();
    __syncthreads();

    for (int kt = 0; kt < ntiles; ++kt) {
        bf16_t* stage = smem + (kt & 1) * (C::STAGE_BYTES / 2);
        if (kt + 1 < ntiles)
            request_tile<D, NW, PASS>(J, X, Y, T.lse, T.delta, (kt + 1) * C::BN, w, lane,
                                      smem + ((kt + 1) & 1) * (C::STAGE_BYTES / 2));
        const int j0 = kt * C::BN, j1 = min(j0 + C::BN, J.nstr) - 1;   // first and last live streamed row
        // does this wave's 32 x 32 block hold no visible pair, only visible pairs, or both?
        bool none = !has_rows, cut = j0 + C::BN > J.nstr;
        int z0 = 0, z1 = 0;   // VIS_MEMKEYS: chunk of the tile's first and last row
        bool r0_first = false, r0_last = false;
        if (J.vis == VIS_CAUSAL) {
            none = none || j0 > J.cb + r_hi;
            cut = cut || j0 + C::BN - 1 > J.cb + row0;
        } else if (J.vis == VIS_FROM_ROW) {
            none = none || j1 < row0;
            cut = cut || j0 < r_hi;
        } else {
            int a0, a1;
            list_row(J.str, j0, &a0);
            list_row(J.str, j1, &a1);
            r0_first = j0 < J.str.n0; r0_last = j1 < J.str.n0;
            z0 = J.y_first + a0 + (r0_first ? 1 : 0);
            z1 = J.y_first + a1 + (r0_last ? 1 : 0);
            if (r0_first != r0_last || z0 != z1) cut = true;
            else if (r0_first) { none = none || yk_lo >= z0; cut = cut || yk_hi >= z0; }
            else { none = none || z0 < yk_lo || z0 > yk_hi; cut = cut || yk_lo != z0 || yk_hi != z0; }
        }
        if (!none) {
            const bf16_t* Xs = stage;
            const bf16_t* Ys = stage + C::TILE;
            // ---- S' = X xo^T, dP' = Y yo^T: accumulator i of lane (l32, g) is streamed row 8*(i/4) + 4*g + i%4 ----
            f32x16 S = zero16, dP = zero16;
#pragma unroll
            for (int ks = 0; ks < C::KSTEPS; ++ks) {
                const bf16x8 ax = *reinterpret_cast<const bf16x8*>(Xs + poff[ks]);
                const bf16x8 ay = *reinterpret_cast<const bf16x8*>(Ys + poff[ks]);
                S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ax, xo[ks], S, 0, 0, 0);
                dP = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ay, yo[ks], dP, 0, 0, 0);
            }
            // ---- P = exp2(S' sc - lse log2 e), dS = P (dP' - delta) ----------------------------------------------
            if constexpr (PASS == PASS_DQ) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float p = __builtin_amdgcn_exp2f(fmaf(S[i], sc, nl_own));
                    S[i] = p;
                    dP[i] = p * (dP[i] - dl_own);
                }
            } else {
                const float4* ld = reinterpret_cast<const float4*>(stage + 2 * C::TILE);
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    const float4 ls = ld[2 * a + g], dl = ld[8 + 2 * a + g];
                    const float lsv[4] = {ls.x, ls.y, ls.z, ls.w}, dlv[4] = {dl.x, dl.y, dl.z, dl.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float p = __builtin_amdgcn_exp2f(fmaf(S[4 * a + e], sc, -lsv[e] * LOG2E));
                        S[4 * a + e] = p;
                        dP[4 * a + e] = p * (dP[4 * a + e] - dlv[e]);
                    }
                }
            }
            if (cut) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int j = j0 + 8 * (i >> 2) + 4 * g + (i & 3);
                    bool vis = j < J.nstr;
                    if (J.vis == VIS_CAUSAL) vis = vis && j <= J.cb + r_own;
                    else if (J.vis == VIS_FROM_ROW) vis = vis && j >= r_own;
                    else {
                        int a;
                        list_row(J.str, min(j, J.nstr - 1), &a);
                        vis = vis && (j < J.str.n0 ? yk < J.y_first + 1 + a : yk == J.y_first + a);
                    }
                    S[i] = vis ? S[i] : 0.f;
                    dP[i] = vis ? dP[i] : 0.f;
                }
            }
            // ---- acc^T += X^T dS (and accY^T += Y^T P): 16 streamed rows per step ---------------------------------
            auto pack8 = [&](const f32x16& A, int step) -> bf16x8 {
                uint4 pw;
                pw.x = pack_bf16(A[8 * step + 0], A[8 * step + 1]);
                pw.y = pack_bf16(A[8 * step + 2], A[8 * step + 3]);
                pw.z = pack_bf16(A[8 * step + 4], A[8 * step + 5]);
                pw.w = pack_bf16(A[8 * step + 6], A[8 * step + 7]);
                return __builtin_bit_cast(bf16x8, pw);
            };
            auto read_t = [&](const bf16_t* base, int step, int dt) -> bf16x8 {
                const s16x4 lo = lds_read_tr(base + toff[0][dt] + 16 * step * D);
                const s16x4 hi = lds_read_tr(base + toff[1][dt] + 16 * step * D);
                return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
            };
#pragma unroll
            for (int step = 0; step < 2; ++step) {
                const bf16x8 bds = pack8(dP, step);
                const bf16x8 bp = pack8(S, step);
#pragma unroll
                for (int dt = 0; dt < C::DT; ++dt) {
                    accX[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_t(Xs, step, dt), bds, accX[dt], 0, 0, 0);
                    if constexpr (PASS == PASS_DKV)
                        accY[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_t(Ys, step, dt), bp, accY[dt], 0, 0, 0);
                }
            }
        }
        wait_direct_loads();
        __syncthreads();
    }

    // rows leave through the wave's own fp32 staging area (the tile stages are free: the loop ended on a barrier)
    float* Of = reinterpret_cast<float*>(smem) + w * (C::WAVE_STAGING_BYTES / 4);
    if (has_rows) {
        stage_acc<D>(accX, scale, Of, lane);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        if constexpr (PASS == PASS_DQ) {
            if (J.rep) store_staged_rep<D>(Of, T, J, row0, scale, sc, lane);
            else store_staged<D>(Of, T.dq, J, row0, lane);
        } else {
            store_staged<D>(Of, T.dk, J, row0, lane);
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            stage_acc<D>(accY, 1.f, Of, lane);
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            store_staged<D>(Of, T.dv, J, row0, lane);
        }
    }
}

struct BwdParams {
    BwdTensors T;       // at sequence 0
    int nbh, n, t, R, s;
    int bm;             // owner rows per workgroup
    float scale, sc;    // scale, scale * log2(e)
};

__device__ __forceinline__ void split_block(long long id, int nbh, int jobs_per_bh, int& bh, int& u) {
    // (b,h) pairs are dealt to the 8 XCDs (workgroup id % 8) so that one pair's rows stay in one L2
    if (nbh % 8 == 0) {
        const int xcd = (int)(id % 8);
        const long long k = id / 8;
        bh = xcd + 8 * (int)(k / jobs_per_bh);
        u = (int)(k % jobs_per_bh);
    } else {
        bh = (int)(id % nbh);
        u = (int)(id / nbh);
    }
}

__device__ __forceinline__ RowList one_range(int base, int n) {
    RowList L;
    L.base0 = 0; L.n0 = 0; L.slab0 = 1; L.stride0 = 1; L.magic0 = 0;
    L.base1 = base; L.n1 = n; L.slab1 = 1; L.stride1 = 1; L.magic1 = 0;
    return L;
}
__device__ __forceinline__ RowList owner_range(int base) {   // entry r of range 0 is row base + r
    RowList L = one_range(0, 0);
    L.base0 = base; L.n0 = 0x7fffffff;
    return L;
}

__device__ __forceinline__ BwdTensors at_sequence(const BwdTensors& T, long seq, int D) {
    BwdTensors U;
    U.q = T.q + seq * D; U.k = T.k + seq * D; U.v = T.v + seq * D; U.dout = T.dout + seq * D;
    U.lse = T.lse + seq; U.delta = T.delta + seq;
    U.dq = T.dq + seq * D; U.dk = T.dk + seq * D; U.dv = T.dv + seq * D;
    return U;
}

// dQ pass: the forward pass's blocks (one zone of one chunk, bm rows), last chunk first
template <int D, int NW>
__global__ __launch_bounds__(64 * NW) void bwd_dq_kernel(BwdParams P) {
    extern __shared__ __align__(16) bf16_t smem[];
    const MaskSchedule sch = MaskSchedule::make(P.nbh, P.t, P.R / P.t, P.n, P.bm);
    const MaskJob mj = sch.decode(blockIdx.x);
    const int chunk = mj.y * P.s;
    BwdJob J;
    J.ooff = 0; J.orows = mj.rows;
    J.vis = VIS_CAUSAL; J.cb = NO_CAUSAL; J.t = P.t; J.y_first = 0; J.magic_t = 0; J.rep = 0;
    if (mj.zone == ZONE_READ) {
        J.own = owner_range(chunk + mj.o0);
        J.str = one_range(chunk, mj.o0 + mj.rows);
        J.str.base0 = P.R; J.str.n0 = mj.y * P.t; J.str.slab0 = P.t; J.str.stride0 = P.s; J.str.magic0 = magic_of(P.t);
        J.cb = J.str.n0 + mj.o0;
    } else if (mj.zone == ZONE_MEM) {
        J.own = owner_range(chunk + P.R + mj.o0);
        J.str = one_range(chunk, P.R + P.t);
    } else {
        J.own = owner_range(chunk + P.R + P.t + mj.o0);
        J.str = one_range(chunk + P.R, P.t);
        J.rep = 1;
    }
    J.nstr = J.str.n0 + J.str.n1;
    const BwdTensors T = at_sequence(P.T, (long)mj.bh * P.n * P.s, D);
    bwd_job<D, NW, PASS_DQ>(J, T, P.scale, P.sc, smem);
}

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

// delta[row] = dout[row] . out[row], rows in the row layout (lane = 16-byte piece)
template <int D>
__global__ __launch_bounds__(256) void bwd_delta_kernel(const bf16_t* out, const bf16_t* dout, float* delta, long rows) {
    constexpr int CPR = D / 8;
    const long row = ((long)blockIdx.x * 256 + threadIdx.x) / CPR;
    const int pc = threadIdx.x % CPR;
    const long rc = row < rows ? row : rows - 1;
    const u32x4 a = *reinterpret_cast<const u32x4*>(out + rc * D + pc * 8);
    const u32x4 b = *reinterpret_cast<const u32x4*>(dout + rc * D + pc * 8);
    const float s = row_sum<CPR>(dot8(a, b));
    if (pc == 0 && row < rows) delta[row] = s;
}

template <typename K>
int launch(K kernel, long long grid, int threads, int smem_bytes, const BwdParams& P, hipStream_t st) {
    if (grid <= 0 || grid > 0x7fffffffLL) return LOMA_ERR_UNSUPPORTED;
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            smem_bytes) != hipSuccess)
        return LOMA_ERR_LAUNCH;
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(threads), smem_bytes, st, P);
    return hipGetLastError() == hipSuccess ? LOMA_OK : LOMA_ERR_LAUNCH;
}

template <int D, int NW>
int launch_passes(const BwdParams& P, hipStream_t st) {
    const int smem = BCfg<D>::smem_bytes(NW);
    const long long dq_grid = MaskSchedule::make(P.nbh, P.t, P.R / P.t, P.n, P.bm).size();
    if (int rc = launch(bwd_dq_kernel<D, NW>, dq_grid, 64 * NW, smem, P, st)) return rc;
    const long long nMK = ((long long)P.n * P.t + P.bm - 1) / P.bm, nRB = (P.R + P.bm - 1) / P.bm;
    return launch(bwd_dkv_kernel<D, NW>, (long long)P.nbh * (nMK + (long long)P.n * nRB), 64 * NW, smem, P, st);
}

template <int D>
int launch_d(const BwdParams& P, const void* out, long long rows, hipStream_t st) {
    const long long dgrid = (rows * (D / 8) + 255) / 256;
    if (dgrid > 0x7fffffffLL) return LOMA_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(bwd_delta_kernel<D>, dim3((unsigned)dgrid), dim3(256), 0, st, (const bf16_t*)out, P.T.dout,
                       const_cast<float*>(P.T.delta), (long)rows);
    if (hipGetLastError() != hipSuccess) return LOMA_ERR_LAUNCH;
    if (P.bm == 128) return launch_passes<D, 4>(P, st);
    if (P.bm == 64) return launch_passes<D, 2>(P, st);
    return launch_passes<D, 1>(P, st);
}

}  // namespace

bool mask_attn_bwd_mfma_fits(const Geometry& g) {
    // the slab divisions by multiplication are exact while (list index) * (slab length) < 2^32
    return (long long)g.S * g.s < (1LL << 32);
}

int launch_mask_attn_bwd_mfma(const void* q, const void* k, const void* v, const void* out, const float* lse,
                              const void* dout, void* dq, void* dk, void* dv, float* delta,
                              int nbh, int D, const Geometry& g, float scale, hipStream_t st) {
    BwdParams P;
    P.T.q = (const bf16_t*)q; P.T.k = (const bf16_t*)k; P.T.v = (const bf16_t*)v; P.T.dout = (const bf16_t*)dout;
    P.T.lse = lse; P.T.delta = delta;
    P.T.dq = (bf16_t*)dq; P.T.dk = (bf16_t*)dk; P.T.dv = (bf16_t*)dv;
    P.nbh = nbh; P.n = g.n; P.t = g.t; P.R = g.R; P.s = g.s;
    P.bm = mask_block_rows(g.R);
    P.scale = scale; P.sc = scale * LOG2E;
    const long long rows = (long long)nbh * g.S;
    if (D == 128) return launch_d<128>(P, out, rows, st);
    return launch_d<64>(P, out, rows, st);
}

}  // namespace loma
