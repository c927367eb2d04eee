// MFMA kernels of the LoMA hot path for gfx950: the mask pass (Sec. 4.3 Eq. 1-3 with
// Sec. 4.4 Eq. 5-7) and the compression pass of the generation form (Sec. 3.1 step 2).
//
// One workgroup owns up to 32*NW query rows of ONE zone of ONE chunk; every wave owns 32 of
// them.  The keys such a block can see form a short list of contiguous row ranges that
// follows from (chunk, zone) alone -- the mask is never stored and tiles outside the list
// are never touched:
//     reading rows   : memory zones of chunks 0..y-1 (t rows every s rows), then rows
//                      0..o of the own reading zone (causal, only the last tiles are cut);
//     memory rows    : the own reading zone followed by the own memory zone, uncut;
//     repetition rows: the own memory zone, plus each row's own key (done on the vector
//                      ALU from registers: a diagonal is no MFMA tile).
// Per 32x32 tile the scores are produced TRANSPOSED, S^T = K Q^T (keys down the rows,
// queries across the lanes), so a query's softmax statistics live in two lanes (l, l^32)
// and the probabilities come out of the accumulators already in the register layout the
// second product O^T += V^T P^T wants as its B operand.  K and V tiles go from HBM straight into
// LDS (global_load_lds_dwordx4: no registers, no LDS store instructions), row-major with the
// 16-byte pieces of every row XOR-permuted so that both read patterns are free of bank
// conflicts: the K operand is a plain 16-byte LDS read, the V^T operand comes from the
// transposing LDS read of gfx950 (ds_read_b64_tr_b16: inside 16 lanes, lane i receives the i-th
// 16-bit column of four rows).  Tiles are double-buffered: the loads for tile i+1 are in flight
// while tile i is multiplied; one barrier per tile.
#include <mutex>
#include <set>
#include <type_traits>
#include <utility>

#include "loma_mfma.h"
#include "loma_rope.h"

namespace loma {
namespace {

using namespace mfma;

constexpr float LAZY_TAU = 8.f;   // a softmax reference may lag the running maximum by this much (exp2 units)

struct FlashJob {
    const bf16_t* q;   // first query row of this block, rows contiguous
    bf16_t* out;
    float* lse;        // first row's slot, or nullptr
    int q_rows;        // valid rows in this block
    // keys: three ranges walked back to back; range 0 is slab-strided
    const bf16_t *k0, *k1, *k2, *v0, *v1, *v2;
    int n0, n1, n2;
    int slab;          // rows per slab in range 0
    unsigned slab_magic;  // floor(2^32 / slab) + 1: j / slab == umulhi(j, magic) while j * slab < 2^32
    long slab_stride;  // elements between slabs
    int causal_base;   // key j is visible to block row r iff j <= causal_base + r
    int rows_grouped;  // every range boundary and the slab length are multiples of the rows one direct load covers
    const bf16_t *k_self, *v_self;  // rows aligned with q (repetition zone) or nullptr
};

template <int D, int NW, int BN>
struct Cfg {
    static constexpr int NT = 64 * NW;
    static constexpr int WROWS = 32;        // query rows per wave
    static constexpr int BM = WROWS * NW;
    static constexpr int CPR = D / 8;        // 16-byte pieces per row
    // Tiles are dense [BN][D] in LDS (the direct loads write 1 KB runs); instead of padding, the
    // 16-byte piece c of tile row r is stored at piece position c ^ swizzle(r):
    //   K: swizzle = r % CPR        -> 16 lanes reading one piece of 16 consecutive rows hit 16 banks groups
    //   V: swizzle = 4*(r % 4) % CPR -> the 4 rows x 32 B of a transposing read (two column halves at
    //                                   once) fall into 8 different 32-byte groups
    static constexpr int KBUF = BN * D;
    static constexpr int VBUF = BN * D;
    // tile stages in flight: the loads run NS-1 tiles ahead of the math
    static constexpr int NS = 2;
    static constexpr int RING_BYTES = NS * (KBUF + VBUF) * 2;
    // repetition rows leave through an fp32 staging area (one per wave: 32 rows, padded, plus 32 row factors)
    static constexpr int FSTR = D + 4;
    static constexpr int REP_STAGE_BYTES = NW * (32 * FSTR + 32) * 4;
    // what the repetition rows' job needs: one tile and every wave's queries, later the staging area
    static constexpr int REP_LOAD_BYTES = (KBUF + VBUF + NW * 32 * D) * 2;
    static constexpr int REP_BYTES = REP_LOAD_BYTES > REP_STAGE_BYTES ? REP_LOAD_BYTES : REP_STAGE_BYTES;
    static constexpr int SMEM_BYTES = RING_BYTES > REP_BYTES ? RING_BYTES : REP_BYTES;
    static constexpr int OSTR = D + 8;                   // row stride of the output staging area
    static constexpr int RPI = 64 / CPR;                 // tile rows one wave-wide direct load covers
    static constexpr int IPW = BN / RPI / NW;            // direct loads per wave, per tensor, per tile
    static constexpr int NSUB = BN / 32;
    static constexpr int KSTEPS = D / 16;
    static constexpr int DT = D / 32;
    static_assert(BN % 32 == 0 && D % 32 == 0, "tile shape");
    // what a kernel needs of the configuration it LOADS tiles with (a configuration may also just describe
    // the part of a tile one wave works on)
    static constexpr bool LOADABLE = BN % (RPI * NW) == 0 &&        // tile rows split evenly over the waves
                                     NW <= 2 * (BN / 32) &&          // a ring stage holds the block's queries
                                     NS * (KBUF + VBUF) >= NW * 32 * OSTR;   // output staging fits in the tile buffers
};

// Global row of key j of the job's key list, written with selects only.  (Takes the job by
// value: selecting between fields of a struct that lives behind a reference would turn into an
// indexed load and pin the whole job description in scratch memory.)
template <int D>
__device__ __forceinline__ void key_row(const FlashJob J, int j, const bf16_t*& kp, const bf16_t*& vp) {
    const unsigned a = J.slab == 1 ? (unsigned)j : __umulhi((unsigned)j, J.slab_magic);
    const long off0 = (long)a * J.slab_stride + (long)(j - (int)a * J.slab) * D;
    const int j1 = j - J.n0, j2 = j1 - J.n1;
    const bool in0 = j < J.n0, in1 = j1 < J.n1;
    const long off = in0 ? off0 : (long)(in1 ? j1 : j2) * D;
    kp = (in0 ? J.k0 : (in1 ? J.k1 : J.k2)) + off;
    vp = (in0 ? J.v0 : (in1 ? J.v1 : J.v2)) + off;
}

// Direct HBM -> LDS copy of one K and one V tile.  A wave-wide load moves 64 x 16 B into 1 KB of
// LDS (lane l lands at byte 16*l): RPI whole tile rows.  Each lane picks the global piece that
// belongs at its LDS position under the row's XOR permutation.  Keys past the end of the list
// are clamped to the last key: their scores are masked and their probabilities are exactly 0,
// so any finite row will do and no lane ever branches.
template <int D, int NW, int BN>
__device__ __forceinline__ void load_tile_async(const FlashJob& J, int k0, int nkeys, int w, int lane,
                                                bf16_t* Kb, bf16_t* Vb) {
    using C = Cfg<D, NW, BN>;
    const int p = lane % C::CPR;
#pragma unroll
    for (int i = 0; i < C::IPW; ++i) {
        const int rbase = (w * C::IPW + i) * C::RPI;   // wave-uniform
        const int r = rbase + lane / C::CPR;
        const bf16_t *kp, *vp;
        key_row<D>(J, min(k0 + r, nkeys - 1), kp, vp);
        const int ck = p ^ (r % C::CPR);
        const int cv = p ^ ((4 * (r % 4)) % C::CPR);
        direct_load_16B(kp + ck * 8, Kb + rbase * D);
        direct_load_16B(vp + cv * 8, Vb + rbase * D);
    }
}

// Where wave w keeps its 32 query rows in LDS: the last stage of the tile ring (free until the
// first tile request inside the loop), laid out like a key tile, so the B-operand reads use the
// same per-lane offsets as the K reads.
template <int D, int NW, int BN, int NS = 2>
__device__ __forceinline__ bf16_t* query_stage(bf16_t* smem, int w) {
    using C = Cfg<D, NW, BN>;
    static_assert(C::LOADABLE, "tile configuration");
    bf16_t* Ks = smem;
    bf16_t* Vt = smem + NS * C::KBUF;
    return w < C::NSUB ? Ks + (NS - 1) * C::KBUF + w * 32 * D : Vt + (NS - 1) * C::VBUF + (w - C::NSUB) * 32 * D;
}
// Direct HBM -> LDS copy of the wave's 32 query rows: whole 1 KB runs per instruction instead of
// 32 scattered 32-byte pieces (rows past the block replay its last row, never stored).
template <int D, int NW, int BN>
__device__ __forceinline__ void load_queries_async(const FlashJob& J, int row0, int lane, bf16_t* Qs) {
    using C = Cfg<D, NW, BN>;
    const int p = lane % C::CPR;
#pragma unroll
    for (int i = 0; i < 32 / C::RPI; ++i) {
        const int r = i * C::RPI + lane / C::CPR;
        const int src = min(row0 + r, J.q_rows - 1);
        direct_load_16B(J.q + (long)src * D + (p ^ (r % C::CPR)) * 8, Qs + i * C::RPI * D);
    }
}

// Same copy when the row addresses of a wave-wide load are wave-uniform and advance by a fixed
// stride from tile to tile: the pointers live in scalar registers and cost two scalar adds per
// load and tile; every lane adds a loop-invariant offset.  No vector instruction is spent on
// addresses.  (Possible when the range boundaries and the slab length are multiples of RPI --
// the RPI rows of one load are then consecutive rows of one range -- and a tile covers whole slabs.)
template <int D, int NW, int BN>
__device__ __forceinline__ void load_tile_async_stream(const bf16_t* (&kptr)[Cfg<D, NW, BN>::IPW],
                                                       const bf16_t* (&vptr)[Cfg<D, NW, BN>::IPW],
                                                       long tile_stride, int w,
                                                       const unsigned (&goffk)[Cfg<D, NW, BN>::IPW],
                                                       unsigned goffv, bf16_t* Kb, bf16_t* Vb) {
    using C = Cfg<D, NW, BN>;
#pragma unroll
    for (int i = 0; i < C::IPW; ++i) {
        const int rbase = (w * C::IPW + i) * C::RPI;   // wave-uniform
        const unsigned kdst = __builtin_amdgcn_readfirstlane(
            (unsigned)(size_t)(__attribute__((address_space(3))) bf16_t*)(Kb + rbase * D));
        const unsigned vdst = __builtin_amdgcn_readfirstlane(
            (unsigned)(size_t)(__attribute__((address_space(3))) bf16_t*)(Vb + rbase * D));
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(kdst), "v"(goffk[i]), "s"(kptr[i])
                     : "memory", "m0");
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(vdst), "v"(goffv), "s"(vptr[i])
                     : "memory", "m0");
        kptr[i] += tile_stride;
        vptr[i] += tile_stride;
    }
}

// One key tile for one wave: scores, online softmax, PV.  FULL = every key of the tile is visible
// to every row of the wave (no mask, no sub-tile skipping): the hot path, written as straight-line
// code with the LDS operand reads issued well ahead of the MFMAs that consume them.
template <int D, int NW, int BN, bool FULL>
__device__ __forceinline__ void score_phase(const bf16_t* Kb, const int (&koff)[Cfg<D, NW, BN>::KSTEPS],
                                            const bf16x8 (&qreg)[Cfg<D, NW, BN>::KSTEPS],
                                            f32x16 (&S)[Cfg<D, NW, BN>::NSUB],
                                            int k0, int nsub, const int &my_lim, int lane) {
    using C = Cfg<D, NW, BN>;
    const int g = lane >> 5;
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if constexpr (!FULL) {
#pragma unroll
            for (int sub = 0; sub < C::NSUB; ++sub)
#pragma unroll
                for (int i = 0; i < 16; ++i) S[sub][i] = 0.f;
    }

    // ---- S^T = K Q^T ----------------------------------------------------------------------------
    if constexpr (FULL) {
        // K operands are read AHEAD k-steps before the MFMAs that use them; the scheduling
        // barriers keep the compiler from sinking the reads back next to their uses.
        constexpr int AHEAD = (C::KSTEPS >= 4) ? 4 : C::KSTEPS;
        bf16x8 ka[C::NSUB][AHEAD];
#pragma unroll
        for (int ks = 0; ks < AHEAD; ++ks)
#pragma unroll
            for (int sub = 0; sub < C::NSUB; ++sub)
                ka[sub][ks] = *reinterpret_cast<const bf16x8*>(Kb + koff[ks] + 32 * sub * D);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = 0; ks < C::KSTEPS; ++ks) {
#pragma unroll
            for (int sub = 0; sub < C::NSUB; ++sub)
                if (ks == 0)
                    S[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[sub][0], qreg[0], zero16, 0, 0, 0);
                else
                    S[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[sub][ks % AHEAD], qreg[ks],
                                                                         S[sub], 0, 0, 0);
            if (ks + AHEAD < C::KSTEPS) {
#pragma unroll
                for (int sub = 0; sub < C::NSUB; ++sub)
                    ka[sub][ks % AHEAD] = *reinterpret_cast<const bf16x8*>(
                        Kb + koff[(ks + AHEAD) % C::KSTEPS] + 32 * sub * D);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    } else {
#pragma unroll
        for (int sub = 0; sub < C::NSUB; ++sub)
            if (sub < nsub) {
#pragma unroll
                for (int ks = 0; ks < C::KSTEPS; ++ks) {
                    const bf16x8 a = *reinterpret_cast<const bf16x8*>(Kb + koff[ks] + 32 * sub * D);
                        S[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[ks], S[sub], 0, 0, 0);
                }
            }
        // accumulator i of lane (l32, g) is key 8*(i/4) + 4*g + i%4 of the sub-tile
#pragma unroll
            for (int sub = 0; sub < C::NSUB; ++sub)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int j = k0 + 32 * sub + 8 * (i >> 2) + 4 * g + (i & 3);
                    if (j > my_lim) S[sub][i] = -INFINITY;
                }
    }
}

// Largest score of every query over one fully visible tile, joined with the running reference m.
template <int D, int NW, int BN>
__device__ __forceinline__ void tile_row_max(const f32x16 (&S)[Cfg<D, NW, BN>::NSUB], const float &m,
                                             float &mx) {
    using C = Cfg<D, NW, BN>;
    float x = m;
#pragma unroll
    for (int sub = 0; sub < C::NSUB; ++sub)
#pragma unroll
        for (int i = 0; i < 16; ++i) x = fmaxf(x, S[sub][i]);
    mx = pair_max(x);
}

// RESCALE = false: the caller has checked that no query's maximum exceeds its reference m by more
// than LAZY_TAU (in exp2 units), so m, and with it the scale of O and of the running sum, stay as
// they are: probabilities are at most 2^LAZY_TAU, harmless in fp32 and in bf16, and the 64
// multiplies of O are saved.  The final normalisation divides by a sum taken in the same scale.
template <int D, int NW, int BN, bool FULL, bool RESCALE = true, bool HAVE_MAX = false>
__device__ __forceinline__ void softmax_pv_phase(const bf16_t* Vb, const int (&voff)[Cfg<D, NW, BN>::DT],
                                                 f32x16 (&S)[Cfg<D, NW, BN>::NSUB],
                                                 f32x16 (&O)[Cfg<D, NW, BN>::DT], float &m,
                                                 float &lsum, float sc, int nsub, int lane,
                                                 const float* mx_in = nullptr) {
    using C = Cfg<D, NW, BN>;
    // ---- online softmax (per query: lanes l and l^32) ---------------------------------------------
    float mx = m;
    if constexpr (RESCALE) {
        if constexpr (HAVE_MAX) {
            mx = *mx_in;
        } else {
#pragma unroll
            for (int sub = 0; sub < C::NSUB; ++sub)
                if (FULL || sub < nsub) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) mx = fmaxf(mx, S[sub][i]);
                }
            mx = pair_max(mx);
        }
        // rescale by exp2((m_old - m_new) * sc): exactly 1 for the rows whose maximum did not move.
        // (No branch around it here: a branch makes the compiler keep two copies of O.)
        // A row that has seen no key yet and sees none in a cut tile (possible when the keys of a tile are
        // split over wave groups) keeps m = -inf; the arithmetic then runs against 0 instead: factor 0 on
        // an O that is 0, probabilities exp2(-inf) = 0.
        const float mref = (!FULL && mx == -INFINITY) ? 0.f : mx;
        const float alpha = __builtin_amdgcn_exp2f((m - mref) * sc);
        lsum *= alpha;
#pragma unroll
        for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
            for (int i = 0; i < 16; ++i) O[dt][i] *= alpha;
        m = mx;
        mx = mref;
    }
    const float mc = mx * sc;
    float ps = 0.f;
#pragma unroll
    for (int sub = 0; sub < C::NSUB; ++sub)
        if (FULL || sub < nsub) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float p = __builtin_amdgcn_exp2f(S[sub][i] * sc - mc);
                ps += p;
                S[sub][i] = p;
            }
        }
    lsum += ps;

    // ---- O^T += V^T P^T ---------------------------------------------------------------------------------
    // V^T operand: lane (d = 32*dt + l32, half g) needs keys 16*step + 8*a + 4*g + 0..3, a = 0,1
    auto read_v = [&](int step, int dt) -> bf16x8 {
        const bf16_t* vp = Vb + voff[dt] + 16 * step * D;
        const s16x4 lo = lds_read_tr(vp);
        const s16x4 hi = lds_read_tr(vp + 8 * D);
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    auto pack_p = [&](int step) -> bf16x8 {
        const int sub = step >> 1, jj = step & 1;
        uint4 pw;
        pw.x = pack_bf16(S[sub][8 * jj + 0], S[sub][8 * jj + 1]);
        pw.y = pack_bf16(S[sub][8 * jj + 2], S[sub][8 * jj + 3]);
        pw.z = pack_bf16(S[sub][8 * jj + 4], S[sub][8 * jj + 5]);
        pw.w = pack_bf16(S[sub][8 * jj + 6], S[sub][8 * jj + 7]);
        return __builtin_bit_cast(bf16x8, pw);
    };
    constexpr int NSTEP = 2 * C::NSUB;
    if constexpr (FULL) {
        bf16x8 va[2][C::DT];
#pragma unroll
        for (int dt = 0; dt < C::DT; ++dt) va[0][dt] = read_v(0, dt);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int step = 0; step < NSTEP; ++step) {
            if (step + 1 < NSTEP) {
#pragma unroll
                for (int dt = 0; dt < C::DT; ++dt) va[(step + 1) & 1][dt] = read_v(step + 1, dt);
            }
            bf16x8 pb;
            pb = pack_p(step);
#pragma unroll
            for (int dt = 0; dt < C::DT; ++dt)
                    O[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[step & 1][dt], pb, O[dt], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    } else {
#pragma unroll
        for (int step = 0; step < NSTEP; ++step)
            if ((step >> 1) < nsub) {
                bf16x8 pb;
                pb = pack_p(step);
#pragma unroll
                for (int dt = 0; dt < C::DT; ++dt) {
                    const bf16x8 a = read_v(step, dt);
                        O[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb, O[dt], 0, 0, 0);
                }
            }
    }
}

// The query row's own K and V rows, in the register layouts of the Q operand (K) and of the O
// accumulators (V): lane (row l32, half g) holds head-dim 16*ks + 8*g.. of K and 32*dt + 8*i4 + 4*g.. of V.
template <int D, int NW, int BN>
__device__ __forceinline__ void load_self_rows(const FlashJob& J, int r, int g,
                                               bf16x8 (&kself)[Cfg<D, NW, BN>::KSTEPS],
                                               uint2 (&vself)[Cfg<D, NW, BN>::DT][4]) {
    using C = Cfg<D, NW, BN>;
    const int rc = min(r, J.q_rows - 1);   // lanes past the block replay its last row (never stored)
    const bf16_t* kp = J.k_self + (long)rc * D + 8 * g;
    const bf16_t* vp = J.v_self + (long)rc * D + 4 * g;
#pragma unroll
    for (int ks = 0; ks < C::KSTEPS; ++ks)
        kself[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(kp + 16 * ks));
#pragma unroll
    for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) vself[dt][i4] = *reinterpret_cast<const uint2*>(vp + 32 * dt + 8 * i4);
}

// One more key for every query, its own (identity block of Eq. 1, second term of Eq. 9): a dot
// product and an axpy per row on the vector ALU -- a diagonal is no MFMA tile.
template <int D, int NW, int BN>
__device__ __forceinline__ void self_term(const bf16x8 (&qreg)[Cfg<D, NW, BN>::KSTEPS],
                                          const bf16x8 (&kself)[Cfg<D, NW, BN>::KSTEPS],
                                          const uint2 (&vself)[Cfg<D, NW, BN>::DT][4],
                                          f32x16 (&O)[Cfg<D, NW, BN>::DT], float& m, float& lsum, float sc, int g) {
    using C = Cfg<D, NW, BN>;
    float part = 0.f;
#pragma unroll
    for (int ks = 0; ks < C::KSTEPS; ++ks) {
        const bf16x8 kk = kself[ks], qq = qreg[ks];
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            const bf16x2 a = {qq[e], qq[e + 1]};
            const bf16x2 b = {kk[e], kk[e + 1]};
            part = __builtin_amdgcn_fdot2_f32_bf16(a, b, part, false);
        }
    }
    const float sself = pair_sum(part);
    const float mx = fmaxf(m, sself);
    const float alpha = __builtin_amdgcn_exp2f((m - mx) * sc);
    const float p = __builtin_amdgcn_exp2f((sself - mx) * sc);
    lsum = lsum * alpha + (g == 0 ? p : 0.f);
    m = mx;
#pragma unroll
    for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
            const uint2 x = vself[dt][i4];
            O[dt][4 * i4 + 0] = O[dt][4 * i4 + 0] * alpha + p * bf16_lo(x.x);
            O[dt][4 * i4 + 1] = O[dt][4 * i4 + 1] * alpha + p * bf16_hi(x.x);
            O[dt][4 * i4 + 2] = O[dt][4 * i4 + 2] * alpha + p * bf16_lo(x.y);
            O[dt][4 * i4 + 3] = O[dt][4 * i4 + 3] * alpha + p * bf16_hi(x.y);
        }
}

// Normalise, transpose through LDS (the tile buffers are free by now), store rows as 16-byte
// pieces; one query tile at a time through the wave's own 32-row staging area.
template <int D, int NW, int BN>
__device__ __forceinline__ void store_rows(const FlashJob& J, f32x16 (&O)[Cfg<D, NW, BN>::DT],
                                           const float &m, const float &lsum, float sc, bf16_t* smem,
                                           int w, int lane, int row0, bool has_rows) {
    using C = Cfg<D, NW, BN>;
    const int g = lane >> 5, l32 = lane & 31;
    bf16_t* Os = smem + w * 32 * C::OSTR;
    const int rbase = row0;
    const float ltot = pair_sum(lsum);
    const float inv = 1.f / ltot;
    if (has_rows) {
#pragma unroll
        for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                uint2 x;
                x.x = pack_bf16(O[dt][4 * i4 + 0] * inv, O[dt][4 * i4 + 1] * inv);
                x.y = pack_bf16(O[dt][4 * i4 + 2] * inv, O[dt][4 * i4 + 3] * inv);
                *reinterpret_cast<uint2*>(Os + l32 * C::OSTR + 32 * dt + 8 * i4 + 4 * g) = x;
            }
        if (J.lse != nullptr && g == 0 && rbase + l32 < J.q_rows)
            J.lse[rbase + l32] = (m * sc + __builtin_amdgcn_logf(ltot)) * LN2;
    }
    __syncthreads();
    if (has_rows) {
#pragma unroll
        for (int it = 0; it < 32 * C::CPR / 64; ++it) {
            const int idx = it * 64 + lane;
            const int r = idx / C::CPR, ch = idx % C::CPR;
            if (rbase + r < J.q_rows)
                *reinterpret_cast<uint4*>(J.out + (long)(rbase + r) * D + ch * 8) =
                    *reinterpret_cast<const uint4*>(Os + r * C::OSTR + ch * 8);
        }
    }
}

// KS > 1 splits the KEYS of every tile over KS groups of waves (for launches with few workgroups, where
// one workgroup walks a long key list alone): the block has 32 * NW / KS rows, wave w owns row group
// w % (NW / KS) and, of every tile of BN keys, the BN / KS keys of key group w / (NW / KS).  All waves
// share the loads; the groups' partial results (same register layout in every wave) meet in LDS at
// the end.
template <int D, int NW, int BN, int KS = 1, int NS = 2>
__device__ __forceinline__ void flash_job(const FlashJob& J, float sc, bf16_t* smem) {
    using C = Cfg<D, NW, BN>;            // tiles as they are loaded (the ring has NS stages)
    constexpr int BNC = BN / KS;             // keys of a tile one wave works on
    using CC = Cfg<D, NW, BNC>;
    constexpr int RG = NW / KS;              // row groups
    static_assert(NW % KS == 0 && BN % (32 * KS) == 0, "key split");
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave index, kept in a scalar register
    const int kg = w / RG;                                      // key group of this wave
    const int g = lane >> 5, l32 = lane & 31;
    bf16_t* Ks = smem;
    bf16_t* Vt = smem + NS * C::KBUF;
    const int wk0 = kg * BNC;                                   // first key of the wave's part of a tile

    const int nkeys = J.n0 + J.n1 + J.n2;
    const int kend_wg = min(nkeys, J.causal_base + J.q_rows);
    const int ntiles = (kend_wg + BN - 1) / BN;
    const int row0 = C::WROWS * (w % RG);                 // first block row of this wave
    const bool has_rows = row0 < J.q_rows;
    const int row_hi = min(row0 + C::WROWS, J.q_rows);    // exclusive
    const int kend_w = has_rows ? min(nkeys, J.causal_base + row_hi) : 0;
    int my_lim;                                       // last key each of this lane's queries sees
        my_lim = min(J.causal_base + min(row0 + l32, J.q_rows - 1), nkeys - 1);

    // Q^T as the B operand: lane (query l32, half g) holds head-dim 16*ks + 8*g .. +7; it arrives through LDS
    bf16x8 qreg[C::KSTEPS];
    bf16_t* Qs = query_stage<D, NW, BN, NS>(smem, w);
    load_queries_async<D, NW, BN>(J, row0, lane, Qs);

    f32x16 O[C::DT];
    float m, lsum;
    m = -INFINITY;
    lsum = 0.f;
#pragma unroll
    for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) O[dt][i] = 0.f;

    // per-lane LDS offsets (elements) of the operand reads, under the tiles' XOR permutations
    int koff[C::KSTEPS], voff[C::DT];
#pragma unroll
    for (int ks = 0; ks < C::KSTEPS; ++ks) koff[ks] = l32 * D + (((2 * ks + g) ^ (l32 % C::CPR)) * 8);
    {
        const int i = lane & 15, q = i >> 2;   // source-lane role in the transposing read: row q, columns 4*(i%4)..
#pragma unroll
        for (int dt = 0; dt < C::DT; ++dt)
            voff[dt] = (4 * g + q) * D + (4 * (dt ^ (q % (C::CPR / 4))) + 2 * ((lane >> 4) & 1) + ((i & 3) >> 1)) * 8 +
                       4 * (i & 1);
    }

    // per-lane byte offsets of the streamed direct loads (row inside the group, permuted piece)
    unsigned goffk[C::IPW], goffv;
    {
        const int rl = lane / C::CPR, pc = lane % C::CPR;
#pragma unroll
        for (int i = 0; i < C::IPW; ++i)
            goffk[i] = 2u * (rl * D + ((pc ^ (((w * C::IPW + i) * C::RPI + rl) % C::CPR)) * 8));
        goffv = 2u * (rl * D + ((pc ^ ((4 * (rl % 4)) % C::CPR)) * 8));
    }

    // Tiles that every row of the block sees in full come first and run in a loop of their own:
    // straight-line code, no per-wave decisions except that a wave without rows (a block shorter
    // than BM) only helps with the loads.  This is where the time goes.
    const int nfull = min(ntiles, (min(J.causal_base, nkeys - 1) + 1) / BN);
    // Leading tiles whose loads can stream with scalar pointers: whole slabs of range 0 per tile,
    // or a contiguous range 1 when there is no range 0.
    int nstream = 0;
    long tile_stride = 0;
    if (J.rows_grouped) {
        if (J.n0 > 0) {
            if (BN % J.slab == 0) { nstream = min(nfull, J.n0 / BN); tile_stride = (long)(BN / J.slab) * J.slab_stride; }
        } else {
            nstream = min(nfull, J.n1 / BN);
            tile_stride = (long)BN * D;
        }
    }
    constexpr int AHEAD = NS - 1;          // tiles requested ahead of the one being multiplied
    constexpr int LPT = 2 * C::IPW;           // direct loads per wave and tile
    const bf16_t *kptr[C::IPW], *vptr[C::IPW];
#pragma unroll
    for (int i = 0; i < C::IPW; ++i) {
        const bf16_t *kp, *vp;
        key_row<D>(J, min((w * C::IPW + i) * C::RPI, nkeys - 1), kp, vp);
        kptr[i] = uniform_ptr(kp) + AHEAD * tile_stride;   // the first streamed tile is tile AHEAD
        vptr[i] = uniform_ptr(vp) + AHEAD * tile_stride;
    }
    // request tile `t` into its stage (streamed with scalar pointers when it qualifies)
    auto request_tile = [&](int t) {
        bf16_t* Kd = Ks + (t % NS) * C::KBUF;
        bf16_t* Vd = Vt + (t % NS) * C::VBUF;
        if (t >= AHEAD && t < nstream)
            load_tile_async_stream<D, NW, BN>(kptr, vptr, tile_stride, w, goffk, goffv, Kd, Vd);
        else
            load_tile_async<D, NW, BN>(J, t * BN, nkeys, w, lane, Kd, Vd);
    };
#pragma unroll
    for (int t = 0; t < AHEAD; ++t)
        if (t < ntiles) request_tile(t);
    wait_next_tile<LPT, AHEAD - 1>(min(AHEAD, ntiles) - 1);   // tile 0 and the queries are in
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < C::KSTEPS; ++ks) qreg[ks] = *reinterpret_cast<const bf16x8*>(Qs + koff[ks]);
    __syncthreads();   // ring stage 1 belongs to the tiles from here on

    // The fast loop keeps the softmax reference m (and so the scale of O) while no query's maximum
    // moves up by more than LAZY_TAU; when one does, the wave leaves the loop with the scores in
    // hand, finishes that tile with a rescale and comes back.  Every path passes one barrier per tile.
    {
        int kt = 0;
        while (kt < nfull) {
            f32x16 S[CC::NSUB];
            float mx;
            bool moved = false;
            for (; kt < nfull; ++kt) {
                const int st = kt % NS;
                if (kt + AHEAD < ntiles) request_tile(kt + AHEAD);
                if (has_rows) {
                    score_phase<D, NW, BNC, true>(Ks + st * C::KBUF + wk0 * D, koff, qreg, S, kt * BN + wk0, CC::NSUB,
                                                      my_lim, lane);
                    tile_row_max<D, NW, BNC>(S, m, mx);
                    if (__builtin_amdgcn_ballot_w64((mx - m) * sc > LAZY_TAU) != 0) { moved = true; break; }
                    softmax_pv_phase<D, NW, BNC, true, false>(Vt + st * C::VBUF + wk0 * D, voff, S, O, m, lsum, sc,
                                                                  CC::NSUB, lane);
                }
                wait_next_tile<LPT, AHEAD - 1>(min(kt + AHEAD, ntiles - 1) - (kt + 1));
                __syncthreads();
            }
            if (moved) {
                softmax_pv_phase<D, NW, BNC, true, true, true>(Vt + (kt % NS) * C::VBUF + wk0 * D, voff, S, O, m, lsum,
                                                                    sc, CC::NSUB, lane, &mx);
                wait_next_tile<LPT, AHEAD - 1>(min(kt + AHEAD, ntiles - 1) - (kt + 1));
                __syncthreads();
                ++kt;
            }
        }
    }
    // The remaining tiles: cut by the causal diagonal or by the end of the key list, differently
    // for every wave (a wave past its last visible key only helps with the loads).
    for (int kt = nfull; kt < ntiles; ++kt) {
        const int st = kt % NS;
        const int k0 = kt * BN + wk0;    // first key of this wave's part of the tile
        if (kt + AHEAD < ntiles) request_tile(kt + AHEAD);
        if (k0 < kend_w) {
            const int nsub = min(CC::NSUB, (kend_w - k0 + 31) >> 5);
            f32x16 S[CC::NSUB];
            score_phase<D, NW, BNC, false>(Ks + st * C::KBUF + wk0 * D, koff, qreg, S, k0, nsub, my_lim, lane);
            softmax_pv_phase<D, NW, BNC, false>(Vt + st * C::VBUF + wk0 * D, voff, S, O, m, lsum, sc, nsub, lane);
        }
        wait_next_tile<LPT, AHEAD - 1>(min(kt + AHEAD, ntiles - 1) - (kt + 1));
        __syncthreads();
    }

    // key groups 1.. hand their partial results to group 0 of the same rows: every wave holds O, m and the
    // running sum in the same registers of the same lanes, so they cross LDS as plain [register][lane] arrays
    if constexpr (KS > 1) {
        float* xs = reinterpret_cast<float*>(smem);   // the ring is free: the loop's last barrier has been passed
        constexpr int PER_WAVE = (16 * C::DT + 2) * 64;
        if (kg > 0 && has_rows) {
            float* dst = xs + (size_t)(w - RG) * PER_WAVE + lane;
#pragma unroll
            for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
                for (int i = 0; i < 16; ++i) dst[(16 * dt + i) * 64] = O[dt][i];
            dst[16 * C::DT * 64] = m;
            dst[(16 * C::DT + 1) * 64] = lsum;
        }
        __syncthreads();
        if (kg == 0 && has_rows) {
#pragma unroll
            for (int k = 1; k < KS; ++k) {
                const float* src = xs + (size_t)(w + (k - 1) * RG) * PER_WAVE + lane;
                const float mb = src[16 * C::DT * 64], lb = src[(16 * C::DT + 1) * 64];
                const float mx = fmaxf(m, mb);
                // a group that saw no key has m = -inf, sum 0 and O = 0: its factor is exp2(-inf) = 0
                const float fa = __builtin_amdgcn_exp2f((m - mx) * sc), fb = __builtin_amdgcn_exp2f((mb - mx) * sc);
                lsum = lsum * fa + lb * fb;
                m = mx;
#pragma unroll
                for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
                    for (int i = 0; i < 16; ++i) O[dt][i] = O[dt][i] * fa + src[(16 * dt + i) * 64] * fb;
            }
        }
        __syncthreads();   // the exchange area becomes the staging area of store_rows
    }
    const bool owns_rows = has_rows && kg == 0;
    // the row's own key (identity block of Eq. 1, second term of Eq. 9), on the vector ALU
    if (J.k_self != nullptr && owns_rows) {
        bf16x8 kself[C::KSTEPS];
        uint2 vself[C::DT][4];
        load_self_rows<D, NW, BN>(J, row0 + l32, g, kself, vself);
        self_term<D, NW, BN>(qreg, kself, vself, O, m, lsum, sc, g);
    }
    store_rows<D, NW, BN>(J, O, m, lsum, sc, smem, w, lane, row0, owns_rows);
}

// ---- the pipelined job ----------------------------------------------------------------------------------
// For blocks with long key lists (reading rows behind many memory zones) the matrix pipe and the vector ALU have
// about the same amount of work per tile (32 MFMAs of 32 cycles against ~800 cycles of exponentials, packing and
// sums), and a wave that does them one after the other leaves each unit idle half of the time.  Here the loop
// over the tiles (fully visible ones first, then those cut by the causal diagonal or the end of the key list, with a
// per-lane key threshold) is software-pipelined over HALF tiles of 32 keys: while the vector ALU turns the
// scores of half h into probabilities, the matrix pipe multiplies the scores of half h+1 and the P.V product of
// half h-1, one MFMA every few vector instructions, in one instruction stream.  Half h-1's V rows must stay
// while half h+1's K rows are read, so the ring holds two K stages and three V stages of 64 keys (80 KB at
// head_dim 128: two workgroups per CU); one barrier per tile, between its two halves.
//
// The softmax reference m is taken from the first half tile and kept while no probability leaves the range
// [0, 2^PIPE_TAU]: the test is one compare per half on the lane's partial sum (a probability cannot exceed a sum
// it is part of); when it trips, the wave leaves the pipelined loop and finishes its tiles one by one, moving
// the reference as it goes.
constexpr float PIPE_TAU = 40.f;

// Ring of the pipelined job: NSK stages of K and NSK + 1 stages of V tiles of 64 keys (a V tile is needed one half
// tile longer than its K tile), loads running NSK - 1 tiles ahead.  Queries are staged in the last QP K stages and
// the last QP V stages (two waves per stage), which are free until tile NSK - QP is requested.
template <int D, int NW, int NSK>
struct PipeCfg {
    using C = Cfg<D, NW, 64>;
    static constexpr int NSV = NSK + 1;
    static constexpr int QP = (NW + 3) / 4;                                     // stage pairs holding the queries
    static constexpr int RING = NSK * C::KBUF + NSV * C::VBUF;                  // elements
    static constexpr int SMEM_BYTES = RING * 2;
    static_assert(RING >= NW * 32 * C::OSTR, "output staging fits in the ring");
    static_assert(NSK >= 2 && NSK <= 4 && QP < NSK, "ring depth");
};

// One step of the pipeline.  Matrix pipe: Sn = K rows of half h+1 times Q (HAVE_S), O += V^T of half h-1 times
// Pp (HAVE_PV), alternating; vector ALU, between them: probabilities Pc of the scores Sc of half h (HAVE_P).
// Kh / Vh point at the first of the 32 rows of the respective half inside its ring stage.
// The step is cut into slots of one MFMA, the slot's share of the scores and the operand read that runs RA products
// ahead, with a scheduling fence after every slot; the exponentials, the packing and the MFMAs are volatile
// statements, which the compiler keeps in source order among themselves and against the fences (written as plain
// arithmetic it sank every exponential behind the MFMAs; given as scheduling groups the order held but ran 2-3 %
// slower than this).  Nothing reads an MFMA's result before the next step.
template <int D, bool HAVE_S, bool HAVE_PV, bool HAVE_P = true, bool MASKED = false>
__device__ __forceinline__ float pipe_half(const bf16_t* Kh, const bf16_t* Vh, const int (&koff)[D / 16], const int (&voff)[D / 32],
                                           const bf16x8 (&qreg)[D / 16], const f32x16& Sc, f32x16& Sn,
                                           const bf16x8 (&Pp)[2], bf16x8 (&Pc)[2], f32x16 (&O)[D / 32], float sc, float mc,
                                           int thr = 0) {
    constexpr int KSTEPS = D / 16, DT = D / 32, NPV = 2 * DT;
    static_assert(NPV == KSTEPS, "as many P.V products as score products per half tile");
    constexpr int NSLOT = 2 * KSTEPS, EPS = 16 / NSLOT;      // slots of one MFMA each; scores handled per slot
    constexpr int RA = 2;                                   // operand reads run this many products of their kind ahead
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    auto read_k = [&](int ks) -> bf16x8 { return *reinterpret_cast<const bf16x8*>(Kh + koff[ks]); };
    auto read_v = [&](int idx) -> bf16x8 {      // product idx: 16-key step idx / DT, head-dim block idx % DT
        const bf16_t* vp = Vh + voff[idx % DT] + 16 * (idx / DT) * D;
        const s16x4 lo = lds_read_tr(vp);
        const s16x4 hi = lds_read_tr(vp + 8 * D);
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    bf16x8 ka[KSTEPS], va[NPV];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < RA; ++i) {
        if constexpr (HAVE_S) ka[i] = read_k(i);
        if constexpr (HAVE_PV) va[i] = read_v(i);
    }
    __builtin_amdgcn_sched_barrier(0);
    uint32_t pw[8];
    float pe[2];
    float ps = 0.f;
    static_for<0, NSLOT>([&](auto sc_) {
        constexpr int slot = sc_.value, j = slot >> 1;
        if constexpr (HAVE_P) {
            static_for<slot * EPS, (slot + 1) * EPS>([&](auto ec) {
                constexpr int e = ec.value;
                float y = exp2_at(__builtin_fmaf(Sc[e], sc, -mc));
                // MASKED: element e is key 8 (e / 4) + e % 4 (+ 4 g, folded into thr) of the half tile; the lane's row
                // sees it iff that number does not exceed the lane's threshold
                if constexpr (MASKED) y = (8 * (e / 4) + e % 4 <= thr) ? y : 0.f;
                pe[e & 1] = y;
                ps += y;
                if constexpr (e & 1) pw[e >> 1] = pack_bf16_at(pe[0], pe[1]);
            });
        }
        if constexpr ((slot & 1) == 0) {
            if constexpr (HAVE_S) {
                if constexpr (j == 0) mfma_first_at(Sn, ka[0], qreg[0]);
                else mfma_at(Sn, ka[j], qreg[j]);
                if constexpr (j + RA < KSTEPS) ka[j + RA] = read_k(j + RA);
            }
        } else {
            if constexpr (HAVE_PV) {
                mfma_at(O[j % DT], va[j], Pp[j / DT]);
                if constexpr (j + RA < NPV) va[j + RA] = read_v(j + RA);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    });
    if constexpr (!HAVE_P) return 0.f;
    Pc[0] = __builtin_bit_cast(bf16x8, uint4{pw[0], pw[1], pw[2], pw[3]});
    Pc[1] = __builtin_bit_cast(bf16x8, uint4{pw[4], pw[5], pw[6], pw[7]});
    return ps;
}

template <int D, int NW, int NSK>
__device__ __forceinline__ void flash_job_pipe(const FlashJob& J, float sc, bf16_t* smem) {
    constexpr int BN = 64;
    using C = Cfg<D, NW, BN>;
    using PC = PipeCfg<D, NW, NSK>;
    constexpr int NSV = PC::NSV;
    constexpr int LPT = 2 * C::IPW;        // direct loads per wave and tile
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 5, l32 = lane & 31;
    bf16_t* Ks = smem;
    bf16_t* Vt = smem + NSK * C::KBUF;
    auto kstage = [&](int t) { return Ks + (t % NSK) * C::KBUF; };
    auto vstage = [&](int t) { return Vt + (t % NSV) * C::VBUF; };

    const int nkeys = J.n0 + J.n1 + J.n2;
    const int kend_wg = min(nkeys, J.causal_base + J.q_rows);
    const int ntiles = (kend_wg + BN - 1) / BN;
    const int row0 = 32 * w;
    const bool has_rows = row0 < J.q_rows;
    const int row_hi = min(row0 + 32, J.q_rows);
    const int kend_w = has_rows ? min(nkeys, J.causal_base + row_hi) : 0;
    const int my_lim = min(J.causal_base + min(row0 + l32, J.q_rows - 1), nkeys - 1);

    // queries: staged like key tiles in the last QP stages of K and of V, two waves per stage
    bf16x8 qreg[C::KSTEPS];
    bf16_t* Qs = (w & 2) ? Vt + (NSV - 1 - (w >> 2)) * C::VBUF + (w & 1) * 32 * D
                         : Ks + (NSK - 1 - (w >> 2)) * C::KBUF + (w & 1) * 32 * D;
    load_queries_async<D, NW, BN>(J, row0, lane, Qs);

    f32x16 O[C::DT];
    float m = -INFINITY, lsum = 0.f;
#pragma unroll
    for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) O[dt][i] = 0.f;

    int koff[C::KSTEPS], voff[C::DT];
#pragma unroll
    for (int ks = 0; ks < C::KSTEPS; ++ks) koff[ks] = l32 * D + (((2 * ks + g) ^ (l32 % C::CPR)) * 8);
    {
        const int i = lane & 15, q = i >> 2;
#pragma unroll
        for (int dt = 0; dt < C::DT; ++dt)
            voff[dt] = (4 * g + q) * D + (4 * (dt ^ (q % (C::CPR / 4))) + 2 * ((lane >> 4) & 1) + ((i & 3) >> 1)) * 8 +
                       4 * (i & 1);
    }
    unsigned goffk[C::IPW], goffv;
    {
        const int rl = lane / C::CPR, pc = lane % C::CPR;
#pragma unroll
        for (int i = 0; i < C::IPW; ++i)
            goffk[i] = 2u * (rl * D + ((pc ^ (((w * C::IPW + i) * C::RPI + rl) % C::CPR)) * 8));
        goffv = 2u * (rl * D + ((pc ^ ((4 * (rl % 4)) % C::CPR)) * 8));
    }

    // tiles every row of the block sees in full, and tiles every row of THIS WAVE sees in full: the pipelined loop
    // runs over the latter (a wave-dependent count: the barriers and requests per tile are the same on every path)
    const int nfull_wg = min(ntiles, (min(J.causal_base, nkeys - 1) + 1) / BN);
    const int nfull = has_rows ? min(ntiles, (min(J.causal_base + row0, nkeys - 1) + 1) / BN) : 0;
    int nstream = 0;
    long tile_stride = 0;
    if (J.rows_grouped) {
        if (J.n0 > 0) {
            if (BN % J.slab == 0) { nstream = min(nfull_wg, J.n0 / BN); tile_stride = (long)(BN / J.slab) * J.slab_stride; }
        } else {
            nstream = min(nfull_wg, J.n1 / BN);
            tile_stride = (long)BN * D;
        }
    }
    constexpr int FIRST_STREAMED = NSK;    // tiles 0 .. NSK-1 are requested in the prologue, with per-lane addresses
    const bf16_t *kptr[C::IPW], *vptr[C::IPW];
#pragma unroll
    for (int i = 0; i < C::IPW; ++i) {
        const bf16_t *kp, *vp;
        key_row<D>(J, min((w * C::IPW + i) * C::RPI, nkeys - 1), kp, vp);
        kptr[i] = uniform_ptr(kp) + FIRST_STREAMED * tile_stride;
        vptr[i] = uniform_ptr(vp) + FIRST_STREAMED * tile_stride;
    }
    int next_req = 0;                      // tiles are requested in order; this is the next one
    auto request_next = [&]() {
        const int t = next_req++;
        if (t >= FIRST_STREAMED && t < nstream)
            load_tile_async_stream<D, NW, BN>(kptr, vptr, tile_stride, w, goffk, goffv, kstage(t), vstage(t));
        else
            load_tile_async<D, NW, BN>(J, t * BN, nkeys, w, lane, kstage(t), vstage(t));
    };
    // the wave's loads of every tile up to `upto` have landed (younger requested tiles may still be in flight)
    auto wait_tile = [&](int upto) { wait_next_tile<LPT, NSK - 1>(max(0, next_req - 1 - upto)); };
#pragma unroll
    for (int t = 0; t < NSK - PC::QP; ++t)
        if (t < ntiles) request_next();    // the tiles whose stages the queries do not occupy
    wait_direct_loads();
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < C::KSTEPS; ++ks) qreg[ks] = *reinterpret_cast<const bf16x8*>(Qs + koff[ks]);
    __syncthreads();                       // all stages belong to the tiles from here on
#pragma unroll
    for (int t = 0; t < PC::QP; ++t)
        if (next_req < ntiles) request_next();   // tiles up to NSK-1

    // Pipelined loop.  It runs while every probability stays in range; a half
    // that leaves the range ends it (wave by wave: the barrier count per tile is the same on both paths), and the
    // tile-by-tile loop below, which moves the reference as it goes, takes over at `resume`, after redoing the
    // half in question (`redo_half`) if the tile's first half had already been accumulated.
    int resume = 0;          // first tile the tile-by-tile loop has to do
    int redo_half = -1;      // tile whose second half it has to do first, from its scores, which `Sb` still holds
    int redo_thr = 64;       // ... of whose keys the lane's row sees those up to this number (see pipe_half)
    f32x16 Sa, Sbv[1];       // the two score sets of the pipelined loop; the second one holds the scores to redo
    f32x16& Sb = Sbv[0];
    // Tiles cut by the causal diagonal or by the end of the key list go through the same loop with a per-lane key
    // threshold (MASKED steps), up to the last tile any row of the wave sees; the tile-by-tile loop is left with
    // the barriers and requests of the tiles after it -- and with everything when no tile is fully visible (the
    // reference needs a first half tile without a mask) or the range test trips.
    const int npipe = nfull > 0 ? min(ntiles, (kend_w + BN - 1) / BN) : 0;
    if (nfull > 0) {
        resume = npipe;
        if (has_rows) {
            bf16x8 Pa[2], Pb[2];
            const float range = __builtin_amdgcn_exp2f(PIPE_TAU);
            // scores of the first half tile, alone; the reference is their maximum
            {
                const bf16_t* K0 = kstage(0);
                const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < C::KSTEPS; ++ks) {
                    const bf16x8 a = *reinterpret_cast<const bf16x8*>(K0 + koff[ks]);
                    Sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[ks], ks == 0 ? zero16 : Sa, 0, 0, 0);
                }
                float mx = Sa[0];
#pragma unroll
                for (int i = 1; i < 16; ++i) mx = fmaxf(mx, Sa[i]);
                m = pair_max(mx);
            }
            const float mc = m * sc;
            // first half of tile 0: nothing to multiply by V yet (no probability exceeds 1 here)
            lsum += pipe_half<D, true, false>(kstage(0) + 32 * D, nullptr, koff, voff, qreg, Sa, Sb, Pb, Pa, O, sc, mc);
            // One trip: every wave is done with K stage t and V stage t-1, and everybody's part of tile t+1 is in;
            // second half of tile t (its probabilities; scores of (t+1, 0); P.V of (t, 0)), then first half of tile
            // t+1 (its probabilities; scores of (t+1, 1); P.V of (t, 1)).  The lane's row sees key k of half (T, h)
            // iff 64 T + 32 h + k <= my_lim.
#define LOMA_PIPE_TILE(MASKED_)                                                                                              \
    {                                                                                                                        \
        wait_tile(t + 1);                                                                                                    \
        __syncthreads();                                                                                                     \
        if (next_req < ntiles) request_next(); /* tile t + NSK */                                                            \
        const int thr_b = my_lim - BN * t - 32 - 4 * g, thr_a = my_lim - BN * (t + 1) - 4 * g;                               \
        const float psb = pipe_half<D, true, true, true, MASKED_>(kstage(t + 1), vstage(t), koff, voff, qreg, Sb, Sa, Pa, Pb, \
                                                                  O, sc, mc, thr_b);                                         \
        if (__builtin_amdgcn_ballot_w64(!(psb <= range)) != 0) {                                                             \
            redo_half = t; redo_thr = MASKED_ ? thr_b : 64; resume = t + 1;                                                  \
            break;                                                                                                           \
        }                                                                                                                    \
        lsum += psb;                                                                                                         \
        const float psa = pipe_half<D, true, true, true, MASKED_>(kstage(t + 1) + 32 * D, vstage(t) + 32 * D, koff, voff,    \
                                                                  qreg, Sa, Sb, Pb, Pa, O, sc, mc, thr_a);                   \
        if (__builtin_amdgcn_ballot_w64(!(psa <= range)) != 0) { resume = t + 1; break; }                                    \
        lsum += psa;                                                                                                         \
    }
            int t = 0;
            for (; t + 1 < nfull; ++t) LOMA_PIPE_TILE(false)
            if (resume == npipe)      // (a trip that left the loop early has set `resume` to an earlier tile)
                for (; t + 1 < npipe; ++t) LOMA_PIPE_TILE(true)
#undef LOMA_PIPE_TILE
            if (resume == npipe && t + 1 == npipe) {   // the loop ran to its end: second half of the last tile, then its P.V
                wait_tile(t + 1);
                __syncthreads();
                if (next_req < ntiles) request_next();
                const int thr_b = my_lim - BN * t - 32 - 4 * g;
                // (masked in any case: a fully visible half passes the test in every lane)
                const float psb = pipe_half<D, false, true, true, true>(nullptr, vstage(t), koff, voff, qreg, Sb, Sa, Pa, Pb, O, sc, mc, thr_b);
                if (__builtin_amdgcn_ballot_w64(!(psb <= range)) != 0) {
                    redo_half = t;
                    redo_thr = thr_b;
                } else {
                    lsum += psb;
                    f32x16 none;
                    bf16x8 unused[2];
                    (void)pipe_half<D, false, true, false>(nullptr, vstage(t) + 32 * D, koff, voff, qreg, Sb, none, Pb, unused, O, sc, mc);
                }
            }
        }
    }
    // the pipelined loop's MFMAs are invisible to the compiler's hazard bookkeeping: let the last of them write its
    // accumulator before ordinary code reads the scores or the output accumulators
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 7" ::: "memory");
    if (redo_half >= 0) {
        // second half of tile `redo_half` with a moving reference, from its scores (masked here if the half is a cut
        // one; its K rows may be gone by now, its V rows stay until tile redo_half + 3 is requested)
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if (8 * (i >> 2) + (i & 3) > redo_thr) Sbv[0][i] = -INFINITY;
        softmax_pv_phase<D, NW, 32, false>(vstage(redo_half) + 32 * D, voff, Sbv, O, m, lsum, sc, 1, lane);
    }
    // Tile by tile: what the pipelined loop left, and the tiles cut by the causal diagonal or by the end of the key
    // list, differently for every wave.  Tile kt is in (everybody's part: the barrier that ended the previous tile
    // came after the wait for it).
    for (int kt = resume; kt < ntiles; ++kt) {
        if (next_req <= kt + NSK - 1 && next_req < ntiles) request_next();
        const int k0 = kt * BN;
        if (k0 < kend_w) {
            const int nsub = min(C::NSUB, (kend_w - k0 + 31) >> 5);
            f32x16 S[C::NSUB];
            score_phase<D, NW, BN, false>(kstage(kt), koff, qreg, S, k0, nsub, my_lim, lane);
            softmax_pv_phase<D, NW, BN, false>(vstage(kt), voff, S, O, m, lsum, sc, nsub, lane);
        }
        wait_tile(kt + 1);
        __syncthreads();
    }
    __syncthreads();   // a wave whose tiles were all full ones comes straight from reads of the ring the staging overlaps
    store_rows<D, NW, BN>(J, O, m, lsum, sc, smem, w, lane, row0, has_rows);
}

// Repetition rows when the memory zone fits one tile: t memory keys plus the row's own key
// (Eq. 1 row 3, Eq. 9).  Repetition rows are nearly half of all rows and almost pure HBM traffic
// (q, k, v in, out written, a few dozen keys of math), so everything the block reads is
// requested up front -- ONE memory round trip -- and every request covers whole 1 KB runs:
// the queries and the memory-zone tile go straight to LDS, the rows' own K and V go to
// registers in the layout of the row-wise store (lane = 16-byte piece of a row).  The own key's
// score is a dot product in that layout (q read back from LDS the same way) summed over the
// lanes of a row; its V term is added when the rows leave through an fp32 staging area, so the
// output is rounded once.
template <int D, int NW, int BN>
__device__ __forceinline__ void rep_job(const FlashJob& J, float sc, bf16_t* smem) {
    using C = Cfg<D, NW, BN>;
    constexpr int NR = 32 / C::RPI;             // wave-wide row-layout accesses that cover 32 rows
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 5, l32 = lane & 31;
    bf16_t* Ks = smem;                          // LDS: the memory-zone tile (K, V), then the queries of every wave
    bf16_t* Vt = smem + C::KBUF;
    const int nkeys = J.n1;                     // <= BN
    const int row0 = 32 * w;
    const bool has_rows = row0 < J.q_rows;
    const int rl = lane / C::CPR, pc = lane % C::CPR;   // row-layout role: row rl of each group of RPI rows, piece pc

    bf16_t* Qs = smem + C::KBUF + C::VBUF + w * 32 * D;
    load_queries_async<D, NW, BN>(J, row0, lane, Qs);
    load_tile_async<D, NW, BN>(J, 0, nkeys, w, lane, Ks, Vt);
    u32x4 kc[NR], vc[NR];
#pragma unroll
    for (int i = 0; i < NR; ++i) {
        const long src = (long)min(row0 + i * C::RPI + rl, J.q_rows - 1) * D + pc * 8;
        kc[i] = *reinterpret_cast<const u32x4*>(J.k_self + src);
        vc[i] = *reinterpret_cast<const u32x4*>(J.v_self + src);
    }
    __builtin_amdgcn_sched_barrier(0);   // all requests are out before anything waits
    int koff[C::KSTEPS], voff[C::DT];
#pragma unroll
    for (int ks = 0; ks < C::KSTEPS; ++ks) koff[ks] = l32 * D + (((2 * ks + g) ^ (l32 % C::CPR)) * 8);
    {
        const int i = lane & 15, q = i >> 2;
#pragma unroll
        for (int dt = 0; dt < C::DT; ++dt)
            voff[dt] = (4 * g + q) * D + (4 * (dt ^ (q % (C::CPR / 4))) + 2 * ((lane >> 4) & 1) + ((i & 3) >> 1)) * 8 +
                       4 * (i & 1);
    }
    f32x16 O[C::DT];
    float m = -INFINITY, lsum = 0.f;
#pragma unroll
    for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) O[dt][i] = 0.f;

    wait_direct_loads();
    __syncthreads();
    float inv = 0.f;
    if (has_rows) {
        bf16x8 qreg[C::KSTEPS];
#pragma unroll
        for (int ks = 0; ks < C::KSTEPS; ++ks) qreg[ks] = *reinterpret_cast<const bf16x8*>(Qs + koff[ks]);
        // the own key's score: q . k in the row layout, summed over the lanes of a row
        float ss[NR];
#pragma unroll
        for (int i = 0; i < NR; ++i) {
            const int r = i * C::RPI + rl;
            const u32x4 qq = *reinterpret_cast<const u32x4*>(Qs + r * D + ((pc ^ (r % C::CPR)) * 8));
            const uint32_t k0 = kc[i].x, k1 = kc[i].y, k2 = kc[i].z, k3 = kc[i].w;
            const uint32_t q0 = qq.x, q1 = qq.y, q2 = qq.z, q3 = qq.w;
            float a = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q0), __builtin_bit_cast(bf16x2, k0), 0.f, false);
            a = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q1), __builtin_bit_cast(bf16x2, k1), a, false);
            a = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q2), __builtin_bit_cast(bf16x2, k2), a, false);
            a = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q3), __builtin_bit_cast(bf16x2, k3), a, false);
            ss[i] = row_sum<C::CPR>(a);
        }
        // hand each row's score to the lanes that own the row in the accumulator layout (through the
        // wave's own query area, which has been read by now)
        float* xs = reinterpret_cast<float*>(Qs);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        if (pc == 0) {
#pragma unroll
            for (int i = 0; i < NR; ++i) xs[i * C::RPI + rl] = ss[i];
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        const float sself = xs[l32];

        const int my_lim = nkeys - 1;
        const int nsub = min(C::NSUB, (nkeys + 31) >> 5);
        f32x16 S[C::NSUB];
        score_phase<D, NW, BN, false>(Ks, koff, qreg, S, 0, nsub, my_lim, lane);
        softmax_pv_phase<D, NW, BN, false>(Vt, voff, S, O, m, lsum, sc, nsub, lane);
        // one more key: the row itself
        const float mx = fmaxf(m, sself);
        const float alpha = __builtin_amdgcn_exp2f((m - mx) * sc);
        const float p = __builtin_amdgcn_exp2f((sself - mx) * sc);
        lsum = lsum * alpha + (g == 0 ? p : 0.f);
        m = mx;
        const float ltot = pair_sum(lsum);
        inv = 1.f / ltot;
        const float oscale = alpha * inv;
#pragma unroll
        for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
            for (int i = 0; i < 16; ++i) O[dt][i] *= oscale;
        if (J.lse != nullptr && g == 0 && row0 + l32 < J.q_rows)
            J.lse[row0 + l32] = (mx * sc + __builtin_amdgcn_logf(ltot)) * LN2;
        inv *= p;   // weight of the row's own V in the output
    }
    __syncthreads();   // every wave is done with the tile and the queries before the staging areas overwrite them
    if (has_rows) {
        float* Of = reinterpret_cast<float*>(smem) + w * (32 * C::FSTR + 32);
        float* wf = Of + 32 * C::FSTR;
#pragma unroll
        for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                float4 x;
                x.x = O[dt][4 * i4 + 0]; x.y = O[dt][4 * i4 + 1]; x.z = O[dt][4 * i4 + 2]; x.w = O[dt][4 * i4 + 3];
                *reinterpret_cast<float4*>(Of + l32 * C::FSTR + 32 * dt + 8 * i4 + 4 * g) = x;
            }
        if (g == 0) wf[l32] = inv;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
        for (int i = 0; i < NR; ++i) {
            const int r = i * C::RPI + rl;
            const float4 a = *reinterpret_cast<const float4*>(Of + r * C::FSTR + pc * 8);
            const float4 b = *reinterpret_cast<const float4*>(Of + r * C::FSTR + pc * 8 + 4);
            const float wv = wf[r];
            const uint32_t v0 = vc[i].x, v1 = vc[i].y, v2 = vc[i].z, v3 = vc[i].w;
            uint4 o;
            o.x = pack_bf16(a.x + wv * bf16_lo(v0), a.y + wv * bf16_hi(v0));
            o.y = pack_bf16(a.z + wv * bf16_lo(v1), a.w + wv * bf16_hi(v1));
            o.z = pack_bf16(b.x + wv * bf16_lo(v2), b.y + wv * bf16_hi(v2));
            o.w = pack_bf16(b.z + wv * bf16_lo(v3), b.w + wv * bf16_hi(v3));
            if (row0 + r < J.q_rows) *reinterpret_cast<uint4*>(J.out + (long)(row0 + r) * D + pc * 8) = o;
        }
    }
}

// ---- mask pass -------------------------------------------------------------------------------
struct MaskParams {
    const bf16_t *q, *k, *v;
    bf16_t* out;
    float* lse;
    MaskSchedule sched;
    unsigned slab_magic;  // floor(2^32 / t) + 1
    float sc;             // scale * log2(e)
};

// PIPE: reading and memory rows take the pipelined job (long key lists), repetition rows the single-trip job.
template <int D, int NW, int BN, bool PIPE>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(2))) void mask_attn_kernel(
    MaskParams P) {
    extern __shared__ __align__(16) bf16_t smem[];
    const MaskSchedule& sch = P.sched;
    const MaskJob mj = sch.decode(blockIdx.x);
    const long seq = (long)mj.bh * sch.n * sch.s;   // first row of this (b,h)
    const long chunk = seq + (long)mj.y * sch.s;    // first row of the chunk
    FlashJob J;
    J.k0 = J.k1 = J.k2 = P.k;
    J.v0 = J.v1 = J.v2 = P.v;
    J.n0 = J.n1 = J.n2 = 0;
    J.slab = 1; J.slab_magic = 0; J.slab_stride = 0;
    J.causal_base = NO_CAUSAL;
    J.k_self = J.v_self = nullptr;
    J.rows_grouped = (sch.t % (64 / (D / 8))) == 0;
    J.q_rows = mj.rows;
    long qrow;
    if (mj.zone == ZONE_READ) {
        qrow = chunk + mj.o0;
        J.k0 = P.k + (seq + sch.R) * D; J.v0 = P.v + (seq + sch.R) * D;   // memory zone of chunk 0
        J.n0 = mj.y * sch.t; J.slab = sch.t; J.slab_magic = P.slab_magic; J.slab_stride = (long)sch.s * D;
        J.k1 = P.k + chunk * D; J.v1 = P.v + chunk * D;
        J.n1 = mj.o0 + mj.rows;
        J.causal_base = mj.y * sch.t + mj.o0;
    } else if (mj.zone == ZONE_MEM) {
        qrow = chunk + sch.R + mj.o0;
        J.k1 = P.k + chunk * D; J.v1 = P.v + chunk * D;
        J.n1 = sch.R + sch.t;
    } else {
        qrow = chunk + sch.R + sch.t + mj.o0;
        J.k1 = P.k + (chunk + sch.R) * D; J.v1 = P.v + (chunk + sch.R) * D;
        J.n1 = sch.t;
        J.k_self = P.k + qrow * D; J.v_self = P.v + qrow * D;
    }
    J.q = P.q + qrow * D;
    J.out = P.out + qrow * D;
    J.lse = P.lse ? P.lse + qrow : nullptr;
    if (mj.zone == ZONE_REP && sch.t <= BN) {
        rep_job<D, NW, BN>(J, P.sc, smem);
    } else if constexpr (PIPE) {
        static_assert(BN == 64, "the pipelined job walks tiles of 64 keys");
        if constexpr (NW <= 4) {
            if (mj.zone == ZONE_REP) { flash_job<D, NW, BN>(J, P.sc, smem); return; }
        }
        // (with eight waves the host only picks this kernel when the memory zone fits one tile: no such rows here)
        flash_job_pipe<D, NW, (NW > 4 ? 4 : 2)>(J, P.sc, smem);
    } else {
        flash_job<D, NW, BN>(J, P.sc, smem);
    }
}

// ---- compression pass ----------------------------------------------------------------------------
struct CompressParams {
    const bf16_t *q_mem, *k_mem, *v_mem, *k_read, *v_read;
    bf16_t *k_cache, *v_cache, *out;
    int t, R, nblk;         // nblk = row blocks per (b,h)
    long cache_row0;        // n_mem_chunks * t
    long cache_rows;        // mem_capacity
    float sc;
};

// ROPE: q_mem and k_mem arrive unrotated.  A prologue turns the t <m> keys by their position ids and writes them
// where they belong anyway -- the cache rows of the splice -- and turns the block's queries into its rows of
// `out` (free until the results are stored); after a device-scope fence and a barrier the block reads both back
// like any other rows.  Blocks of one (b,h) write the same key bytes.
struct NoRopeArg {};
template <int D, int NW, int BN, bool ROPE>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(2))) void compress_kernel(
    CompressParams P, std::conditional_t<ROPE, RopeTable, NoRopeArg> RT) {
    extern __shared__ __align__(16) bf16_t smem[];
    constexpr int BM = 32 * NW;
    constexpr int CPR = D / 8;
    const int bh = blockIdx.x / P.nblk, blk = blockIdx.x % P.nblk;
    const int o0 = blk * BM;
    FlashJob J;
    J.k0 = J.k1 = P.k_read; J.v0 = J.v1 = P.v_read; J.n0 = 0; J.slab = 1; J.slab_magic = 0; J.slab_stride = 0;
    J.k1 = P.k_read + (long)bh * P.R * D; J.v1 = P.v_read + (long)bh * P.R * D; J.n1 = P.R;
    J.k2 = P.k_mem + (long)bh * P.t * D;  J.v2 = P.v_mem + (long)bh * P.t * D;  J.n2 = P.t;
    J.causal_base = NO_CAUSAL;
    J.k_self = J.v_self = nullptr;
    J.rows_grouped = (P.t % (64 / (D / 8))) == 0;
    J.q_rows = min(BM, P.t - o0);
    J.q = P.q_mem + ((long)bh * P.t + o0) * D;
    J.out = P.out + ((long)bh * P.t + o0) * D;
    J.lse = nullptr;
    bf16_t* kd = P.k_cache + ((long)bh * P.cache_rows + P.cache_row0) * D;
    bf16_t* vd = P.v_cache + ((long)bh * P.cache_rows + P.cache_row0) * D;
    if constexpr (ROPE) {
        for (int i = threadIdx.x; i < P.t * CPR; i += 64 * NW) {
            const int r = i / CPR, pc = i % CPR;
            const u32x4 x = rope::load_rotated_piece<D>(J.k2 + (long)r * D, pc, RT.pos_first + r * RT.pos_stride, RT);
            *reinterpret_cast<u32x4*>(kd + (long)r * D + pc * 8) = x;
        }
        for (int i = threadIdx.x; i < J.q_rows * CPR; i += 64 * NW) {
            const int r = i / CPR, pc = i % CPR;
            const u32x4 x = rope::load_rotated_piece<D>(J.q + (long)r * D, pc, RT.pos_first + (o0 + r) * RT.pos_stride, RT);
            *reinterpret_cast<u32x4*>(J.out + (long)r * D + pc * 8) = x;
        }
        __threadfence();
        __syncthreads();
        J.k2 = kd;
        J.q = J.out;
    }
    flash_job<D, NW, BN>(J, P.sc, smem);
    // splice: the t new memory KVs join the compressed cache (Sec. 3.1 step 3)
    if (blk == 0) {
        const int pieces = P.t * D / 8;
        const uint4* ks = reinterpret_cast<const uint4*>(J.k2);
        const uint4* vs = reinterpret_cast<const uint4*>(J.v2);
        uint4* kd4 = reinterpret_cast<uint4*>(kd);
        uint4* vd4 = reinterpret_cast<uint4*>(vd);
        for (int i = threadIdx.x; i < pieces; i += 64 * NW) {
            if (!ROPE) kd4[i] = ks[i];
            vd4[i] = vs[i];
        }
    }
}

// ---- several new tokens against the cache (Appendix A, more than one input token) ----------------------
struct PrefillParams {
    const bf16_t *q, *k_new, *v_new, *k_cache, *v_cache;
    bf16_t *k_read, *v_read, *out;
    float* lse;
    int n_new, R, nblk;     // nblk = row blocks per (b,h)
    int n_mem_keys, read_fill;
    long cache_rows;        // mem_capacity
    float sc;
};

// Keys of a block of new tokens: the memory cache (contiguous), the live reading-zone rows, then the
// new tokens themselves up to the block's last row, read from k_new/v_new and cut by the causal
// diagonal -- a reading-zone block of the mask pass whose earlier memory zones sit in one piece.
template <int D, int NW, int BN, int KS, int NS>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(2))) void prefill_kernel(PrefillParams P) {
    extern __shared__ __align__(16) bf16_t smem[];
    constexpr int BM = 32 * NW / KS;
    const int bh = blockIdx.x / P.nblk;
    const int blk = P.nblk - 1 - blockIdx.x % P.nblk;   // last rows (most keys) first
    const int o0 = blk * BM;
    const int rows = min(BM, P.n_new - o0);
    const long new0 = (long)bh * P.n_new;
    FlashJob J;
    J.k0 = P.k_cache + (long)bh * P.cache_rows * D; J.v0 = P.v_cache + (long)bh * P.cache_rows * D;
    J.n0 = P.n_mem_keys; J.slab = 1; J.slab_magic = 0; J.slab_stride = D;
    J.k1 = P.k_read + (long)bh * P.R * D; J.v1 = P.v_read + (long)bh * P.R * D; J.n1 = P.read_fill;
    J.k2 = P.k_new + new0 * D; J.v2 = P.v_new + new0 * D; J.n2 = o0 + rows;
    J.causal_base = P.n_mem_keys + P.read_fill + o0;
    J.k_self = J.v_self = nullptr;
    J.rows_grouped = (P.n_mem_keys % (64 / (D / 8))) == 0 && (P.n_mem_keys > 0 || P.read_fill % (64 / (D / 8)) == 0);
    J.q_rows = rows;
    J.q = P.q + (new0 + o0) * D;
    J.out = P.out + (new0 + o0) * D;
    J.lse = P.lse ? P.lse + new0 + o0 : nullptr;
    flash_job<D, NW, BN, KS, NS>(J, P.sc, smem);
    // the new tokens join the reading zone (rows no block of this launch reads)
    if (blk == 0) {
        const int pieces = P.n_new * D / 8;
        const uint4* ks = reinterpret_cast<const uint4*>(J.k2);
        const uint4* vs = reinterpret_cast<const uint4*>(J.v2);
        uint4* kd = reinterpret_cast<uint4*>(P.k_read + ((long)bh * P.R + P.read_fill) * D);
        uint4* vd = reinterpret_cast<uint4*>(P.v_read + ((long)bh * P.R + P.read_fill) * D);
        for (int i = threadIdx.x; i < pieces; i += 64 * NW) { kd[i] = ks[i]; vd[i] = vs[i]; }
    }
}

// The dynamic-LDS limit of a kernel is raised once per kernel and device, not on every enqueue.
inline bool lds_limit_is_set(const void* kernel, int smem_bytes) {
    static std::mutex mu;
    static std::set<std::pair<const void*, int>> done;   // (kernel, device)
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return false;
    std::lock_guard<std::mutex> lock(mu);
    if (done.count({kernel, dev})) return true;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, smem_bytes) != hipSuccess) return false;
    done.insert({kernel, dev});
    return true;
}

template <typename K, typename... Args>
int launch(K kernel, long long grid, int threads, int smem_bytes, hipStream_t st, const Args&... args) {
    if (grid <= 0) return LOMA_OK;
    if (grid > 0x7fffffffLL) return LOMA_ERR_UNSUPPORTED;
    if (!lds_limit_is_set(reinterpret_cast<const void*>(kernel), smem_bytes)) return LOMA_ERR_LAUNCH;
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(threads), smem_bytes, st, args...);
    return hipGetLastError() == hipSuccess ? LOMA_OK : LOMA_ERR_LAUNCH;
}

template <int D>
int launch_mask_d(const MaskParams& P, int bm, hipStream_t st) {
    const long long grid = P.sched.size();
    constexpr int PIPE4 = PipeCfg<D, 4, 2>::SMEM_BYTES > Cfg<D, 4, 64>::REP_BYTES ? PipeCfg<D, 4, 2>::SMEM_BYTES : Cfg<D, 4, 64>::REP_BYTES;
    if (bm == 128) return launch(mask_attn_kernel<D, 4, 64, true>, grid, 256, PIPE4, st, P);
    if (bm == 64) return launch(mask_attn_kernel<D, 2, 32, false>, grid, 128, Cfg<D, 2, 32>::SMEM_BYTES, st, P);
    return launch(mask_attn_kernel<D, 1, 32, false>, grid, 64, Cfg<D, 1, 32>::SMEM_BYTES, st, P);
}

template <int D, bool ROPE>
int launch_compress_d(CompressParams& P, int nbh, hipStream_t st, std::conditional_t<ROPE, RopeTable, NoRopeArg> RT) {
    if (P.t > 64) {
        P.nblk = (P.t + 127) / 128;
        return launch(compress_kernel<D, 4, 64, ROPE>, (long long)nbh * P.nblk, 256, Cfg<D, 4, 64>::SMEM_BYTES, st, P, RT);
    }
    if (P.t > 32) {
        P.nblk = 1;
        return launch(compress_kernel<D, 2, 32, ROPE>, nbh, 128, Cfg<D, 2, 32>::SMEM_BYTES, st, P, RT);
    }
    P.nblk = 1;
    return launch(compress_kernel<D, 1, 32, ROPE>, nbh, 64, Cfg<D, 1, 32>::SMEM_BYTES, st, P, RT);
}

template <int D>
int launch_prefill_d(PrefillParams& P, int nbh, hipStream_t st) {
    // Few workgroups (a handful of sequences): one workgroup walks the whole cache of its (b,h) alone, so what
    // counts is how many bytes it keeps in flight and how few dependent steps it takes: a ring of four stages
    // (three tiles requested ahead) and the keys of every tile split over two groups of waves.
    // Many workgroups: the plain variants, more of which fit a CU.
    const bool few = (long long)nbh * ((P.n_new + 63) / 64) < 1024;
    constexpr int RING4 = 2 * Cfg<D, 4, 64>::RING_BYTES;   // 4 stages of 64 keys
    if (few && P.n_new <= 32) {
        P.nblk = 1;
        return launch(prefill_kernel<D, 2, 64, 2, 4>, nbh, 128, RING4, st, P);
    }
    if (few) {
        P.nblk = (P.n_new + 63) / 64;
        return launch(prefill_kernel<D, 4, 64, 2, 4>, (long long)nbh * P.nblk, 256, RING4, st, P);
    }
    if (P.n_new > 64) {
        P.nblk = (P.n_new + 127) / 128;
        return launch(prefill_kernel<D, 4, 64, 1, 2>, (long long)nbh * P.nblk, 256, Cfg<D, 4, 64>::SMEM_BYTES, st, P);
    }
    P.nblk = 1;
    if (P.n_new > 32) return launch(prefill_kernel<D, 2, 64, 1, 2>, nbh, 128, Cfg<D, 2, 64>::SMEM_BYTES, st, P);
    return launch(prefill_kernel<D, 1, 32, 1, 2>, nbh, 64, Cfg<D, 1, 32>::SMEM_BYTES, st, P);
}

}  // namespace

int launch_prefill_mfma(const void* q, const void* k_new, const void* v_new,
                        const void* k_memcache, const void* v_memcache, void* k_read, void* v_read,
                        void* out, float* lse, int nbh, int D, int R, int n_mem_keys, int mem_capacity,
                        int read_fill, int n_new, float scale, hipStream_t st) {
    PrefillParams P;
    P.q = static_cast<const bf16_t*>(q); P.k_new = static_cast<const bf16_t*>(k_new);
    P.v_new = static_cast<const bf16_t*>(v_new);
    P.k_cache = static_cast<const bf16_t*>(k_memcache); P.v_cache = static_cast<const bf16_t*>(v_memcache);
    P.k_read = static_cast<bf16_t*>(k_read); P.v_read = static_cast<bf16_t*>(v_read);
    P.out = static_cast<bf16_t*>(out); P.lse = lse;
    P.n_new = n_new; P.R = R; P.nblk = 1; P.n_mem_keys = n_mem_keys; P.read_fill = read_fill;
    P.cache_rows = mem_capacity;
    P.sc = scale * LOG2E;
    return D == 128 ? launch_prefill_d<128>(P, nbh, st) : launch_prefill_d<64>(P, nbh, st);
}

int launch_mask_attn_mfma(const void* q, const void* k, const void* v, void* out, float* lse,
                          int nbh, int D, const Geometry& g, float scale, hipStream_t st) {
    MaskParams P;
    P.q = static_cast<const bf16_t*>(q); P.k = static_cast<const bf16_t*>(k); P.v = static_cast<const bf16_t*>(v);
    P.out = static_cast<bf16_t*>(out); P.lse = lse;
    const int bm = mask_block_rows(g.R, g.t);
    P.sched = MaskSchedule::make(nbh, g.t, g.c, g.n, bm);
    P.slab_magic = g.t > 1 ? (unsigned)((1ULL << 32) / (unsigned)g.t) + 1u : 0u;
    P.sc = scale * LOG2E;
    return D == 128 ? launch_mask_d<128>(P, bm, st) : launch_mask_d<64>(P, bm, st);
}

int launch_compress_mfma(const void* q_mem, const void* k_mem, const void* v_mem,
                         const void* k_read, const void* v_read, void* k_memcache, void* v_memcache,
                         void* out, int nbh, int D, int t, int c, int n_mem_chunks, int mem_capacity,
                         float scale, hipStream_t st, const RopeTable* rope) {
    CompressParams P;
    P.q_mem = static_cast<const bf16_t*>(q_mem); P.k_mem = static_cast<const bf16_t*>(k_mem);
    P.v_mem = static_cast<const bf16_t*>(v_mem); P.k_read = static_cast<const bf16_t*>(k_read);
    P.v_read = static_cast<const bf16_t*>(v_read);
    P.k_cache = static_cast<bf16_t*>(k_memcache); P.v_cache = static_cast<bf16_t*>(v_memcache);
    P.out = static_cast<bf16_t*>(out);
    P.t = t; P.R = t * c; P.nblk = 1;
    P.cache_row0 = (long)n_mem_chunks * t; P.cache_rows = mem_capacity;
    P.sc = scale * LOG2E;
    if (rope != nullptr)
        return D == 128 ? launch_compress_d<128, true>(P, nbh, st, *rope) : launch_compress_d<64, true>(P, nbh, st, *rope);
    return D == 128 ? launch_compress_d<128, false>(P, nbh, st, {}) : launch_compress_d<64, false>(P, nbh, st, {});
}

}  // namespace loma
