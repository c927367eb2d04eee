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
#pragma once
#include <type_traits>

#include "loma_mfma.h"

namespace loma {

struct BwdTensors {   // all at the first row of the (b,h) sequence
    const mfma::bf16_t *q, *k, *v, *dout, *out;
    const float* lse;
    float *nl, *delta;   // per row: -lse * log2(e) and dout . out; written by the dQ pass (every row is an owner row
                         // of exactly one of its blocks), read by the dK/dV pass
    mfma::bf16_t *dq, *dk, *dv;
};

struct BwdParams {
    BwdTensors T;       // at sequence 0
    int nbh, n, t, R, s;
    int bm;             // owner rows per workgroup
    int split;          // workgroups that share the stream of one block of memory keys in the dK/dV pass (1 or 2)
    float* partials;    // split > 1: fp32 [nbh][split][2 (dK, dV)][n*t][head_dim]
    float scale, sc;    // scale, scale * log2(e)
};

// the two passes, each in a translation unit of its own
int launch_bwd_dq_pass(const BwdParams& P, int D, hipStream_t st);
int launch_bwd_dkv_pass(const BwdParams& P, int D, hipStream_t st);

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

// What a tile of 32 consecutive list entries from j0 on looks like: the row of entry j0, its range and slab,
// and whether the 32 entries exist and are 32 consecutive rows (one range, one slab).  All wave-uniform.
struct TileInfo {
    int row, slab_index;
    bool in0, contig;
};
__device__ __forceinline__ TileInfo tile_info(const RowList L, int nstr, int j0) {
    TileInfo t;
    const int j1 = j0 + 31;
    t.in0 = j0 < L.n0;
    const int jj = t.in0 ? j0 : j0 - L.n0;
    const int slab = t.in0 ? L.slab0 : L.slab1;
    const unsigned magic = t.in0 ? L.magic0 : L.magic1;
    const int a0 = div_slab(jj, slab, magic), a1 = div_slab(jj + 31, slab, magic);
    t.slab_index = a0;
    t.row = (t.in0 ? L.base0 : L.base1) + a0 * (t.in0 ? L.stride0 : L.stride1) + (jj - a0 * slab);
    t.contig = j1 < nstr && (j1 < L.n0) == t.in0 && a0 == a1;
    return t;
}

struct BwdJob {
    RowList own;   // owner rows: entry `ooff + r` for block row r (range 0 only)
    int ooff, orows;
    RowList str;   // streamed rows, nstr of them
    int nstr;
    int vis;       // which rule decides whether streamed row j and owner row r interact
    int cb;        // VIS_CAUSAL: j <= cb + r.   VIS_FROM_ROW: j >= r.
    // VIS_MEMKEYS: owner r is memory key ooff + r of chunk yk = (ooff + r) / t; streamed row j of range 0
    // is a reading row of chunk z0 - slab index (the farthest chunk comes first; visible iff yk < that
    // chunk), of range 1 a memory or repetition row of chunk z1 + slab index (visible iff yk == that chunk)
    int t, z0, z1;
    unsigned magic_t;
    int pipe0, pipe1;   // dK/dV pass: tiles [pipe0, pipe1) of the stream hold only visible pairs, whichever the owner row
    int pipe_end;       // ... and tiles [0, pipe_end) are whole tiles of 32 consecutive rows (pipe1 <= pipe_end)
    int rep;       // dQ pass on repetition rows: add the rows' own-key terms when they leave
    // dK/dV pass of a block whose stream is shared out over several workgroups: fp32 partial sums, row
    // `ooff + r` of each (nullptr: the block is whole and writes dk, dv itself)
    float *part_k, *part_v;
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
    static constexpr int FSTR = D + 4;       // row stride (floats) of the fp32 staging area rows leave through
    static constexpr int WAVE_STAGING_BYTES = 32 * FSTR * 4;
    static constexpr int smem_bytes(int nw, int ns) {
        return ns * STAGE_BYTES > nw * WAVE_STAGING_BYTES ? ns * STAGE_BYTES : nw * WAVE_STAGING_BYTES;
    }
};
// Tile stages and how far the loads run ahead of the arithmetic.  The dQ pass reads one tile at a time and
// reuses a stage as soon as the barrier after its tile has passed (AHEAD = NS - 1); with fewer than four waves it
// walks short lists and would rather fit more workgroups on a CU.  The dK/dV pass runs one workgroup per SIMD set
// anyway (its registers allow no more) and, in its pipelined loop, reads three consecutive tiles in one
// iteration: a stage is reused two barriers after its tile's first use (AHEAD = NS - 2).
template <int PASS, int NW>
struct Stages {
    static constexpr int NS = PASS == 1 ? (NW == 4 ? 6 : 4) : (NW == 4 ? 4 : 2);
    static constexpr int AHEAD = PASS == 1 ? NS - 2 : NS - 1;
};

// position of 16-byte piece c of tile row r: c ^ swz(r).  16 consecutive rows give 16 different values
// (plain reads: one piece of 16 rows), and the four rows r..r+3 of a transposing read differ in the two
// high bits while rows 4 apart differ in the two low bits.
template <int CPR>
__device__ __forceinline__ int swz(int r) { return (4 * (r & 3) + ((r >> 2) & 3)) % CPR; }

// Wave-wide direct loads HBM -> LDS.  The LDS destination is a byte address in a scalar register (taken
// once from the shared-memory pointer: converting a pointer at every load costs a null check each time);
// lane l's data lands at lds_addr + l * (bytes per lane).
__device__ __forceinline__ unsigned lds_address(const void* p) {
    return __builtin_amdgcn_readfirstlane((unsigned)(size_t)(__attribute__((address_space(3))) const char*)p);
}
__device__ __forceinline__ void direct_load_4B(const float* src, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off" ::"s"(lds_addr), "v"(src) : "memory", "m0");
}
__device__ __forceinline__ void direct_load_16B_to(const bf16_t* src, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(src) : "memory", "m0");
}
// ... with the row address in scalar registers and a per-lane byte offset
__device__ __forceinline__ void direct_load_16B_at(const bf16_t* sbase, unsigned voff, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(voff), "s"(sbase)
                 : "memory", "m0");
}

// per-lane constants of the tile loads
template <int D, int NW>
struct LoadLane {
    static constexpr int IPW = BCfg<D>::BN / BCfg<D>::RPI / NW;   // wave-wide loads per tensor and tile
    static_assert(IPW >= 1, "tile rows split over the waves");
    unsigned off[IPW];      // byte offset of the lane's piece from the tile's first row, when the rows are consecutive
    const float* ld;        // lanes 0..31: nl of tile row `lane`; lanes 32..63: delta of tile row `lane - 32` (tile at row 0)
};

// Direct HBM -> LDS copy of streamed tile [j0, j0 + 32): X and Y rows and, for the dK/dV pass, the rows' nl
// and delta.  A tile of 32 consecutive rows (nearly all are) is addressed from a scalar base, no vector
// arithmetic; otherwise every lane looks its row up (entries past the list replay its last row; the
// arithmetic masks them).
template <int D, int NW, int PASS>
__device__ __forceinline__ void request_tile(const BwdJob& J, const bf16_t* X, const bf16_t* Y, const LoadLane<D, NW>& LL,
                                             int j0, int w, int lane, unsigned stage_addr) {
    using C = BCfg<D>;
    constexpr int IPW = LoadLane<D, NW>::IPW;
    const unsigned xs = stage_addr, ys = stage_addr + 2 * C::TILE, ls = stage_addr + 4 * C::TILE;   // LDS byte addresses
    const TileInfo ti = tile_info(J.str, J.nstr, j0);
    if (ti.contig) {
        const bf16_t* xb = uniform_ptr(X + (long)ti.row * D);
        const bf16_t* yb = uniform_ptr(Y + (long)ti.row * D);
#pragma unroll
        for (int i = 0; i < IPW; ++i) {
            const unsigned rb = 2u * ((w * IPW + i) * C::RPI * D);   // wave-uniform
            direct_load_16B_at(xb, LL.off[i], xs + rb);
            direct_load_16B_at(yb, LL.off[i], ys + rb);
        }
        if constexpr (PASS == PASS_DKV) direct_load_4B(LL.ld + ti.row, ls);
        return;
    }
    const int p = lane % C::CPR;
#pragma unroll
    for (int i = 0; i < IPW; ++i) {
        const int rbase = (w * IPW + i) * C::RPI;
        const int r = rbase + lane / C::CPR;
        const long row = list_row(J.str, min(j0 + r, J.nstr - 1));
        const int c = p ^ swz<C::CPR>(r);
        direct_load_16B_to(X + row * D + c * 8, xs + 2u * (rbase * D));
        direct_load_16B_to(Y + row * D + c * 8, ys + 2u * (rbase * D));
    }
    if constexpr (PASS == PASS_DKV) {
        // every wave writes the same 64 values (keeps the waves' load counts equal)
        const long row = list_row(J.str, min(j0 + (lane & 31), J.nstr - 1));
        direct_load_4B(LL.ld + (row - (lane & 31)), ls);   // LL.ld already points at the lane's row of a tile at row 0
    }
}

// The dK/dV pass holds 2 x 64 accumulator registers next to 64 operand registers: more than the 256
// ordinary registers of a lane, and as C++ values the compiler copies them between the register files
// on every tile.  They therefore live in the accumulation registers a0..a127 BY NAME for the whole
// kernel: dK^T in a[0:63], dV^T in a[64:127] (16 registers per 32 head-dim columns).  Every statement
// below names them as clobbered, so the compiler keeps nothing of its own there across them (and, with
// fewer than 256 ordinary registers in use, has no reason to touch them in between).  The
// instructions are opaque to the compiler's hazard bookkeeping: consecutive MFMAs name different
// accumulators, and settle_acc() comes before the first read of one.
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

// staged rows -> fp32 rows `J.ooff + row` of a partial-sum buffer
template <int D>
__device__ __forceinline__ void store_staged_partial(const float* Of, float* dst, const BwdJob& J, int row0, int lane) {
    using C = BCfg<D>;
    const int rl = lane / C::CPR, pc = lane % C::CPR;
#pragma unroll
    for (int i = 0; i < 32 / C::RPI; ++i) {
        const int r = i * C::RPI + rl;
        if (row0 + r < J.orows) {
            float* at = dst + (long)(J.ooff + row0 + r) * D + pc * 8;
            *reinterpret_cast<float4*>(at) = *reinterpret_cast<const float4*>(Of + r * C::FSTR + pc * 8);
            *reinterpret_cast<float4*>(at + 4) = *reinterpret_cast<const float4*>(Of + r * C::FSTR + pc * 8 + 4);
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
    // Four row groups at a time: all their loads first, then the arithmetic and the stores.  (Written as one loop
    // the stores of a group, which may alias the next group's loads for all the compiler knows, keep every group's
    // loads behind them: eight dependent memory round trips per block.)
    constexpr int NG = 32 / C::RPI, GB = NG < 4 ? NG : 4;
#pragma unroll
    for (int i0 = 0; i0 < NG; i0 += GB) {
        u32x4 qq[GB], kk[GB], vv[GB], gg[GB], oo[GB];
        float ls[GB];
        long at[GB];
        bool live[GB];
#pragma unroll
        for (int b = 0; b < GB; ++b) {
            const int r = (i0 + b) * C::RPI + rl;
            live[b] = row0 + r < J.orows;
            const long row = list_row(J.own, J.ooff + min(row0 + r, J.orows - 1));   // rows past the block replay its last row
            at[b] = row * D + pc * 8;
            qq[b] = *reinterpret_cast<const u32x4*>(T.q + at[b]);
            kk[b] = *reinterpret_cast<const u32x4*>(T.k + at[b]);
            vv[b] = *reinterpret_cast<const u32x4*>(T.v + at[b]);
            gg[b] = *reinterpret_cast<const u32x4*>(T.dout + at[b]);
            oo[b] = *reinterpret_cast<const u32x4*>(T.out + at[b]);
            ls[b] = T.lse[row];
        }
#pragma unroll
        for (int b = 0; b < GB; ++b) {
            const int r = (i0 + b) * C::RPI + rl;
            const float s = row_sum<C::CPR>(dot8(qq[b], kk[b]));
            const float dw = row_sum<C::CPR>(dot8(gg[b], vv[b]));
            const float delta = row_sum<C::CPR>(dot8(gg[b], oo[b]));   // (formed again here: other lanes hold the prologue's copy)
            const float wgt = __builtin_amdgcn_exp2f(fmaf(s, sc, -ls[b] * LOG2E));
            const float da = wgt * (dw - delta);
            const float4 a = *reinterpret_cast<const float4*>(Of + r * C::FSTR + pc * 8);
            const float4 c = *reinterpret_cast<const float4*>(Of + r * C::FSTR + pc * 8 + 4);
            const float4 z = {0.f, 0.f, 0.f, 0.f};
            if (live[b]) {
                *reinterpret_cast<uint4*>(T.dq + at[b]) = axpb8(scale * da, kk[b], a, c);
                *reinterpret_cast<uint4*>(T.dk + at[b]) = axpb8(scale * da, qq[b], z, z);
                *reinterpret_cast<uint4*>(T.dv + at[b]) = axpb8(wgt, gg[b], z, z);
            }
        }
    }
}

// S' / dP' MFMAs of the dK/dV pass: the owner rows' operand comes from the accumulation registers (constraint "a";
// that is where the 64 registers of k and v live for the whole kernel, past a127), the result goes to ordinary
// registers.  Opaque to the compiler's hazard bookkeeping: settle_scores() comes between the last of them and the
// first read of the result unless other work of at least that length does.
__device__ __forceinline__ void mfma_owner_first(f32x16& acc, bf16x8 a, bf16x8 owner) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(acc) : "v"(a), "a"(owner));
}
__device__ __forceinline__ void mfma_owner(f32x16& acc, bf16x8 a, bf16x8 owner) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "a"(owner));
}
__device__ __forceinline__ void settle_scores() { asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 7" ::: "memory"); }

// One step of the pipelined loop over tiles whose pairs are all visible.  Three tiles are at work:
//     DO_A: S' and dP' of the tile in stage stA into (Sn, dPn)                         -- 2 KSTEPS MFMAs
//     DO_B: P and dS of the tile whose S', dP' are (Sc, dPc), packed to bf16 in pk_out  -- exponentials and vector ALU
//     DO_C: acc^T += X^T dS (and Y^T P) of the tile in stage stC, packed in pk_in      -- the other MFMAs
// cut into 2 KSTEPS slots of one MFMA of A, one of C (dQ pass: every other slot) and a sixteenth of B, with the
// LDS reads of a slot's operands two slots ahead of it.  A scheduling fence ends every slot: the matrix pipe
// runs under the vector arithmetic of ONE instruction stream (one wave per SIMD is all the registers allow).
// stB is the stage that holds B's tile (its rows' -lse log2(e) and delta, dK/dV pass).  pk[0] = P, pk[1] = dS,
// element pairs in accumulator order.  MASKED: B's tile is not fully visible; `thr` says, per lane, from which of
// the tile's rows on the lane's owner row interacts with them (P and dS of the others are zero, and so is what
// their MFMAs add: a wave none of whose rows sees the tile multiplies zeros, where the tile-by-tile path would
// wait at the barrier).
template <int D, int PASS, bool DO_A, bool DO_B, bool DO_C, bool MASKED = false>
__device__ __forceinline__ void pipe_step(const bf16_t* stA, const bf16_t* stB, const bf16_t* stC,
                                          const int (&poff)[BCfg<D>::KSTEPS], const int (&toff)[2][BCfg<D>::DT],
                                          const bf16x8 (&xo)[BCfg<D>::KSTEPS], const bf16x8 (&yo)[BCfg<D>::KSTEPS],
                                          f32x16& Sn, f32x16& dPn, const f32x16& Sc, const f32x16& dPc,
                                          uint32_t (&pk_out)[2][8], const uint32_t (&pk_in)[2][8],
                                          f32x16 (&accX)[BCfg<D>::DT], float sc, float nl_own, float dl_own, int g,
                                          int thr = 0) {
    using C = BCfg<D>;
    constexpr int NSLOT = 2 * C::KSTEPS, EPS = 16 / NSLOT, RA = 2;
    constexpr int CSTRIDE = PASS == PASS_DKV ? 1 : 2;          // a C MFMA every CSTRIDE slots (the odd ones in the dQ pass)
    constexpr int NC = NSLOT / CSTRIDE;
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    bf16x8 aop[NSLOT], cop[NC];
    float4 nlv[4], dlv[4];
    auto read_a = [&](auto jc) {
        constexpr int j = jc.value;
        aop[j] = *reinterpret_cast<const bf16x8*>(stA + ((j & 1) ? C::TILE : 0) + poff[j >> 1]);
    };
    // C MFMA c: dK/dV pass (step, dt, dK or dV) = (c / (2 DT), (c / 2) % DT, c % 2); dQ pass (step, dt) = (c / DT, c % DT)
    auto read_c = [&](auto cc) {
        constexpr int c = cc.value;
        constexpr int step = PASS == PASS_DKV ? c / (2 * C::DT) : c / C::DT;
        constexpr int dt = PASS == PASS_DKV ? (c / 2) % C::DT : c % C::DT;
        const bf16_t* base = stC + ((PASS == PASS_DKV && (c & 1)) ? C::TILE : 0) + 16 * step * D;
        const s16x4 lo = lds_read_tr(base + toff[0][dt]);
        const s16x4 hi = lds_read_tr(base + toff[1][dt]);
        cop[c] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    auto read_rows = [&](auto ac) {   // -lse log2(e) and delta of the four streamed rows of elements 4a .. 4a + 3
        constexpr int a = ac.value;
        const float4* ld = reinterpret_cast<const float4*>(stB + 2 * C::TILE);
        nlv[a] = ld[2 * a + g];
        dlv[a] = ld[8 + 2 * a + g];
    };
    // what the first slots need
    if constexpr (DO_A) static_for<0, RA>(read_a);
    if constexpr (DO_C) static_for<0, (RA + CSTRIDE - 1) / CSTRIDE>(read_c);
    if constexpr (DO_B && PASS == PASS_DKV) static_for<0, 4>([&](auto ac) { if constexpr (4 * ac.value / EPS < RA) read_rows(ac); });
    __builtin_amdgcn_sched_barrier(0);
    float p_even = 0.f, ds_even = 0.f;
    static_for<0, NSLOT>([&](auto jc) {
        constexpr int j = jc.value;
        if constexpr (DO_A && PASS == PASS_DKV) {
            if constexpr (j == 0) mfma_owner_first(Sn, aop[j], xo[0]);
            else if constexpr (j == 1) mfma_owner_first(dPn, aop[j], yo[0]);
            else if constexpr ((j & 1) == 0) mfma_owner(Sn, aop[j], xo[j >> 1]);
            else mfma_owner(dPn, aop[j], yo[j >> 1]);
        } else if constexpr (DO_A) {
            if constexpr ((j & 1) == 0) Sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop[j], xo[j >> 1], j == 0 ? zero16 : Sn, 0, 0, 0);
            else dPn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop[j], yo[j >> 1], j == 1 ? zero16 : dPn, 0, 0, 0);
        }
        if constexpr (DO_B) {
            static_for<j * EPS, (j + 1) * EPS>([&](auto ec) {
                constexpr int e = ec.value;
                float nl = nl_own, dl = dl_own;
                if constexpr (PASS == PASS_DKV) {
                    const float nl4[4] = {nlv[e / 4].x, nlv[e / 4].y, nlv[e / 4].z, nlv[e / 4].w};
                    const float dl4[4] = {dlv[e / 4].x, dlv[e / 4].y, dlv[e / 4].z, dlv[e / 4].w};
                    nl = nl4[e % 4];
                    dl = dl4[e % 4];
                }
                float pr = exp2_at(fmaf(Sc[e], sc, nl));
                // MASKED: element e is streamed row 8 (e / 4) + e % 4 (+ 4 g, folded into thr) of the tile; the lane's
                // owner row interacts with it iff that number reaches the lane's threshold
                if constexpr (MASKED) pr = (8 * (e / 4) + e % 4 >= thr) ? pr : 0.f;
                const float ds = pr * (dPc[e] - dl);
                if constexpr ((e & 1) == 0) {
                    p_even = pr;
                    ds_even = ds;
                } else {
                    pk_out[0][e >> 1] = pack_bf16_at(p_even, pr);
                    pk_out[1][e >> 1] = pack_bf16_at(ds_even, ds);
                }
            });
        }
        if constexpr (DO_C && (j % CSTRIDE) == CSTRIDE - 1) {
            constexpr int c = j / CSTRIDE;
            constexpr int step = PASS == PASS_DKV ? c / (2 * C::DT) : c / C::DT;
            constexpr int dt = PASS == PASS_DKV ? (c / 2) % C::DT : c % C::DT;
            const uint4 wp = {pk_in[0][4 * step], pk_in[0][4 * step + 1], pk_in[0][4 * step + 2], pk_in[0][4 * step + 3]};
            const uint4 wds = {pk_in[1][4 * step], pk_in[1][4 * step + 1], pk_in[1][4 * step + 2], pk_in[1][4 * step + 3]};
            if constexpr (PASS == PASS_DKV) {
                if constexpr ((c & 1) == 0) mfma_named<16 * dt>(cop[c], __builtin_bit_cast(bf16x8, wds));
                else mfma_named<64 + 16 * dt>(cop[c], __builtin_bit_cast(bf16x8, wp));
            } else {
                accX[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cop[c], __builtin_bit_cast(bf16x8, wds), accX[dt], 0, 0, 0);
            }
        }
        // reads for the slots two ahead
        if constexpr (DO_A && j + RA < NSLOT) read_a(std::integral_constant<int, j + RA>{});
        if constexpr (DO_C && ((j + RA) % CSTRIDE) == CSTRIDE - 1 && (j + RA) / CSTRIDE < NC && (j + RA) / CSTRIDE >= (RA + CSTRIDE - 1) / CSTRIDE)
            read_c(std::integral_constant<int, (j + RA) / CSTRIDE>{});
        if constexpr (DO_B && PASS == PASS_DKV)
            static_for<1, 4>([&](auto ac) { if constexpr (4 * ac.value / EPS - RA == j) read_rows(ac); });
        __builtin_amdgcn_sched_barrier(0);
    });
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

    LoadLane<D, NW> LL;
#pragma unroll
    for (int i = 0; i < LoadLane<D, NW>::IPW; ++i) {
        const int r = (w * LoadLane<D, NW>::IPW + i) * C::RPI + lane / C::CPR;
        LL.off[i] = 2u * (r * D + (((lane % C::CPR) ^ swz<C::CPR>(r)) * 8));
    }
    LL.ld = (lane < 32 ? T.nl : T.delta) + (lane & 31);

    const unsigned smem_addr = lds_address(smem);
    // the loads run AHEAD tiles ahead of the arithmetic; tile kt lives in stage kt % NS
    constexpr int NS = Stages<PASS, NW>::NS;
    constexpr int AHEAD = Stages<PASS, NW>::AHEAD;
    constexpr int LPT = 2 * (C::BN / C::RPI / NW) + (PASS == PASS_DKV ? 1 : 0);   // direct loads per wave and tile
    int next_req = 0;   // tiles [0, next_req) have been requested
    auto request_upto = [&](int last) {
        while (next_req <= last && next_req < ntiles) {
            request_tile<D, NW, PASS>(J, X, Y, LL, next_req * C::BN, w, lane, smem_addr + (next_req % NS) * C::STAGE_BYTES);
            ++next_req;
        }
    };
    // this wave's loads of tile `tile` (or of the last one, past the end) have landed; younger tiles stay in flight
    auto wait_for = [&](int tile) { wait_next_tile<LPT, AHEAD - 1>(next_req - 1 - min(tile, ntiles - 1)); };
    request_upto(AHEAD - 1);

    // owner rows as B operands: lane (row l32, half g) holds head-dim 16*ks + 8*g .. +7
    bf16x8 xo[C::KSTEPS], yo[C::KSTEPS];
#pragma unroll
    for (int ks = 0; ks < C::KSTEPS; ++ks) {
        xo[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(Xo + orow * D + 16 * ks + 8 * g));
        yo[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(Yo + orow * D + 16 * ks + 8 * g));
    }
    float nl_own = 0.f, dl_own = 0.f;
    if constexpr (PASS == PASS_DQ) {
        // delta = dout . out of the owner row (half of the head-dim in each of the lanes l and l ^ 32) and the lse in
        // the form the exp2 below wants; both also go to the workspace for the dK/dV pass
        float part = 0.f;
#pragma unroll
        for (int ks = 0; ks < C::KSTEPS; ++ks) {
            const u32x4 oo = *reinterpret_cast<const u32x4*>(T.out + orow * D + 16 * ks + 8 * g);
            part += dot8(oo, __builtin_bit_cast(u32x4, yo[ks]));
        }
        dl_own = pair_sum(part);
        nl_own = -T.lse[orow] * LOG2E;
        if (g == 0 && row0 + l32 < J.orows) {
            T.delta[orow] = dl_own;
            T.nl[orow] = nl_own;
        }
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
    f32x16 accX[C::DT];   // dQ^T (dQ pass; the dK/dV pass accumulates in named registers)
#pragma unroll
    for (int dt = 0; dt < C::DT; ++dt) accX[dt] = zero16;
    if constexpr (PASS == PASS_DKV) static_for<0, 128>([&](auto i) { zero_named<i.value>(); });

    // The first AHEAD tiles were requested before the owner rows; one wait covers everything.  It has to
    // be a full one: the compiler counts only the loads it issued itself (the owner rows), and would
    // otherwise wait for them inside the loop with counts that also drain the tiles in flight.
    wait_direct_loads();
    __syncthreads();

    // All waves leave the barrier together, and the two phases that read operands from LDS would then
    // coincide in every wave, with the LDS idle in between.  Odd waves therefore request the next tile
    // (address arithmetic, no LDS) at the END of their iteration instead of the beginning: their LDS
    // phases fall into the others' arithmetic.  Either way the stage a request overwrites was last read
    // in the iteration before the barrier this wave has passed, and the same loads are in flight at the wait.
    const bool late_request = (w & 1) != 0;
    auto tile_by_tile = [&](int kt) {
        bf16_t* stage = smem + (kt % NS) * (C::STAGE_BYTES / 2);
        if (!late_request) request_upto(kt + AHEAD);
        const int j0 = kt * C::BN, j1 = min(j0 + C::BN, J.nstr) - 1;   // first and last live streamed row
        // does this wave's 32 x 32 block hold no visible pair, only visible pairs, or both?
        bool none = !has_rows, cut = j0 + C::BN > J.nstr;
        bool lane_rule = false, lane_vis = true;   // VIS_MEMKEYS on a tile of one chunk: visibility is a property of the lane
        if (J.vis == VIS_CAUSAL) {
            none = none || j0 > J.cb + r_hi;
            cut = cut || j0 + C::BN - 1 > J.cb + row0;
        } else if (J.vis == VIS_FROM_ROW) {
            none = none || j1 < row0;
            cut = cut || j0 < r_hi;
        } else {
            const TileInfo ti = tile_info(J.str, J.nstr, j0);
            const int z = ti.in0 ? J.z0 - ti.slab_index : J.z1 + ti.slab_index;   // chunk of the tile's rows, if it has just one
            if (!ti.contig) cut = true;
            else {
                if (ti.in0) { none = none || yk_lo >= z; cut = cut || yk_hi >= z; }
                else { none = none || z < yk_lo || z > yk_hi; cut = cut || yk_lo != z || yk_hi != z; }
                // all 32 rows are of chunk z: whether this lane's key sees them does not depend on the row.
                // (Only compiled into the kernels with fewer than 4 waves, whose blocks are the ones that own keys
                // of several chunks per wave at the paper's shapes; in the 4-wave kernel the extra path costs the
                // common case 9 % through code layout alone, measured.)
                if constexpr (NW < 4) {
                    lane_rule = true;
                    lane_vis = ti.in0 ? yk < z : yk == z;
                }
            }
        }
        if (!none) {
            const bf16_t* Xs = stage;
            const bf16_t* Ys = stage + C::TILE;
            auto read_t = [&](const bf16_t* base, int step, int dt) -> bf16x8 {
                const s16x4 lo = lds_read_tr(base + toff[0][dt] + 16 * step * D);
                const s16x4 hi = lds_read_tr(base + toff[1][dt] + 16 * step * D);
                return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
            };
            // ---- S' = X xo^T, dP' = Y yo^T: accumulator i of lane (l32, g) is streamed row 8*(i/4) + 4*g + i%4 ----
            // The LDS operands are read PF k-steps ahead of the MFMAs that use them (the scheduling
            // barriers keep the reads from sinking back next to their uses).
            f32x16 S = zero16, dP = zero16;
            {
                constexpr int PF = C::KSTEPS >= 4 ? 4 : C::KSTEPS;
                bf16x8 ax[PF], ay[PF];
#pragma unroll
                for (int ks = 0; ks < PF; ++ks) {
                    ax[ks] = *reinterpret_cast<const bf16x8*>(Xs + poff[ks]);
                    ay[ks] = *reinterpret_cast<const bf16x8*>(Ys + poff[ks]);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int ks = 0; ks < C::KSTEPS; ++ks) {
                    if constexpr (PASS == PASS_DKV) {
                        if (ks == 0) { mfma_owner_first(S, ax[0], xo[0]); mfma_owner_first(dP, ay[0], yo[0]); }
                        else { mfma_owner(S, ax[ks % PF], xo[ks]); mfma_owner(dP, ay[ks % PF], yo[ks]); }
                    } else {
                        S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ax[ks % PF], xo[ks], S, 0, 0, 0);
                        dP = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ay[ks % PF], yo[ks], dP, 0, 0, 0);
                    }
                    if (ks + PF < C::KSTEPS) {
                        ax[ks % PF] = *reinterpret_cast<const bf16x8*>(Xs + poff[ks + PF]);
                        ay[ks % PF] = *reinterpret_cast<const bf16x8*>(Ys + poff[ks + PF]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            // the transposed operands of the first 16 streamed rows are requested before the arithmetic below
            bf16x8 tx[2][C::DT], ty[2][PASS == PASS_DKV ? C::DT : 1];
#pragma unroll
            for (int dt = 0; dt < C::DT; ++dt) {
                tx[0][dt] = read_t(Xs, 0, dt);
                if constexpr (PASS == PASS_DKV) ty[0][dt] = read_t(Ys, 0, dt);
            }
            if constexpr (PASS == PASS_DKV) settle_scores();
            __builtin_amdgcn_sched_barrier(0);
            // ---- P = exp2(S' sc + nl), dS = P (dP' - delta) ----------------------------------------------
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
                        const float p = __builtin_amdgcn_exp2f(fmaf(S[4 * a + e], sc, lsv[e]));
                        S[4 * a + e] = p;
                        dP[4 * a + e] = p * (dP[4 * a + e] - dlv[e]);
                    }
                }
            }
            if (cut && lane_rule) {   // (a tile of consecutive rows lies inside the list: no row is past its end)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    S[i] = lane_vis ? S[i] : 0.f;
                    dP[i] = lane_vis ? dP[i] : 0.f;
                }
            } else if (cut) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int j = j0 + 8 * (i >> 2) + 4 * g + (i & 3);
                    bool vis = j < J.nstr;
                    if (J.vis == VIS_CAUSAL) vis = vis && j <= J.cb + r_own;
                    else if (J.vis == VIS_FROM_ROW) vis = vis && j >= r_own;
                    else {
                        int a;
                        list_row(J.str, min(j, J.nstr - 1), &a);
                        vis = vis && (j < J.str.n0 ? yk < J.z0 - a : yk == J.z1 + a);
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
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int step = 0; step < 2; ++step) {
                if (step == 0) {
#pragma unroll
                    for (int dt = 0; dt < C::DT; ++dt) {
                        tx[1][dt] = read_t(Xs, 1, dt);
                        if constexpr (PASS == PASS_DKV) ty[1][dt] = read_t(Ys, 1, dt);
                    }
                }
                const bf16x8 bds = pack8(dP, step);
                const bf16x8 bp = pack8(S, step);
                if constexpr (PASS == PASS_DKV) {
                    static_for<0, C::DT>([&](auto dt) {
                        mfma_named<16 * dt.value>(tx[step][dt.value], bds);
                        mfma_named<64 + 16 * dt.value>(ty[step][dt.value], bp);
                    });
                } else {
#pragma unroll
                    for (int dt = 0; dt < C::DT; ++dt)
                        accX[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tx[step][dt], bds, accX[dt], 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if (late_request) request_upto(kt + AHEAD);
        wait_for(kt + 1);
        __syncthreads();
    };

    // Tiles [0, q1) are whole tiles of 32 consecutive rows: they go through the pipelined loop, those outside
    // [p0, p1) -- where not every pair is visible -- with its masked steps.  The rest goes tile by tile.
    int p0 = 0, p1 = 0, q1 = 0;
    if constexpr (PASS == PASS_DKV) {
        p0 = J.pipe0; p1 = J.pipe1; q1 = J.pipe_end;
        if (q1 < 3) p0 = p1 = q1 = 0;
    }
    if constexpr (PASS == PASS_DKV) {
        if (q1 > 0) {
            // In iteration i: S', dP' of tile i + 1 and the accumulation of tile i - 1 on the matrix pipe between the
            // exponentials of tile i.  Two sets of score registers and of packed operands take turns.
            f32x16 Sa, dPa, Sb, dPb;
            uint32_t pka[2][8], pkb[2][8];
            auto stage_of = [&](int kt) -> const bf16_t* { return smem + (kt % NS) * (C::STAGE_BYTES / 2); };
            // per-lane threshold of a tile that is not fully visible (see pipe_step)
            auto threshold = [&](int i) -> int {
                if (J.vis == VIS_FROM_ROW) return r_own - C::BN * i - 4 * g;
                const TileInfo ti = tile_info(J.str, J.nstr, i * C::BN);
                const bool vis = ti.in0 ? yk < J.z0 - ti.slab_index : yk == J.z1 + ti.slab_index;
                return vis ? -1 : 64;
            };
            request_upto(AHEAD);
            pipe_step<D, PASS, true, false, false>(stage_of(0), nullptr, nullptr, poff, toff, xo, yo, Sa, dPa, Sa, dPa, pka, pkb,
                                                  accX, sc, nl_own, dl_own, g);
            wait_for(1);
            __syncthreads();
            // even steps read (Sa, dPa) and the packed operands in pkb and write (Sb, dPb) and pka; odd steps the
            // other way round.  The steady loop takes an odd and an even step per trip, in straight-line code, so
            // that no register moves between the sets.
            auto sync_after = [&](int i) {
                wait_for(i + 2);
                __syncthreads();
            };
#define LOMA_STEP_ARGS(I_, SN, DPN, SC, DPC, PKO, PKI) \
    stage_of((I_) + 1), stage_of(I_), stage_of((I_)-1), poff, toff, xo, yo, SN, DPN, SC, DPC, PKO, PKI, accX, sc, nl_own, dl_own, g
#define LOMA_STEP(A_, C_, I_, SN, DPN, SC, DPC, PKO, PKI)                                                             \
    do {                                                                                                              \
        if ((I_) >= p0 && (I_) < p1) pipe_step<D, PASS, A_, true, C_, false>(LOMA_STEP_ARGS(I_, SN, DPN, SC, DPC, PKO, PKI)); \
        else pipe_step<D, PASS, A_, true, C_, true>(LOMA_STEP_ARGS(I_, SN, DPN, SC, DPC, PKO, PKI), threshold(I_));  \
    } while (0)
            int i = 0;
            request_upto(i + AHEAD);
            LOMA_STEP(true, false, i, Sb, dPb, Sa, dPa, pka, pkb);
            sync_after(i);
            ++i;
            for (; i + 2 < q1; i += 2) {
                request_upto(i + AHEAD);
                LOMA_STEP(true, true, i, Sa, dPa, Sb, dPb, pkb, pka);
                sync_after(i);
                request_upto(i + 1 + AHEAD);
                LOMA_STEP(true, true, i + 1, Sb, dPb, Sa, dPa, pka, pkb);
                sync_after(i + 1);
            }
            // one or two steps are left (q1 >= 3): the last one starts no new tile
            if (i + 2 == q1) {
                request_upto(i + AHEAD);
                LOMA_STEP(true, true, i, Sa, dPa, Sb, dPb, pkb, pka);
                sync_after(i);
                request_upto(i + 1 + AHEAD);
                LOMA_STEP(false, true, i + 1, Sb, dPb, Sa, dPa, pka, pkb);
                sync_after(i + 1);
                pipe_step<D, PASS, false, false, true>(LOMA_STEP_ARGS(q1, Sa, dPa, Sb, dPb, pkb, pka));
            } else {
                request_upto(i + AHEAD);
                LOMA_STEP(false, true, i, Sa, dPa, Sb, dPb, pkb, pka);
                sync_after(i);
                pipe_step<D, PASS, false, false, true>(LOMA_STEP_ARGS(q1, Sb, dPb, Sa, dPa, pka, pkb));
            }
#undef LOMA_STEP
#undef LOMA_STEP_ARGS
        }
    }
    for (int kt = q1; kt < ntiles; ++kt) tile_by_tile(kt);

    // rows leave through the wave's own fp32 staging area (the tile stages are free: the loop ended on a barrier)
    float* Of = reinterpret_cast<float*>(smem) + w * (C::WAVE_STAGING_BYTES / 4);
    if constexpr (PASS == PASS_DKV) settle_acc();
    if (has_rows) {
        if constexpr (PASS == PASS_DQ) {
            stage_acc<D>(accX, scale, Of, lane);
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            if (J.rep) store_staged_rep<D>(Of, T, J, row0, scale, sc, lane);
            else store_staged<D>(Of, T.dq, J, row0, lane);
        } else {
            fetch_named<0, C::DT>(accX);
            stage_acc<D>(accX, scale, Of, lane);
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            if (J.part_k) store_staged_partial<D>(Of, J.part_k, J, row0, lane);
            else store_staged<D>(Of, T.dk, J, row0, lane);
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            fetch_named<64, C::DT>(accX);
            stage_acc<D>(accX, 1.f, Of, lane);
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            if (J.part_v) store_staged_partial<D>(Of, J.part_v, J, row0, lane);
            else store_staged<D>(Of, T.dv, J, row0, lane);
        }
    }
}

__device__ __forceinline__ void split_block(long long id, int nbh, int jobs_per_bh, int nlong, int& bh, int& u) {
    // (b,h) pairs are dealt to the 8 XCDs (workgroup id % 8) so that one pair's rows stay in one L2.  Jobs
    // 0 .. nlong-1 of a pair are its long ones, longest first: an XCD starts with job 0 of each of its pairs, then
    // job 1 of each, ..., and only then walks the short jobs pair by pair.  Workgroups are handed out in id order as
    // slots come free, so this is longest-first list scheduling over the XCD's CUs: the launch ends within a percent
    // of the even split (simulated for the long-context shape; walking the pairs one after the other, long and short
    // jobs together, started the last pair's longest job at three quarters of the launch and ended 30 % late).
    // Measured alternative: the long jobs pair by pair (a pair's jobs, which stream the same rows, start together)
    // moves 9 % fewer bytes at the same time at the long-context shape and is 10 % slower at the Llama-7B shape.
    if (nbh % 8 == 0) {
        const int xcd = (int)(id % 8), pairs = nbh / 8;
        const long long k = id / 8;
        if (k < (long long)pairs * nlong) {
            bh = xcd + 8 * (int)(k % pairs);
            u = (int)(k / pairs);
        } else {
            const long long k2 = k - (long long)pairs * nlong;
            const int nshort = jobs_per_bh - nlong;
            bh = xcd + 8 * (int)(k2 / nshort);
            u = nlong + (int)(k2 % nshort);
        }
    } else {
        bh = (int)(id % nbh);
        u = (int)(id / nbh);
    }
}

constexpr int ONE_SLAB = 1 << 30;   // slab length of a range that is a single run of rows (its magic is 0: slab index 0)
__device__ __forceinline__ RowList one_range(int base, int n) {
    RowList L;
    L.base0 = 0; L.n0 = 0; L.slab0 = ONE_SLAB; L.stride0 = 0; L.magic0 = 0;
    L.base1 = base; L.n1 = n; L.slab1 = ONE_SLAB; L.stride1 = 0; L.magic1 = 0;
    return L;
}
__device__ __forceinline__ RowList owner_range(int base) {   // entry r of range 0 is row base + r
    RowList L = one_range(0, 0);
    L.base0 = base; L.n0 = 0x7fffffff;
    return L;
}

__device__ __forceinline__ BwdTensors at_sequence(const BwdTensors& T, long seq, int D) {
    BwdTensors U;
    U.q = T.q + seq * D; U.k = T.k + seq * D; U.v = T.v + seq * D; U.dout = T.dout + seq * D; U.out = T.out + seq * D;
    U.lse = T.lse + seq; U.nl = T.nl + seq; U.delta = T.delta + seq;
    U.dq = T.dq + seq * D; U.dk = T.dk + seq * D; U.dv = T.dv + seq * D;
    return U;
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

}  // namespace
}  // namespace loma
