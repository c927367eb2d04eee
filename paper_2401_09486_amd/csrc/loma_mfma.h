// Device helpers shared by the MFMA kernels of libloma (gfx950): vector types, bf16 packing, the
// half-wave and row reductions, direct HBM -> LDS loads with hand-placed waits, the transposing
// LDS read.  Not part of the ABI.
#pragma once
#include <type_traits>

#include "loma_internal.h"

namespace loma {
namespace mfma {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef uint16_t bf16_t;  // storage type of bf16 tensors

constexpr int NO_CAUSAL = 1 << 29;
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// two floats -> packed bf16 pair, round to nearest even
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    f32x2 f = {a, b};
    bf16x2 h = __builtin_convertvector(f, bf16x2);
    return __builtin_bit_cast(uint32_t, h);
}

// value held by the other half-wave's lane (l ^ 32) and own value: returns max / sum over the pair
__device__ __forceinline__ float pair_max(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float pair_sum(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// sum over the CPR consecutive lanes (8 or 16) that hold one row; every lane gets the total
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x) {
    const int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false);
    return x + __int_as_float(y);
}
template <int CPR>
__device__ __forceinline__ float row_sum(float x) {
    static_assert(CPR == 8 || CPR == 16, "lanes per row");
    x = dpp_add<0xB1>(x);   // quad_perm [1,0,3,2]
    x = dpp_add<0x4E>(x);   // quad_perm [2,3,0,1]
    x = dpp_add<0x141>(x);  // row_half_mirror
    if (CPR == 16) x = dpp_add<0x140>(x);  // row_mirror
    return x;
}

// One wave-wide direct load: lane l's 16 bytes at `src` land at LDS byte 16*l past `lds_dst`
// (wave-uniform).  Written as inline assembly so that the compiler does not order later LDS
// reads of the OTHER tile buffer behind it; the waits are placed by hand (wait_direct_loads).
__device__ __forceinline__ void direct_load_16B(const bf16_t* src, bf16_t* lds_dst) {
    const unsigned dst = __builtin_amdgcn_readfirstlane(
        (unsigned)(size_t)(__attribute__((address_space(3))) bf16_t*)lds_dst);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(dst), "v"(src) : "memory", "m0");
}

// a pointer every lane agrees on, moved to scalar registers
__device__ __forceinline__ const bf16_t* uniform_ptr(const bf16_t* p) {
    const uint64_t x = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)x);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(x >> 32));
    return reinterpret_cast<const bf16_t*>(((uint64_t)hi << 32) | lo);
}

// all direct loads of this wave have landed in LDS (vmcnt(0); the other counters untouched)
__device__ __forceinline__ void wait_direct_loads() { __builtin_amdgcn_s_waitcnt(0x0F70); }
// all but the newest N vector-memory operations of this wave are complete
template <int N>
__device__ __forceinline__ void wait_direct_loads_but() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}
// the tile after the current one has landed although `ahead` younger tiles (LPT loads each) are still in flight
template <int LPT, int MAXAHEAD>
__device__ __forceinline__ void wait_next_tile(int ahead) {
    static_assert(MAXAHEAD <= 3 && MAXAHEAD * LPT < 64, "wait depth");
    if (MAXAHEAD >= 3 && ahead >= 3) wait_direct_loads_but<(MAXAHEAD >= 3 ? 3 : 0) * LPT>();
    else if (MAXAHEAD >= 2 && ahead == 2) wait_direct_loads_but<(MAXAHEAD >= 2 ? 2 : 0) * LPT>();
    else if (MAXAHEAD >= 1 && ahead == 1) wait_direct_loads_but<LPT>();
    else wait_direct_loads();
}

// Transposing LDS read: the 16 lanes of a group each point at 8 bytes; lane i of the group
// receives element (i % 4) of the lanes 4e + i/4, e = 0..3.  With lane i pointing at row i/4,
// columns 4*(i%4).., lane i ends up with column i of four consecutive rows.
typedef __attribute__((ext_vector_type(4))) short s16x4;
__device__ __forceinline__ s16x4 lds_read_tr(const bf16_t* p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) s16x4*)(const_cast<bf16_t*>(p)));
}

// ---- instructions pinned to their place in the instruction stream --------------------------------------------
// v_exp_f32 and the bf16 packing AT THEIR PLACE in the instruction stream: the compiler orders volatile statements
// among themselves and against the scheduling fences, so these two pin a score's arithmetic (which hangs between
// them by its data dependences) to the slot of the pipelined loop it is written in.
__device__ __forceinline__ float exp2_at(float x) {
    float y;
    asm volatile("v_exp_f32 %0, %1" : "=v"(y) : "v"(x));
    return y;
}
__device__ __forceinline__ uint32_t pack_bf16_at(float a, float b) {
    uint32_t r;
    asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// MFMA with its accumulator in ordinary registers, as a volatile statement (same ordering guarantee).  Opaque to
// the compiler's hazard bookkeeping in both directions.  After: the result is read by other code only many
// instructions later (callers see to that).  Before: the compiler may have written an operand with a vector-ALU
// instruction just ahead of the statement -- it copies a 16-register accumulator to other registers when it likes,
// and did so right before an MFMA in a rarely run path -- and the matrix pipe must not read a register within two
// wait states of such a write: the two idle cycles come with the instruction.
__device__ __forceinline__ void mfma_at(f32x16& acc, bf16x8 a, bf16x8 b) {
    asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
}
__device__ __forceinline__ void mfma_first_at(f32x16& acc, bf16x8 a, bf16x8 b) {   // accumulator starts at zero
    asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(acc) : "v"(a), "v"(b));
}

// ---- accumulators that live in the accumulation registers a0..a127 BY NAME ------------------------------------
// For kernels whose MFMA accumulators do not fit the 256 ordinary registers of a lane next to everything else
// (as C++ values the compiler copies them between the register files on every tile).  Every statement names all
// 128 registers as clobbered, so the compiler keeps nothing of its own there across them.  The instructions are
// opaque to the compiler's hazard bookkeeping: consecutive MFMAs must name different accumulators, and
// settle_acc() comes before the first read of one.
#define LOMA_ACC_REGS "a0","a1","a2","a3","a4","a5","a6","a7","a8","a9","a10","a11","a12","a13","a14","a15","a16","a17","a18","a19","a20","a21","a22","a23","a24","a25","a26","a27","a28","a29","a30","a31","a32","a33","a34","a35","a36","a37","a38","a39","a40","a41","a42","a43","a44","a45","a46","a47","a48","a49","a50","a51","a52","a53","a54","a55","a56","a57","a58","a59","a60","a61","a62","a63","a64","a65","a66","a67","a68","a69","a70","a71","a72","a73","a74","a75","a76","a77","a78","a79","a80","a81","a82","a83","a84","a85","a86","a87","a88","a89","a90","a91","a92","a93","a94","a95","a96","a97","a98","a99","a100","a101","a102","a103","a104","a105","a106","a107","a108","a109","a110","a111","a112","a113","a114","a115","a116","a117","a118","a119","a120","a121","a122","a123","a124","a125","a126","a127"
template <int BASE>
__device__ __forceinline__ void mfma_named(bf16x8 a, bf16x8 b) {
    asm volatile("v_mfma_f32_32x32x16_bf16 a[%2:%3], %0, %1, a[%2:%3]" ::"v"(a), "v"(b), "n"(BASE), "n"(BASE + 15)
                 : LOMA_ACC_REGS);
}
template <int I>
__device__ __forceinline__ void zero_named() {
    asm volatile("v_accvgpr_write_b32 a[%0], 0" ::"n"(I) : LOMA_ACC_REGS);
}
template <int I>
__device__ __forceinline__ float read_named() {
    float x;
    asm volatile("v_accvgpr_read_b32 %0, a[%1]" : "=v"(x) : "n"(I) : LOMA_ACC_REGS);
    return x;
}
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}
// the last MFMA (16 passes of 4 cycles) has written its accumulator
__device__ __forceinline__ void settle_acc() { asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory"); }
// a[BASE .. BASE + 16 DT) -> accumulator values in the layout of the MFMA result
template <int BASE, int DT>
__device__ __forceinline__ void fetch_named(f32x16 (&acc)[DT]) {
    static_for<0, 16 * DT>([&](auto i) { acc[i.value / 16][i.value % 16] = read_named<BASE + i.value>(); });
}

template <int I>
__device__ __forceinline__ void write_named(float x) {
    asm volatile("v_accvgpr_write_b32 a[%0], %1" ::"n"(I), "v"(x) : LOMA_ACC_REGS);
}

}  // namespace mfma
}  // namespace loma
