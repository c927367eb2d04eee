// Rotary position embedding applied while q and k rows are loaded (position ids of Sec. 4.5 / Appendix A).
// Convention: head-dim element i < D/2 pairs with element i + D/2; the pair turns by pos * theta^(-2i/D):
//     y[i] = x[i] cos - x[i + D/2] sin,   y[i + D/2] = x[i + D/2] cos + x[i] sin.
// The host fills a table of the D/2 frequencies in TURNS per position (fp64: theta^(-2i/D) / 2 pi); the device
// multiplies by the integer position in fp64, keeps the fractional turn and evaluates sin and cos of it in fp32,
// so the angle is good to ~1e-7 rad at any position the ids can reach.  Not part of the ABI.
#pragma once
#include <cmath>

#include "loma_internal.h"

namespace loma {

struct RopeTable {
    double turns[64];   // per pair i < D/2 (D <= 128): theta^(-2i/D) / (2 pi)
    int pos_first;      // position id of row 0
    int pos_stride;     // id step from row to row
};

inline RopeTable make_rope_table(int D, float theta, int pos_first, int pos_stride) {
    RopeTable T = {};
    const double two_pi = 6.283185307179586476925286766559;
    for (int i = 0; i < D / 2; ++i) T.turns[i] = std::pow((double)theta, -2.0 * i / D) / two_pi;
    T.pos_first = pos_first;
    T.pos_stride = pos_stride;
    return T;
}

namespace rope {

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;

__device__ __forceinline__ unsigned pack2(float a, float b) {
    f32x2 f = {a, b};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(f, bf16x2));   // round to nearest even
}

// One 16-byte piece (8 consecutive head-dim elements starting at e0, a multiple of 8) of a row at position `pos`,
// rotated.  `own` is that piece, `partner` the piece 8 * ((e0 / 8 + D / 16) % (D / 8)) of the same row.
// Every product and sum is written out with its rounding, so that two call sites produce the same bits.
template <int D>
__device__ __forceinline__ u32x4 rotate_piece(u32x4 own, u32x4 partner, int e0, int pos, const RopeTable& T) {
    const bool low = e0 < D / 2;              // low half: y = x cos - p sin; high half: y = x cos + p sin
    const int i0 = low ? e0 : e0 - D / 2;
    float y[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const unsigned xw = own[j >> 1], pw = partner[j >> 1];
        const float x = __uint_as_float((j & 1) ? (xw & 0xffff0000u) : (xw << 16));
        const float p = __uint_as_float((j & 1) ? (pw & 0xffff0000u) : (pw << 16));
        double u = (double)pos * T.turns[i0 + j];
        u -= floor(u);                         // fraction of a turn, [0, 1)
        float s, c;
        sincospif(2.f * (float)u, &s, &c);
        const float ps = __fmul_rn(p, s);
        y[j] = __fmaf_rn(x, c, low ? -ps : ps);
    }
    u32x4 r;
    r[0] = pack2(y[0], y[1]); r[1] = pack2(y[2], y[3]); r[2] = pack2(y[4], y[5]); r[3] = pack2(y[6], y[7]);
    return r;
}

// The rotated piece `piece` (of D / 8) of the bf16 row at `row`.
template <int D>
__device__ __forceinline__ u32x4 load_rotated_piece(const uint16_t* row, int piece, int pos, const RopeTable& T) {
    constexpr int CPR = D / 8;
    const u32x4 own = *reinterpret_cast<const u32x4*>(row + piece * 8);
    const u32x4 partner = *reinterpret_cast<const u32x4*>(row + ((piece + CPR / 2) % CPR) * 8);
    return rotate_piece<D>(own, partner, piece * 8, pos, T);
}

}  // namespace rope
}  // namespace loma
