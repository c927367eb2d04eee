// dQ pass of the mask pass's gradients on the matrix cores (engine and notation: loma_bwd_engine.h).
#include "loma_bwd_engine.h"

namespace loma {
namespace {

// dQ pass: the forward pass's blocks (one zone of one chunk, bm rows), last chunk first
template <int D, int NW>
__global__ __launch_bounds__(64 * NW) void bwd_dq_kernel(BwdParams P) {
    extern __shared__ __align__(16) bf16_t smem[];
    const MaskSchedule sch = MaskSchedule::make(P.nbh, P.t, P.R / P.t, P.n, P.bm);
    const MaskJob mj = sch.decode(blockIdx.x);
    const int chunk = mj.y * P.s;
    BwdJob J;
    J.ooff = 0; J.orows = mj.rows;
    J.vis = VIS_CAUSAL; J.cb = NO_CAUSAL; J.t = P.t; J.z0 = J.z1 = 0; J.magic_t = 0; J.rep = 0;
    J.part_k = J.part_v = nullptr;
    J.pipe0 = J.pipe1 = J.pipe_end = 0;
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

template <int D>
int launch_dq(const BwdParams& P, hipStream_t st) {
    const long long grid = MaskSchedule::make(P.nbh, P.t, P.R / P.t, P.n, P.bm).size();
    if (P.bm == 128) return launch(bwd_dq_kernel<D, 4>, grid, 256, BCfg<D>::smem_bytes(4, Stages<PASS_DQ, 4>::NS), P, st);
    if (P.bm == 64) return launch(bwd_dq_kernel<D, 2>, grid, 128, BCfg<D>::smem_bytes(2, Stages<PASS_DQ, 2>::NS), P, st);
    return launch(bwd_dq_kernel<D, 1>, grid, 64, BCfg<D>::smem_bytes(1, Stages<PASS_DQ, 1>::NS), P, st);
}

}  // namespace

int launch_bwd_dq_pass(const BwdParams& P, int D, hipStream_t st) {
    return D == 128 ? launch_dq<128>(P, st) : launch_dq<64>(P, st);
}

}  // namespace loma
