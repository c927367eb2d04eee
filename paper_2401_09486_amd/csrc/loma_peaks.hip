// Measuring sticks for bench.py (built into their own small library, libloma_peaks.so; not part of the
// product ABI): how fast this chip runs the matrix instruction the attention kernels are built on, how fast
// a plain streaming copy moves bytes, and what a vector-ALU instruction of the softmax costs a SIMD.  The roofline fractions are quoted against the published peaks; these say
// how much of those a kernel can reach at all on the box at hand.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

// Every wave issues `iters` x 8 independent v_mfma_f32_32x32x16_bf16 (4 accumulator sets, so the pipe never waits
// for a result); operands stay in registers.  2 * 32 * 32 * 16 flop per instruction.
__global__ __launch_bounds__(256) void mfma_loop_kernel(int iters, float* sink) {
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(0.001f * (threadIdx.x + i)); b[i] = (__bf16)(0.002f * (threadIdx.x - i)); }
    f32x16 acc[4] = {};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int s = 0; s < 4; ++s) acc[s] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[s], 0, 0, 0);
    }
    float x = 0.f;
    for (int s = 0; s < 4; ++s)
        for (int i = 0; i < 16; ++i) x += acc[s][i];
    if (x == 12345.678f) sink[0] = x;   // keeps the loop alive without a store on the usual path
}

// Every wave issues `iters` x 16 vector-ALU instructions of one kind with no dependences between neighbours
// (eight result registers in turn): KIND 0 = v_exp_f32 (the softmax's exponential, a transcendental), KIND 1 =
// v_fma_f32 (stands for the plain fp32 instructions).  One workgroup per CU with 4 or 8 waves gives one or two
// waves per SIMD: the time per instruction is what the instruction occupies the SIMD's vector ALU for (two waves)
// or what a lone wave can issue (one wave).
template <int KIND>
__global__ __launch_bounds__(512) void valu_loop_kernel(int iters, float* sink) {
    float x[8];
    for (int i = 0; i < 8; ++i) x[i] = 0.001f * threadIdx.x + i;
    const float a = 0.999f, b = 0.25f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < 16; ++s) {
            if (KIND == 0) asm volatile("v_exp_f32 %0, %1" : "=v"(x[s & 7]) : "v"(b));
            else asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(x[s & 7]) : "v"(a), "v"(b));
        }
    }
    float y = 0.f;
    for (int i = 0; i < 8; ++i) y += x[i];
    if (y == 12345.678f) sink[0] = y;
}

// Grid-stride copy with 16-byte accesses, four independent pieces per thread and trip: reads n16 * 16 bytes and
// writes as many.
__global__ __launch_bounds__(256) void stream_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n16) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const u32x4 a = __builtin_nontemporal_load(src + i), b = __builtin_nontemporal_load(src + i + stride);
        const u32x4 c = __builtin_nontemporal_load(src + i + 2 * stride), d = __builtin_nontemporal_load(src + i + 3 * stride);
        __builtin_nontemporal_store(a, dst + i);
        __builtin_nontemporal_store(b, dst + i + stride);
        __builtin_nontemporal_store(c, dst + i + 2 * stride);
        __builtin_nontemporal_store(d, dst + i + 3 * stride);
    }
    for (; i < n16; i += stride) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}
// Read-only stream (what decode does): eight independent 16-byte loads per thread and trip, folded into one word.
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4* __restrict__ src, size_t n16, unsigned* sink) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    unsigned x = 0;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; i + 7 * stride < n16; i += 8 * stride) {
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < 8; ++u) x ^= v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
    }
    for (; i < n16; i += stride) {
        const u32x4 v = __builtin_nontemporal_load(src + i);
        x ^= v[0] ^ v[1] ^ v[2] ^ v[3];
    }
    if (x == 0x12345678u) sink[0] = x;
}

}  // namespace

extern "C" {

// Enqueue the MFMA loop: `workgroups` x 4 waves x iters x 8 instructions.  Returns the flop it performs, 0 on a failed launch.
double loma_peaks_mfma_loop(int workgroups, int iters, float* sink, void* stream) {
    if (workgroups < 1 || iters < 1) return 0.0;
    hipLaunchKernelGGL(mfma_loop_kernel, dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(stream), iters, sink);
    if (hipGetLastError() != hipSuccess) return 0.0;
    return (double)workgroups * 4.0 * iters * 8.0 * (2.0 * 32 * 32 * 16);
}

// Enqueue the vector-ALU loop of `kind` (0: v_exp_f32, 1: v_fma_f32) on `workgroups` workgroups of `waves` waves (4 or 8).
// Returns the instructions one wave issues (iters x 16), 0 on a bad argument or a failed launch.
double loma_peaks_valu_loop(int kind, int waves, int workgroups, int iters, float* sink, void* stream) {
    if ((kind != 0 && kind != 1) || (waves != 4 && waves != 8) || workgroups < 1 || iters < 1) return 0.0;
    if (kind == 0) hipLaunchKernelGGL(valu_loop_kernel<0>, dim3(workgroups), dim3(64 * waves), 0, static_cast<hipStream_t>(stream), iters, sink);
    else hipLaunchKernelGGL(valu_loop_kernel<1>, dim3(workgroups), dim3(64 * waves), 0, static_cast<hipStream_t>(stream), iters, sink);
    if (hipGetLastError() != hipSuccess) return 0.0;
    return (double)iters * 16.0;
}

// Enqueue a copy of `bytes` (multiple of 16) from src to dst; returns 0 on success.
int loma_peaks_stream_copy(const void* src, void* dst, size_t bytes, int workgroups, void* stream) {
    if (src == nullptr || dst == nullptr || bytes % 16 != 0 || workgroups < 1) return -1;
    hipLaunchKernelGGL(stream_copy_kernel, dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u32x4*>(src), static_cast<u32x4*>(dst), bytes / 16);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

int loma_peaks_stream_read(const void* src, size_t bytes, int workgroups, unsigned* sink, void* stream) {
    if (src == nullptr || bytes % 16 != 0 || workgroups < 1) return -1;
    hipLaunchKernelGGL(stream_read_kernel, dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u32x4*>(src), bytes / 16, sink);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // extern "C"
