// Matrix-pipe ceiling probe: the register-blocked wave tile of the GEMM kernels (8 x 8 blocks of
// 16 x 16, two k sub-steps per iteration, one wave per SIMD, 256 workgroups) with the operand
// fragments held in registers -- no LDS, no global memory inside the loop.  What it reaches on
// the caller's operand values is what the matrix instructions alone sustain on this GPU under
// this load: the number a measured GEMM is to be set beside, next to the nominal peak.  The
// loop is stamped with the shader-clock counter and the constant 100 MHz counter, whose ratio
// is the clock the GPU sustained while the loop ran.
#include <hip/hip_runtime.h>

#include "../../include/prism_gemm.h"
#include "lane.hpp"
#include "wave.hpp"

namespace prism {
namespace {

constexpr int kProbeWorkgroups = 256, kProbeThreads = 256, kProbeFragments = 32;

template <typename T>
__global__ __launch_bounds__(kProbeThreads) void mfma_probe(const u32x4* __restrict__ operands, uint64_t* counters, int iterations)
{
    const persp::Wave wv = persp::Grid::at_kernel_entry().workgroup().wave();
    using frag_t = typename Frag<T>::type;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    frag_t fa[2][8], fb[2][8];
    const u32x4* mine = operands + static_cast<size_t>(blockIdx.x * 4 + wave) * kProbeFragments * 64 + lane;
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            fa[s][i] = __builtin_bit_cast(frag_t, mine[(s * 16 + i) * 64]);
            fb[s][i] = __builtin_bit_cast(frag_t, mine[(s * 16 + 8 + i) * 64]);
        }
    __builtin_amdgcn_s_waitcnt(0);
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            asm volatile("" : "+v"(fa[s][i]));
            asm volatile("" : "+v"(fb[s][i]));
        }
    wave::Tile<T, 8, 8> acc;
    acc.clear();
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) asm volatile("" : "+a"(acc.acc[i][j]));
    const uint64_t c0 = __builtin_readcyclecounter(), r0 = __builtin_amdgcn_s_memrealtime();
    for (int it = 0; it < iterations; ++it) {
        acc.mma(wv, fa[0], fb[0]);
        acc.mma(wv, fa[1], fb[1]);
        __builtin_amdgcn_sched_barrier(0);
    }
    const uint64_t c1 = __builtin_readcyclecounter(), r1 = __builtin_amdgcn_s_memrealtime();
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) asm volatile("" : "+a"(acc.acc[i][j]));
    float total = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) total += acc.acc[i][j][0] + acc.acc[i][j][1] + acc.acc[i][j][2] + acc.acc[i][j][3];
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) total += __shfl_xor(total, d, 64);
    if (lane == 0) {
        uint64_t* out = counters + (blockIdx.x * 4 + wave) * 4;
        out[0] = c1 - c0;
        out[1] = r1 - r0;
        out[2] = __builtin_bit_cast(uint32_t, total);  // keeps the products alive
        out[3] = static_cast<uint64_t>(iterations);
    }
}

}  // namespace
}  // namespace prism

extern "C" prism_status_t prism_mfma_probe(int32_t ab_dtype, const void* operands, size_t operand_bytes, int32_t iterations,
                                           uint64_t* counters, size_t counter_bytes, void* hip_stream)
{
    using namespace prism;
    if (ab_dtype != PRISM_DTYPE_BF16 && ab_dtype != PRISM_DTYPE_F16 && ab_dtype != PRISM_DTYPE_F32) return PRISM_ERR_UNSUPPORTED;
    if (!operands || !counters || iterations < 1) return PRISM_ERR_INVALID_ARG;
    if (operand_bytes < PRISM_MFMA_PROBE_OPERAND_BYTES || counter_bytes < PRISM_MFMA_PROBE_COUNTER_BYTES) return PRISM_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(operands) % 16 != 0 || reinterpret_cast<uintptr_t>(counters) % 8 != 0) return PRISM_ERR_INVALID_ARG;
    static_assert(PRISM_MFMA_PROBE_OPERAND_BYTES == size_t{kProbeWorkgroups} * 4 * kProbeFragments * 64 * 16, "operand layout");
    static_assert(PRISM_MFMA_PROBE_COUNTER_BYTES == size_t{kProbeWorkgroups} * 4 * 4 * 8, "counter layout");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const u32x4* src = static_cast<const u32x4*>(operands);
    if (ab_dtype == PRISM_DTYPE_BF16)
        hipLaunchKernelGGL(mfma_probe<bf16_t>, dim3(kProbeWorkgroups), dim3(kProbeThreads), 0, stream, src, counters, iterations);
    else if (ab_dtype == PRISM_DTYPE_F16)
        hipLaunchKernelGGL(mfma_probe<f16_t>, dim3(kProbeWorkgroups), dim3(kProbeThreads), 0, stream, src, counters, iterations);
    else
        hipLaunchKernelGGL(mfma_probe<f32_t>, dim3(kProbeWorkgroups), dim3(kProbeThreads), 0, stream, src, counters, iterations);
    return hipGetLastError() == hipSuccess ? PRISM_OK : PRISM_ERR_LAUNCH;
}
