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

// ---- layout probes: the lane layouts the kernels rely on, shown on the device ------------------
// One wavefront each.  They use the very functions the GEMM kernels use, so a wrong layout
// assumption in those functions shows up as a wrong matrix on the host.

// D = R * C^T for a 16 x 32 row operand R and a 16 x 32 column operand C (both row-major, K
// contiguous), one matrix instruction; the accumulators are scattered to a row-major 16 x 16
// matrix with lane::acc_row / lane::acc_col.
template <typename T>
__global__ __launch_bounds__(64) void probe_accumulator_layout(const char* r_bits, const char* c_bits, float* d_out)
{
    const persp::Wave wv = persp::Grid::at_kernel_entry().workgroup<64>().wave();
    using frag_t = typename Frag<T>::type;
    const int lane = threadIdx.x;
    // the fragment a lane holds: 8 consecutive k of row lane % 16, k-quarter lane / 16 (lane::load_fragment)
    const int row = lane & 15, k0 = 8 * (lane >> 4);
    const frag_t r = __builtin_bit_cast(frag_t, *reinterpret_cast<const u32x4*>(r_bits + (row * 32 + k0) * 2));
    const frag_t c = __builtin_bit_cast(frag_t, *reinterpret_cast<const u32x4*>(c_bits + (row * 32 + k0) * 2));
    const f32x4 acc = wave::mfma_block(wv, r, c, f32x4{0.f, 0.f, 0.f, 0.f});
#pragma unroll
    for (int reg = 0; reg < 4; ++reg) d_out[lane::acc_row(reg, lane) * 16 + lane::acc_col(lane)] = acc[reg];
}

// A 32 (k) x 128 (elements) 16-bit matrix, row-major, is laid into LDS as the pipeline lays an
// operand kept as k-rows; every fragment half is fetched with wave::read_k_rows_half and written
// out as out[element][k] -- the transposed matrix if the documented lane layout holds.
__global__ __launch_bounds__(64) void probe_k_rows_read(const uint16_t* in, uint16_t* out)
{
    const persp::Wave wv = persp::Grid::at_kernel_entry().workgroup<64>().wave();
    constexpr int ROW_BYTES = 256;
    __shared__ __attribute__((aligned(1024))) char tile[32 * ROW_BYTES];
    const int lane = threadIdx.x;
    for (int q = lane; q < 32 * 16; q += 64) {  // 16-byte chunk c of k-row k at chunk position c ^ 2*(k % 4)
        const int k = q / 16, c = q % 16;
        *reinterpret_cast<u32x4*>(tile + k * ROW_BYTES + ((c ^ (2 * (k % 4))) * 16)) =
            *reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(in) + k * ROW_BYTES + c * 16);
    }
    __syncthreads();
    uint32_t part[4];
#pragma unroll
    for (int jl = 0; jl < 4; ++jl) part[jl] = wave::k_rows_lane_part<ROW_BYTES>(wv, jl, lane);
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const wave::v4s v = wave::read_k_rows_half<ROW_BYTES>(wv, tile, 0, j, 0, h, part);
            // lane (g = lane / 16, i = lane % 16): element 16 j + i, k = 8 g + 4 h + 0..3
            const int element = 16 * j + (lane & 15), k = 8 * (lane >> 4) + 4 * h;
#pragma unroll
            for (int e = 0; e < 4; ++e) out[element * 32 + k + e] = static_cast<uint16_t>(v[e]);
        }
}

}  // namespace
}  // namespace prism

extern "C" prism_status_t prism_layout_probe(int32_t what, const void* in0, const void* in1, void* out, void* hip_stream)
{
    using namespace prism;
    if (!in0 || !out || reinterpret_cast<uintptr_t>(in0) % 16 != 0 || reinterpret_cast<uintptr_t>(out) % 16 != 0) return PRISM_ERR_INVALID_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (what == PRISM_LAYOUT_ACCUMULATOR_BF16 || what == PRISM_LAYOUT_ACCUMULATOR_F16) {
        if (!in1 || reinterpret_cast<uintptr_t>(in1) % 16 != 0) return PRISM_ERR_INVALID_ARG;
        const char* r = static_cast<const char*>(in0);
        const char* c = static_cast<const char*>(in1);
        if (what == PRISM_LAYOUT_ACCUMULATOR_BF16)
            hipLaunchKernelGGL(probe_accumulator_layout<bf16_t>, dim3(1), dim3(64), 0, stream, r, c, static_cast<float*>(out));
        else
            hipLaunchKernelGGL(probe_accumulator_layout<f16_t>, dim3(1), dim3(64), 0, stream, r, c, static_cast<float*>(out));
    } else if (what == PRISM_LAYOUT_K_ROWS_READ) {
        hipLaunchKernelGGL(probe_k_rows_read, dim3(1), dim3(64), 0, stream, static_cast<const uint16_t*>(in0), static_cast<uint16_t*>(out));
    } else {
        return PRISM_ERR_UNSUPPORTED;
    }
    return hipGetLastError() == hipSuccess ? PRISM_OK : PRISM_ERR_LAUNCH;
}

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
