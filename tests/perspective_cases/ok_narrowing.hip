// MUST COMPILE: a kernel takes the grid token at entry and narrows it step by step.
#include "workgroup.hpp"
using namespace prism;
__device__ float per_lane(persp::Lane, float x) { return x + 1.0f; }
__device__ f32x4 per_wave(persp::Wave w, bf16x8 a, bf16x8 b, f32x4 acc)
{
    acc = wave::mfma_block(w, a, b, acc);          // wave-collective: allowed with a wave token
    acc[0] = per_lane(w.lane(), acc[0]);           // narrowing to one lane is always allowed
    return acc;
}
__global__ void kernel(float* out)
{
    const persp::Workgroup wgp = persp::Grid::at_kernel_entry().workgroup();
    const persp::Wave w = wgp.wave();
    const persp::Threads<128> pair = wgp.destruct().group<128>();   // two of the four waves
    f32x4 acc = per_wave(pair.group<64>(), bf16x8{}, bf16x8{}, f32x4{0, 0, 0, 0});
    acc = per_wave(w, bf16x8{}, bf16x8{}, acc);
    wg::barrier(wgp);                              // workgroup-collective: allowed with the workgroup token
    out[threadIdx.x] = acc[0];
}
