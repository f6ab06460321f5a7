// MUST COMPILE: legal splits and call sites.
#include "workgroup.hpp"
using namespace prism;
__device__ float per_lane(persp::Lane, float x) { return x + 1.0f; }
__device__ f32x4 per_wave(persp::Wave w, bf16x8 a, bf16x8 b, f32x4 acc)
{
    acc = wave::mfma_block(w, a, b, acc);
    acc[0] = per_lane(w, acc[0]);                  // thread[64] where thread[1] is required: broader, fine
    return acc;
}
// the paper's example split (section 3.2): thread[4] into branches of 2, 1 and 1
__device__ int example(persp::Threads<4> t, int index)
{
    const auto s = t.split<2, 1, 1>();
    static_assert(decltype(s)::offset<0>() == 0 && decltype(s)::offset<1>() == 2 && decltype(s)::offset<2>() == 3, "branch offsets");
    const persp::Threads<2> pair = s.branch<0>();
    const persp::Lane single = s.branch<1>();
    (void)pair; (void)single;
    return decltype(s)::holds<0>(index) ? 0 : (decltype(s)::holds<1>(index) ? 1 : 2);
}
__global__ void kernel(float* out)
{
    const persp::Workgroup wgp = persp::Grid::at_kernel_entry().workgroup();
    // warp specialisation on four wavefronts: one producer wave and three consumer waves, each its own branch
    const auto roles = wgp.destruct().split<64, 64, 64, 64>();
    const int thread = threadIdx.x;
    f32x4 acc = {0, 0, 0, 0};
    if (decltype(roles)::holds<0>(thread)) acc = per_wave(roles.branch<0>(), bf16x8{}, bf16x8{}, acc);   // producer
    else acc = per_wave(roles.branch<1>(), bf16x8{}, bf16x8{}, acc);                                       // a consumer
    // two groups of two waves (the paper's `group`): thread[128] twice, each made of two wavefronts
    const persp::Threads<128> half = wgp.destruct().group<128>();
    acc = per_wave(half, bf16x8{}, bf16x8{}, acc);   // called with a broader perspective: both waves run it
    acc = per_wave(wgp, bf16x8{}, bf16x8{}, acc);    // and from block level: all four
    // the smallest binary split rule T-Split allows here: 64 and 64 out of 256 (64 | 64 + 256)
    const auto two = wgp.destruct().split<64, 64>();
    (void)two;
    wg::barrier(wgp);
    out[thread] = acc[0];
}
