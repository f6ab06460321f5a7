// MUST NOT COMPILE: per-lane code reaches for the wave-collective matrix instruction.
// EXPECT: no matching function for call to 'mfma_block'
#include "workgroup.hpp"
using namespace prism;
__device__ f32x4 per_lane(persp::Lane l, bf16x8 a, bf16x8 b, f32x4 acc)
{
    return wave::mfma_block(l, a, b, acc);
}
