// MUST NOT COMPILE: a function whose bound is thread[64] (a whole wavefront) called from
// thread[32]: the call site's perspective is narrower than the callee requires (section 3.5).
// EXPECT: no known conversion from
#include "workgroup.hpp"
using namespace prism;
__device__ f32x4 needs_a_wave(persp::Threads<64> w, bf16x8 a, bf16x8 b, f32x4 acc) { return wave::mfma_block(w, a, b, acc); }
__device__ f32x4 half_wave(persp::Threads<32> h, bf16x8 a, bf16x8 b, f32x4 acc)
{
    return needs_a_wave(h, a, b, acc);
}
