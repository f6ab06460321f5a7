// MUST NOT COMPILE: a token made from nothing.
// EXPECT: private constructor
#include "workgroup.hpp"
using namespace prism;
__device__ f32x4 helper(bf16x8 a, bf16x8 b, f32x4 acc)
{
    persp::Wave w;
    return wave::mfma_block(w, a, b, acc);
}
