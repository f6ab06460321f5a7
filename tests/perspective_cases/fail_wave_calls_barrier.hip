// MUST NOT COMPILE: code that only knows it is run by one wave asks for a workgroup barrier.
// EXPECT: no viable conversion from
#include "workgroup.hpp"
using namespace prism;
__device__ void per_wave(persp::Wave w)
{
    wg::barrier(w);
}
