// MUST NOT COMPILE: thread[96] is broader than thread[64] in count but not in the paper's order
// (64 does not divide 96, so the 96 threads are not made of whole aligned wavefronts).
// EXPECT: no known conversion from
#include "workgroup.hpp"
using namespace prism;
__device__ void needs_a_wave(persp::Wave) {}
__device__ void ninety_six(persp::Threads<96> t)
{
    needs_a_wave(t);
}
