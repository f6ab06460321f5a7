// MUST NOT COMPILE: inside one branch of a split workgroup (two of its four waves) the
// whole-workgroup barrier is out of reach.
// EXPECT: no viable conversion from
#include "workgroup.hpp"
using namespace prism;
__device__ void producers(persp::Threads<128> two_waves)
{
    wg::barrier(two_waves);
}
