// MUST NOT COMPILE: inside one group of a split workgroup the whole-workgroup barrier is out of reach.
// EXPECT: no viable conversion from
#include "workgroup.hpp"
using namespace prism;
__device__ void producer(persp::WaveGroup<1, 4> g)
{
    wg::barrier(g);
}
