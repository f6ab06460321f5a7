// MUST NOT COMPILE: there is no way from a lane back up to its wave.
// EXPECT: no member named 'wave' in 'prism::persp::Threads<1>'
#include "workgroup.hpp"
using namespace prism;
__device__ void per_lane(persp::Lane l)
{
    persp::Wave w = l.wave();
    (void)w;
}
