// MUST NOT COMPILE: the paper's first illegal group (section 3.2, "Illegal uses of group"):
// from thread[2] there is no way to a block.
// EXPECT: no member named 'workgroup' in 'prism::persp::Threads<2>'
#include "workgroup.hpp"
using namespace prism;
__device__ void two_threads(persp::Threads<2> t)
{
    const auto b = t.workgroup();
    (void)b;
}
