// MUST NOT COMPILE: the paper's illegal split whose second branch is not aligned to its size
// (section 3.2, "Illegal split violates alignment": thread[3] into 1 and 2; rule T-Split).
// EXPECT: split: the branches must fit into the perspective side by side
#include "workgroup.hpp"
using namespace prism;
__device__ void three_threads(persp::Threads<3> t)
{
    const auto s = t.split<1, 2>();
    (void)s;
}
