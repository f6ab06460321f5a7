// MUST NOT COMPILE: the paper's illegal split that asks for more units than there are
// (section 3.2, "Illegal split exceeds the available perspectives": thread[4] into 4 and 1).
// EXPECT: split: the branches must fit into the perspective side by side
#include "workgroup.hpp"
using namespace prism;
__device__ void four_threads(persp::Threads<4> t)
{
    const auto s = t.split<4, 1>();
    (void)s;
}
