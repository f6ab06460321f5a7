// MUST NOT COMPILE: the paper's second illegal group (section 3.2, "Illegal uses of group"):
// block[5] cannot be replicated evenly over block[6] (rule T-Group).
// EXPECT: group: a narrower perspective replicates evenly only when its size divides the current one
#include "workgroup.hpp"
using namespace prism;
__global__ void kernel()
{
    const auto six = persp::Grid::at_kernel_entry().blocks<6>();
    const auto five = six.group<5>();
    (void)five;
}
