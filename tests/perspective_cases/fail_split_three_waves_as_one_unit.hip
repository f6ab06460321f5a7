// MUST NOT COMPILE: one producer wave and the other three waves as ONE perspective: thread[192]
// is not a perspective a workgroup of 256 threads can be split into (192 does not divide 256;
// rule T-Split).  Three consumer waves are three branches of thread[64], see ok_split_waves.hip.
// EXPECT: split: the branches must fit into the perspective side by side
#include "workgroup.hpp"
using namespace prism;
__global__ void kernel()
{
    const persp::Workgroup wgp = persp::Grid::at_kernel_entry().workgroup();
    const auto s = wgp.destruct().split<64, 192>();
    (void)s;
}
