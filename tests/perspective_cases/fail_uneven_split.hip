// MUST NOT COMPILE: four waves do not split into groups of three.
// EXPECT: a workgroup splits only into equal groups of waves
#include "workgroup.hpp"
using namespace prism;
__global__ void kernel()
{
    const persp::Workgroup wgp = persp::Grid::at_kernel_entry().workgroup();
    const auto g = wgp.split<3, 4>();
    (void)g;
}
