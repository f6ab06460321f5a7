// Perspectives as compile-time tokens.
//
// The paper's language gives every piece of device code a perspective -- the group of
// threads that executes it together (thread, warp, block, grid; sections 3.1-3.2) -- and
// makes it a type error to call an operation from a perspective that cannot perform it:
// a warp-collective matrix instruction from per-thread code, a block barrier from a single
// warp (section 3.5).  Perspectives are erased before code generation (section 5).
//
// Here a perspective is an empty token object.  Holding a persp::Wave means "this code is
// executed by all 64 lanes of a wavefront, converged"; a function that needs that takes a
// persp::Wave parameter.  Tokens cannot be made from nothing: a kernel obtains the grid
// token at its entry and narrows it (grid -> workgroup -> wave -> lane, the paper's
// `group` going down); there is no way back up, so per-lane code, which only ever holds a
// persp::Lane, cannot reach a wave- or workgroup-collective operation.  The tokens are empty
// and every function that takes one is inlined, so they leave no trace in the machine code.
//
// What C++ cannot express and the paper's checker can: a token that is still in scope
// inside a divergent branch can be misused there.  The rule for this code base is that a
// branch on a per-lane condition only uses persp::Lane operations.
#pragma once

#include <hip/hip_runtime.h>

namespace prism {
namespace persp {

class Lane {
    friend class Wave;
    __device__ constexpr Lane() {}
};

class Wave {
    friend class Workgroup;
    template <int, int> friend class WaveGroup;
    __device__ constexpr Wave() {}

public:
    // every lane of a converged wave may run per-lane code
    __device__ constexpr Lane lane() const { return Lane(); }
};

// A group of COUNT consecutive waves out of a workgroup of TOTAL waves (the paper's `split`
// of a block into warp groups): only exists when the split is even, and only yields wave
// tokens -- a barrier over the whole workgroup is out of reach from inside one group.
template <int COUNT, int TOTAL>
class WaveGroup {
    friend class Workgroup;
    static_assert(COUNT > 0 && TOTAL % COUNT == 0, "a workgroup splits only into equal groups of waves");
    __device__ constexpr WaveGroup() {}

public:
    __device__ constexpr Wave wave() const { return Wave(); }
};

class Workgroup {
    friend class Grid;
    __device__ constexpr Workgroup() {}

public:
    __device__ constexpr Wave wave() const { return Wave(); }
    template <int COUNT, int TOTAL>
    __device__ constexpr WaveGroup<COUNT, TOTAL> split() const { return WaveGroup<COUNT, TOTAL>(); }
};

class Grid {
    __device__ constexpr Grid() {}

public:
    // Only the first statement of a __global__ function may call this: at kernel entry all
    // threads of the grid are present and converged.
    __device__ static constexpr Grid at_kernel_entry() { return Grid(); }
    __device__ constexpr Workgroup workgroup() const { return Workgroup(); }
};

}  // namespace persp
}  // namespace prism
