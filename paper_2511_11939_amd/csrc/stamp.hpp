// Measurement aid: time stamps a kernel leaves for the host when it is given a place for them.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace prism {

// Time stamps of a stamped launch: workgroup g writes, at each of four points, the shader-clock
// counter and the constant 100 MHz counter into stamps[g * kStampWords + 2 * point ..].
constexpr int kStampWords = 8;
enum : int { STAMP_ENTRY = 0, STAMP_FIRST_FRAGMENTS = 1, STAMP_K_LOOP_DONE = 2, STAMP_STORES_DONE = 3 };
__device__ __forceinline__ void stamp(uint64_t* stamps, int point)
{
    if (stamps && threadIdx.x == 0) {
        uint64_t* slot = stamps + static_cast<size_t>(blockIdx.x) * kStampWords + 2 * point;
        slot[0] = __builtin_readcyclecounter();
        slot[1] = __builtin_amdgcn_s_memrealtime();
    }
}

}  // namespace prism
