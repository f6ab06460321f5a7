// Host-visible launchers of the device kernels (defined in kernels.hip).
#pragma once

#include <hip/hip_runtime.h>

#include "grid.hpp"

namespace prism {

// Workgroup-tile configurations of the direct-to-LDS pipeline.
struct PipeConfig {
    int id;
    int tile_m, tile_n, tile_k, waves, stages;
    const char* name;
};
constexpr int kNumPipeConfigs = 9;  // 0, 1: both operands K-contiguous; 2-4: B along n, A along m, both; 5-8: fp32, same four
extern const PipeConfig kPipeConfigs[kNumPipeConfigs];

constexpr int kStagedTileM = 128, kStagedTileN = 128, kStagedWaves = 4;

// Each returns the launch error of the HIP runtime (hipSuccess when accepted).
// `workgroups` = p.tiles_m * p.tiles_n * p.batch * p.split_k.
hipError_t launch_pipelined(int config, int ab_dtype, const GemmParams& p, int workgroups, hipStream_t stream);
hipError_t launch_staged(int ab_dtype, const GemmParams& p, int workgroups, hipStream_t stream);
// 256x256x64 tile, `workgroups` persistent workgroups walking `total` (tile, unit) pairs;
// every unit must span at least two K steps of 64.
hipError_t launch_persistent(int ab_dtype, const GemmParams& p, int total, int workgroups, hipStream_t stream);
// Sums the split_k partial slabs in slice order and applies the epilogue; with
// p.split_k == 0 it writes C <- bias + beta*C (the K == 0 case).
hipError_t launch_reduce(const GemmParams& p, hipStream_t stream);

// The scan's own hook (PRISM_SCAN_SPIN_LIMIT), read again from the environment.
void scan_reread_environment();

}  // namespace prism
