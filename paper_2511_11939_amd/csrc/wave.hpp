// Wave layer: operations that all 64 lanes of one wavefront issue together.
//
// The matrix-core instruction is the gfx950 counterpart of the warp-collective
// `mma.sync` / warpgroup-collective `wgmma` the paper builds its kernels on
// (sections 2.3 and 6.2): it only means something when a whole, aligned group
// of lanes executes it, so these functions must be called with the complete
// wavefront converged: each takes a persp::Wave token, which per-lane code cannot obtain.
#pragma once

#include "lane.hpp"

namespace prism {
namespace wave {

// D[i][j] += sum_k R[i][k] * C[j][k]  for a 16 x 16 block and the k range of one fragment
// pair (32 k of a 16-bit type, 16 k of fp32).
// `r` / `c`: each lane's 8 consecutive k of row (lane%16), k-quarter (lane/16).
// Result layout: see lane::acc_row / lane::acc_col.  Of the two bf16 shapes of
// gfx950 (16x16x32 and 32x32x16) this one reads and writes a quarter of the
// accumulator registers per instruction for the same multiply-adds; the whole
// GEMM kernel was measured about 7 % faster with it.
__device__ __forceinline__ f32x4 mfma_block(persp::Wave, bf16x8 r, bf16x8 c, f32x4 acc)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(r, c, acc, 0, 0, 0);
}
__device__ __forceinline__ f32x4 mfma_block(persp::Wave, f16x8 r, f16x8 c, f32x4 acc)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(r, c, acc, 0, 0, 0);
}

// fp32 operands: a fragment holds 4 consecutive k per lane; MFMA e of the four takes element
// e of both fragments, so lane group g (lane/16) contributes k = 4g + e to it.
__device__ __forceinline__ f32x4 mfma_block(persp::Wave, f32x4 r, f32x4 c, f32x4 acc)
{
#pragma unroll
    for (int e = 0; e < 4; ++e) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(r[e], c[e], acc, 0, 0, 0);
    return acc;
}

// One matrix instruction of a block: for 16-bit operands the whole block (part 0 of 1), for
// fp32 the e-th of its four.  Issuing the same e for all blocks before the next e keeps
// consecutive instructions independent of each other.
constexpr int mfma_parts(bf16x8) { return 1; }
constexpr int mfma_parts(f16x8) { return 1; }
constexpr int mfma_parts(f32x4) { return 4; }
__device__ __forceinline__ f32x4 mfma_part(persp::Wave w, bf16x8 r, bf16x8 c, int, f32x4 acc) { return mfma_block(w, r, c, acc); }
__device__ __forceinline__ f32x4 mfma_part(persp::Wave w, f16x8 r, f16x8 c, int, f32x4 acc) { return mfma_block(w, r, c, acc); }
__device__ __forceinline__ f32x4 mfma_part(persp::Wave, f32x4 r, f32x4 c, int e, f32x4 acc)
{
    return __builtin_amdgcn_mfma_f32_16x16x4f32(r[e], c[e], acc, 0, 0, 0);
}

// Register-blocked wave tile: MT x NT accumulator blocks of 16 x 16.  The B
// fragment is the MFMA's row operand, so every lane ends up holding runs of
// four consecutive n for one m, which is what a row-major store wants.
template <typename T, int MT, int NT>
struct Tile {
    using frag_t = typename Frag<T>::type;
    f32x4 acc[MT][NT];

    __device__ __forceinline__ void clear()
    {
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < NT; ++j) acc[i][j] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    }

    // one 32-wide k sub-step over the whole wave tile
    __device__ __forceinline__ void mma(persp::Wave w, const frag_t (&a)[MT], const frag_t (&b)[NT])
    {
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < NT; ++j) acc[i][j] = mfma_block(w, b[j], a[i], acc[i][j]);
    }
};

// Fragments of one k sub-step for a wave tile whose first row in the LDS tile
// is row0: MT (or NT) blocks of 16 rows.
template <typename T, int BK, int NBLK>
__device__ __forceinline__ void load_fragments(persp::Wave w, typename Frag<T>::type (&f)[NBLK], const char* tile,
                                               int row0, int ksub, int lane)
{
#pragma unroll
    for (int i = 0; i < NBLK; ++i) f[i] = lane::load_fragment<T, BK>(w.lane(), tile, row0 + lane::kBlock * i, ksub, lane);
}

}  // namespace wave
}  // namespace prism
