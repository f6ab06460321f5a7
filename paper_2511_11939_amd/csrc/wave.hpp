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

// ---- fragments of a 16-bit operand that lies in LDS as k-rows ----------------------------
// An operand that is contiguous along its other index (a row-major B, a column-major A) is
// kept in LDS as k-rows of ROW_BYTES bytes: k-row k holds the elements of all n (or m) for that
// k, its 16-byte chunk c at chunk position c ^ 2*(k % 4).  The matrix instruction wants, per
// lane, consecutive k of ONE element; the transposing LDS read of gfx950 delivers that: the 16
// lanes of a group each supply the address of 4 consecutive 16-bit elements, and lane i of the
// group receives element i % 4 of the four suppliers i/4, i/4 + 4, i/4 + 8, i/4 + 12.  With
// supplier i pointing at k-row i/4, element quad i%4 of a block of 16 elements, lane i receives
// four consecutive k of element i of the block.  A fragment (8 consecutive k) is two such reads.
//
// k_rows_lane_part: the per-lane share of the read address for the jl-th (0..3) block of 16
// elements inside a group of 64 elements (the swizzle stays inside 8 chunks, so four values
// serve all reads of a wave).  Lane group g = lane/16 reads k-rows 8g .. 8g+3 (+4 for the other half).
using v4s = __attribute__((ext_vector_type(4))) short;
template <int ROW_BYTES>
__device__ __forceinline__ uint32_t k_rows_lane_part(persp::Wave, int jl, int lane)
{
    const int i = lane & 15, kq = lane >> 4, s_row = i >> 2, x = (i & 3) >> 1;
    return (8 * kq + s_row) * ROW_BYTES + (((2 * jl + x) ^ (s_row << 1)) * lane::kChunkBytes) + (i & 1) * 8;
}
// Half h (k = 8*(lane/16) + 4h .. +3 of sub-step ksub) of the fragment of the j-th block of 16
// elements counted from element `first` (a multiple of 64) of the k-rows at `tile`.
template <int ROW_BYTES>
__device__ __forceinline__ v4s read_k_rows_half(persp::Wave, const char* tile, int first, int j, int ksub, int h,
                                                const uint32_t (&lane_part)[4])
{
    const char* src = tile + ((first >> 3) + 8 * (j / 4)) * lane::kChunkBytes + (32 * ksub + 4 * h) * ROW_BYTES + lane_part[j % 4];
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)src);
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
