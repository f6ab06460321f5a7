// Lane layer: what ONE lane of a wavefront does on its own.
//
// Every function here is written from the point of view of a single lane and
// receives that lane's index inside its wavefront (0..63) as an argument; it
// never looks at workgroup or grid coordinates.  This mirrors the paper's
// rule that a function is written at, and callable only at, one granularity
// (perspectives, section 3.2; the thread-level fragment loads of its
// `simple_mma` device function are the counterpart of load_fragment below).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "persp.hpp"

namespace prism {

using bf16x8 = __attribute__((ext_vector_type(8))) __bf16;
using f16x8 = __attribute__((ext_vector_type(8))) _Float16;
using f32x4 = __attribute__((ext_vector_type(4))) float;
using u32x4 = __attribute__((ext_vector_type(4))) uint32_t;
using u32x2 = __attribute__((ext_vector_type(2))) uint32_t;

struct bf16_t {};  // operand tags
struct f16_t {};
struct f32_t {};

// A fragment is one lane's 16 bytes of an operand row: 8 consecutive k of a 16-bit type,
// 4 consecutive k of fp32.
template <typename T> struct Frag;
template <> struct Frag<bf16_t> { using type = bf16x8; static constexpr int kElemBytes = 2; };
template <> struct Frag<f16_t> { using type = f16x8; static constexpr int kElemBytes = 2; };
template <> struct Frag<f32_t> { using type = f32x4; static constexpr int kElemBytes = 4; };

namespace lane {

// ---- LDS tile layout ---------------------------------------------------------
// An operand tile in LDS is `rows` x BK elements, K contiguous, made of
// 16-byte chunks (8 elements).  Chunk c of row r is kept at chunk position
// c ^ swizzle(r).  A 128-bit LDS read is served 16 lanes at a time; with
// swizzle(r) = r % 8 the 16 lanes of a fragment read (16 consecutive rows, one
// logical chunk) were measured free of bank conflicts (SQ_LDS_BANK_CONFLICT = 0),
// for every sub-step and row block of a slot.
constexpr int kChunkBytes = 16;

template <int BK>
struct TileLayout {
    static_assert(BK == 32 || BK == 64, "tile rows are 64 or 128 bytes");
    static constexpr int kTileK = BK;
    static constexpr int kRowBytes = BK * 2;
    static constexpr int kChunksPerRow = kRowBytes / kChunkBytes;
    __host__ __device__ static constexpr int swizzle(int row)
    {
        return BK == 64 ? (row & 7) : (((row >> 1) ^ (row >> 2)) & 3);
    }
    __host__ __device__ static constexpr int offset(int row, int chunk)
    {
        return row * kRowBytes + ((chunk ^ swizzle(row)) * kChunkBytes);
    }
};

// The matrix instruction works on blocks of kBlock rows by kBlockK k.
constexpr int kBlock = 16;
constexpr int kBlockK = 32;

// One lane's share of a 16-row x 32-k MFMA operand fragment: 8 consecutive k
// of row (row0 + lane%16), taken from k-chunk (4*ksub + lane/16) of the tile.
// Both operands use the same lane -> k assignment, which is all the matrix
// instruction needs for the k sum to pair the right elements.
template <typename T, int BK>
__device__ __forceinline__ typename Frag<T>::type
load_fragment(persp::Lane, const char* tile, int row0, int ksub, int lane)
{
    const int row = row0 + (lane & 15);
    const int chunk = 4 * ksub + (lane >> 4);
    const u32x4 raw = *reinterpret_cast<const u32x4*>(tile + TileLayout<BK>::offset(row, chunk));
    return __builtin_bit_cast(typename Frag<T>::type, raw);
}

// The same fragment with the address split into what depends on the lane only and what does
// not: for a block of 16 rows that starts at a multiple of 8 rows the swizzle of a lane's row
// is that of (lane % 16), so  offset(row0 + lane%16, chunk) = row0 * row bytes + lane part.
// Callers keep the lane part (one value per ksub) in a register and add uniform and constant
// terms, which then fold into the instruction's offset field.
template <int BK>
__device__ __forceinline__ uint32_t fragment_lane_part(persp::Lane, int ksub, int lane)
{
    return TileLayout<BK>::offset(lane & 15, 4 * ksub + (lane >> 4));
}
template <typename T>
__device__ __forceinline__ typename Frag<T>::type load_fragment_at(persp::Lane, const char* block_rows, uint32_t lane_part)
{
    const u32x4 raw = *reinterpret_cast<const u32x4*>(block_rows + lane_part);
    return __builtin_bit_cast(typename Frag<T>::type, raw);
}

// ---- accumulator layout of the 16x16 MFMA -----------------------------------------
// With the fragment of the "row" operand r and the "column" operand c,
// D = r * c^T is spread so that lane l holds column l%16 and, in register i
// (0..3), row 4*(l/16) + i.
__host__ __device__ constexpr int acc_row(int reg, int lane) { return 4 * (lane >> 4) + reg; }
__host__ __device__ constexpr int acc_col(int lane) { return lane & 15; }

// ---- pairing the columns of neighbouring blocks --------------------------------------
// A lane's four accumulators of a block are four consecutive columns; a 16-bit result wants
// eight per 16-byte store.  When the rows of the "row" operand's tile are dealt to LDS rows so
// that LDS row 32s + 16h + 4a + b holds tile row 32s + 8a + 4h + b (h in 0..1, a and b in 0..3),
// block column j = 2s + h hands lane l the columns 32s + 8(l/16) + 4h .. +3: the two blocks of
// a pair give every lane eight consecutive columns, and the four lanes that share a row 64
// contiguous bytes of a 16-bit result, straight from the accumulator registers.  The copies
// move whole 128-byte rows, so dealing the rows differently costs nothing.
__host__ __device__ constexpr int paired_tile_row(int lds_row)
{
    return (lds_row & ~31) | ((lds_row & 12) << 1) | ((lds_row & 16) >> 2) | (lds_row & 3);
}
// First of the four columns (relative to the wave tile) that lane `lane` holds of block column j.
template <bool PAIRED>
__host__ __device__ constexpr int acc_first_col(int j, int lane)
{
    return PAIRED ? 32 * (j >> 1) + 8 * (lane >> 4) + 4 * (j & 1) : kBlock * j + 4 * (lane >> 4);
}

// ---- output conversion ---------------------------------------------------------
__device__ __forceinline__ uint16_t to_bf16_bits(float x)
{
    return __builtin_bit_cast(uint16_t, static_cast<__bf16>(x));  // round to nearest even
}
__device__ __forceinline__ uint16_t to_f16_bits(float x)
{
    return __builtin_bit_cast(uint16_t, static_cast<_Float16>(x));  // round to nearest even
}
__device__ __forceinline__ float from_bf16_bits(uint16_t h)
{
    return __builtin_bit_cast(float, static_cast<uint32_t>(h) << 16);
}
__device__ __forceinline__ float from_f16_bits(uint16_t h)
{
    return static_cast<float>(__builtin_bit_cast(_Float16, h));
}

}  // namespace lane
}  // namespace prism
