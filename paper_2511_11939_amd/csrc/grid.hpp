// Grid layer: which workgroup computes which output tile, and what happens to a
// finished accumulator tile (scale, bias, conversion, store, or a split-K
// partial).  The scheduler plays the part of the tile loop with super-tile
// ordering in the paper's persistent hgemm kernel (code appendix, scheduler of
// `my_h100_match_no_tail`); the alpha/beta epilogue is the paper's sgemm
// epilogue (section 6.1) extended by a bias vector.
#pragma once

#include "lane.hpp"
#include "stamp.hpp"

namespace prism {

enum : int { DT_BF16 = 0, DT_F16 = 1, DT_F32 = 2 };

// Problem as the kernels see it: C is row-major (a column-major C has been
// turned into the transposed problem on the host), strides are in elements.
struct GemmParams {
    const char* A;        // element (m, k) at A + esize*(m*a_sm + k*a_sk), esize 2 or 4
    const char* B;        // element (k, n) at B + esize*(n*b_sn + k*b_sk)
    char* C;              // element (m, n) at C + esize*(m*ldc + n)
    const float* bias;    // or nullptr
    float* partial;       // split-K scratch [batch][split_k][M][N] fp32, or nullptr
    int64_t a_sm, a_sk, b_sn, b_sk, ldc;
    int64_t batch_a, batch_b, batch_c;
    int M, N, K;
    int batch, split_k, k_slice;   // k_slice: K extent of one slice, whole K steps
    int tiles_m, tiles_n;
    float alpha, beta;
    int c_dtype;          // DT_*
    int bias_along_m;     // 1 when the problem was transposed on the host
    int a_vec, b_vec;     // operand is K-contiguous with 16-byte aligned rows / chunks
    int c_vec;            // 4-element groups of C (and of the bias) are vector-aligned
    int p_vec;            // 4-element groups of the split-K scratch are 16-byte aligned
    int c_vec8;           // 8-element groups of C (and of the bias) start on 16-byte boundaries
    uint64_t* stamps;     // nullptr, or kStampWords uint64 per workgroup of the main kernel (measurement aid)
};

namespace grid {

constexpr int kDies = 8;        // accelerator dies (XCDs); workgroup ids are dealt round-robin
constexpr int kGroupRows = 4;   // tile rows per super-tile group

struct TileCoord {
    int tile_m, tile_n, unit;
};

// floor(x / d) for 0 <= x, 1 <= d, both below 2^30.  On the device both must be the same in
// every lane of the wave: the estimate from the reciprocal is moved to the scalar unit and
// corrected there, which replaces the compiler's general expansion (four quarter-rate
// integer multiplies per division, in front of a workgroup's first copies) by a handful of
// full-rate instructions.  The correction loops make the result exact whatever the error of
// the estimate, so host and device agree.
__host__ __device__ inline int uniform_quotient(int x, int d)
{
#if defined(__HIP_DEVICE_COMPILE__)
    int q = __builtin_amdgcn_readfirstlane(static_cast<int>(static_cast<float>(x) * __builtin_amdgcn_rcpf(static_cast<float>(d))));
    int rest = x - q * d;
    while (rest < 0) { --q; rest += d; }
    while (rest >= d) { ++q; rest -= d; }
    return __builtin_amdgcn_readfirstlane(q);  // stays on the scalar unit, and so does what is derived from it
#else
    return x / d;
#endif
}

// Position r in the locality order -> tile: groups of kGroupRows tile rows, m fastest, so that
// a contiguous run of positions is a compact block sharing few A and B panels.
__host__ __device__ inline void tile_at(int r, int tiles_m, int tiles_n, int& tile_m, int& tile_n)
{
    const int group_span = kGroupRows * tiles_n;
    const int group = uniform_quotient(r, group_span);
    const int first_m = group * kGroupRows;
    const int rows = tiles_m - first_m < kGroupRows ? tiles_m - first_m : kGroupRows;
    const int in_group = r - group * group_span;
    tile_n = uniform_quotient(in_group, rows);
    tile_m = first_m + in_group - tile_n * rows;
}

// The share of die `die` when `total` positions are dealt to the dies as contiguous runs
// (the first `total % kDies` dies take one more): first position and count.
__host__ __device__ inline void die_run(int die, int total, int& first, int& count)
{
    const int per = (total + kDies - 1) / kDies;
    int tall = total % kDies;
    if (tall == 0) tall = kDies;
    first = die < tall ? die * per : tall * per + (die - tall) * (per - 1);
    count = die < tall ? per : per - 1;
}

// Workgroup id -> (tile, unit).  Step 1 undoes the round-robin dealing so that
// the workgroups resident on one die form a contiguous run of a tile order;
// step 2 walks the tiles in groups of kGroupRows tile rows, m fastest, so that
// such a run is a compact block sharing few A and B panels in that die's L2.
// On the device `wg` must be uniform over the wave (a workgroup id is).
__host__ __device__ inline TileCoord schedule(int wg, int tiles_m, int tiles_n, int units)
{
    const int tiles = tiles_m * tiles_n;
    int first, count;
    die_run(wg % kDies, tiles * units, first, count);
    const int q = first + wg / kDies;
    TileCoord t;
    t.unit = units == 1 ? 0 : uniform_quotient(q, tiles);
    tile_at(q - t.unit * tiles, tiles_m, tiles_n, t.tile_m, t.tile_n);
    return t;
}

// ---- epilogue ------------------------------------------------------------------------
// Four accumulators of one lane: output row m, columns n0..n0+3.
template <int OUT>  // DT_BF16 / DT_F16 / DT_F32
__device__ __forceinline__ void finish4(const GemmParams& p, char* c_problem, int m, int n0, f32x4 v)
{
    if (m >= p.M || n0 >= p.N) return;
    constexpr int esize = OUT == DT_F32 ? 4 : 2;
    char* dst = c_problem + (static_cast<int64_t>(m) * p.ldc + n0) * esize;
    const bool full = p.c_vec && (n0 + 3 < p.N);
    float bias[4] = {0.f, 0.f, 0.f, 0.f};
    if (p.bias) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
            bias[q] = p.bias_along_m ? p.bias[m] : (n0 + q < p.N ? p.bias[n0 + q] : 0.f);
    }
    float out[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) out[q] = p.alpha * v[q] + bias[q];
    if (p.beta != 0.0f) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (n0 + q < p.N) {
                float old;
                if constexpr (OUT == DT_F32) old = reinterpret_cast<const float*>(dst)[q];
                else if constexpr (OUT == DT_BF16) old = lane::from_bf16_bits(reinterpret_cast<const uint16_t*>(dst)[q]);
                else old = lane::from_f16_bits(reinterpret_cast<const uint16_t*>(dst)[q]);
                out[q] += p.beta * old;
            }
        }
    }
    if constexpr (OUT == DT_F32) {
        if (full) {
            *reinterpret_cast<f32x4*>(dst) = f32x4{out[0], out[1], out[2], out[3]};
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (n0 + q < p.N) reinterpret_cast<float*>(dst)[q] = out[q];
        }
    } else {
        uint16_t h[4];
#pragma unroll
        for (int q = 0; q < 4; ++q)
            h[q] = OUT == DT_BF16 ? lane::to_bf16_bits(out[q]) : lane::to_f16_bits(out[q]);
        if (full) {
            *reinterpret_cast<u32x2*>(dst) = u32x2{static_cast<uint32_t>(h[0]) | (static_cast<uint32_t>(h[1]) << 16),
                                                  static_cast<uint32_t>(h[2]) | (static_cast<uint32_t>(h[3]) << 16)};
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (n0 + q < p.N) reinterpret_cast<uint16_t*>(dst)[q] = h[q];
        }
    }
}

// finish4 for the output type named in the descriptor.
__device__ __forceinline__ void finish4_any(const GemmParams& p, char* c_problem, int m, int n0, f32x4 v)
{
    if (p.c_dtype == DT_BF16) finish4<DT_BF16>(p, c_problem, m, n0, v);
    else if (p.c_dtype == DT_F16) finish4<DT_F16>(p, c_problem, m, n0, v);
    else finish4<DT_F32>(p, c_problem, m, n0, v);
}

// Eight consecutive results of one row, no bounds to check and no beta term:
// scale, add the (pre-loaded) bias, convert, store as one or two 16-byte pieces.
// With alpha == 1 and a zero bias the arithmetic is exact, so there is no
// separate path for a plain product.
template <int OUT, bool BIAS>
__device__ __forceinline__ void finish_run(char* dst, float alpha, const float (&bias)[8], f32x4 lo, f32x4 hi)
{
    float o[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
#pragma unroll
    for (int q = 0; q < 8; ++q) o[q] = BIAS ? alpha * o[q] + bias[q] : alpha * o[q];
    if constexpr (OUT == DT_F32) {
        reinterpret_cast<f32x4*>(dst)[0] = f32x4{o[0], o[1], o[2], o[3]};
        reinterpret_cast<f32x4*>(dst)[1] = f32x4{o[4], o[5], o[6], o[7]};
    } else {
        uint32_t w[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t a = OUT == DT_BF16 ? lane::to_bf16_bits(o[2 * q]) : lane::to_f16_bits(o[2 * q]);
            const uint32_t b = OUT == DT_BF16 ? lane::to_bf16_bits(o[2 * q + 1]) : lane::to_f16_bits(o[2 * q + 1]);
            w[q] = a | (b << 16);
        }
        *reinterpret_cast<u32x4*>(dst) = u32x4{w[0], w[1], w[2], w[3]};
    }
}

// The same eight results as the 16 bytes of a 16-bit output type, not yet stored.
template <int OUT, bool BIAS>
__device__ __forceinline__ u32x4 pack_run(float alpha, const float (&bias)[8], f32x4 lo, f32x4 hi)
{
    static_assert(OUT == DT_BF16 || OUT == DT_F16, "16-bit output types");
    float o[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    uint32_t w[4];
#pragma unroll
    for (int q = 0; q < 8; ++q) o[q] = BIAS ? alpha * o[q] + bias[q] : alpha * o[q];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint32_t a = OUT == DT_BF16 ? lane::to_bf16_bits(o[2 * q]) : lane::to_f16_bits(o[2 * q]);
        const uint32_t b = OUT == DT_BF16 ? lane::to_bf16_bits(o[2 * q + 1]) : lane::to_f16_bits(o[2 * q + 1]);
        w[q] = a | (b << 16);
    }
    return u32x4{w[0], w[1], w[2], w[3]};
}

// Raw fp32 partial sums of one K slice.
__device__ __forceinline__ void partial4(const GemmParams& p, float* slab, int m, int n0, f32x4 v)
{
    if (m >= p.M || n0 >= p.N) return;
    float* dst = slab + static_cast<int64_t>(m) * p.N + n0;
    if (p.p_vec && (n0 + 3 < p.N)) {
        *reinterpret_cast<f32x4*>(dst) = v;
    } else {
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (n0 + q < p.N) dst[q] = v[q];
    }
}

}  // namespace grid
}  // namespace prism
