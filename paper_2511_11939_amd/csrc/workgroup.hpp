// Workgroup layer: everything the wavefronts of one workgroup do together --
// moving operand tiles from global memory into LDS, the barriers that order
// those moves against the fragment reads, and the K loop around the wave
// tiles.  Functions take the calling wave's index inside the workgroup and the
// lane's index inside the wave; they never look at grid coordinates.
//
// The structure follows what the paper says a peak-rate matrix multiply needs
// (section 6.2): data movement pipelined under the matrix instructions with
// statically sized, individually synchronised pipeline slots.  On gfx950 the
// asynchronous copy is the direct global->LDS load and the slot hand-over is
// one workgroup barrier per K step, placed by hand where the paper's compiler
// would insert it (section 5, synchronisation at loop back-edges).
#pragma once

#include <type_traits>

#include "lane.hpp"
#include "stamp.hpp"
#include "wave.hpp"

namespace prism {
namespace wg {

// s_waitcnt immediate for gfx9-family encodings: at most `vm` vector-memory and
// `lgkm` LDS/scalar operations of this wave may still be outstanding.
constexpr int waitcnt_imm(int vm, int lgkm)
{
    return (vm & 15) | ((vm >> 4) << 14) | (7 << 4) | ((lgkm & 15) << 8);
}
template <int VM, int LGKM>
__device__ __forceinline__ void wait_counts()
{
    static_assert(VM >= 0 && VM <= 63 && LGKM >= 0 && LGKM <= 15, "counter out of range");
    __builtin_amdgcn_s_waitcnt(waitcnt_imm(VM, LGKM));
}

__device__ __forceinline__ uint32_t lds_address(const void* p)
{
    return static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
        (const __attribute__((address_space(3))) char*)p));
}

// Asynchronous 16-bytes-per-lane copy global -> LDS for one wavefront: lane l
// reads 16 bytes at (uniform_base + lane_offset) and the hardware deposits them
// at lds_addr + 16*l.  The wave's vector-memory counter tracks completion.
__device__ __forceinline__ const char* scalarize(const char* p)
{
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v));
    const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v >> 32));
    return reinterpret_cast<const char*>((static_cast<uint64_t>(hi) << 32) | lo);
}

// Workgroup barrier: only code that holds the workgroup token -- code every wave of the
// workgroup executes -- can reach it (the paper's block-level synchronisation, section 3.5).
__device__ __forceinline__ void barrier(persp::Workgroup) { __builtin_amdgcn_s_barrier(); }
// Barrier that also waits for the caller's outstanding LDS and memory operations.
__device__ __forceinline__ void sync(persp::Workgroup) { __syncthreads(); }

// Race check by construction: built with PRISM_PARANOID_BARRIERS, every phase of a main loop
// that touches LDS ends with a full workgroup barrier (all of the wave's memory operations
// waited for first).  The hand-placed waits and the one barrier per K step are meant to be
// sufficient, so the results of that build must be bit-identical to the normal one's.
#ifdef PRISM_PARANOID_BARRIERS
#define PRISM_PARANOID_SYNC(wgp) ::prism::wg::sync(wgp)
#else
#define PRISM_PARANOID_SYNC(wgp) do { } while (0)
#endif

// One wave-wide copy of 64 x 16 bytes from global memory straight into LDS: lane l's bytes
// land at lds_base + lds_offset + 16*l.  Wave-level: base and LDS address are per-wave
// values; lds_offset must be a compile-time constant at the point of use, so that a copy
// costs two instructions (the LDS address goes to M0 with one scalar add).
__device__ __forceinline__ void copy_async_16(persp::Wave, const char* uniform_base, uint32_t lane_offset,
                                              uint32_t lds_base, int lds_offset)
{
    uniform_base = scalarize(uniform_base);  // no-ops when the values already live in SGPRs
    lds_base = __builtin_amdgcn_readfirstlane(lds_base);
    asm volatile("s_add_u32 m0, %2, %3\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(lane_offset), "s"(uniform_base), "s"(lds_base), "i"(lds_offset)
                 : "memory", "scc");
}

// Drains one wave's accumulator tile through a private LDS patch so that the
// values leave the wave as runs of four consecutive n, whole rows at a time
// (the MFMA leaves each lane with values of 16 different rows).  `patch` must
// hold kDrainRows x (16*NT + 4) floats, is used by this wave only, and must
// not be in use by anybody else (barrier before the first call).
// sink(row_in_wave_tile, col_in_wave_tile, f32x4) receives every group once.
// This is the general path (any bounds, any alignment); see drain_runs below.
constexpr int kDrainRows = 32;  // two 16-row blocks per pass
constexpr int drain_patch_bytes(int nt) { return kDrainRows * (lane::kBlock * nt + 4) * 4; }

// ROWS: rows per pass (32 = two blocks, 16 = one); PAD: floats of row padding (4 keeps the
// accesses free of bank conflicts, 0 fits 16 rows of a 128-wide tile into 8 KiB).
template <int MT, int NT, int ROWS = kDrainRows, int PAD = 4, bool PAIRED = false, typename TileT, typename Sink>
__device__ __forceinline__ void drain(persp::Wave, const TileT& acc, char* patch, int lane, Sink&& sink)
{
    static_assert(ROWS == 16 || (ROWS == 32 && MT % 2 == 0), "a pass takes one or two 16-row blocks");
    constexpr int BLOCKS = ROWS / lane::kBlock;
    constexpr int WTN = lane::kBlock * NT;
    constexpr int PITCH = WTN + PAD;  // floats
    constexpr int LANES_PER_ROW = WTN / 4;
    constexpr int ROWS_PER_ITER = 64 / LANES_PER_ROW > 0 ? 64 / LANES_PER_ROW : 1;
    constexpr int ITERS = ROWS / ROWS_PER_ITER;
    static_assert(LANES_PER_ROW <= 64, "one row per wave pass at most");
    float* buf = reinterpret_cast<float*>(patch);
#pragma unroll
    for (int pass = 0; pass < MT / BLOCKS; ++pass) {
#pragma unroll
        for (int ii = 0; ii < BLOCKS; ++ii) {
            float* wr = buf + (lane::kBlock * ii + lane::acc_col(lane)) * PITCH;
#pragma unroll
            for (int j = 0; j < NT; ++j)
                *reinterpret_cast<f32x4*>(wr + lane::acc_first_col<PAIRED>(j, lane)) = acc.acc[BLOCKS * pass + ii][j];
        }
        const int col = 4 * (lane % LANES_PER_ROW);
#pragma unroll 4
        for (int it = 0; it < ITERS; ++it) {
            const int row = it * ROWS_PER_ITER + lane / LANES_PER_ROW;
            const f32x4 v = *reinterpret_cast<const f32x4*>(buf + row * PITCH + col);
            sink(ROWS * pass + row, col, v);
        }
    }
}

// Fast drain for a wave tile that lies wholly inside C: the accumulators go to
// the patch as they are (straight from the accumulator registers), come back as
// runs of eight consecutive n per lane, and sink(row_uniform, row_lane, v_lo, v_hi)
// finishes and stores each run: row row_uniform + row_lane of the wave tile (the
// first part is the same for all lanes), columns 8*(lane % (2*NT)) .. +7.
// Inside a patch row the 16-byte units are stored evens first, odds second, so
// that both the writes and the two reads of a run are spread over all banks.
template <int MT, int NT, typename TileT, typename Sink>
__device__ __forceinline__ void drain_runs(persp::Wave, const TileT& acc, char* patch, int lane, Sink&& sink)
{
    static_assert(MT % 2 == 0, "a pass takes two 16-row blocks");
    constexpr int WTN = lane::kBlock * NT;
    constexpr int UNITS = WTN / 4;            // 16-byte units per row
    constexpr int PITCH = (WTN + 4) * 4;      // bytes
    constexpr int LANES_PER_ROW = WTN / 8;
    constexpr int ROWS_PER_ITER = 64 / LANES_PER_ROW;
    constexpr int ITERS = kDrainRows / ROWS_PER_ITER;
    // unit u of a row sits at position (u >> 1) + (UNITS / 2) * (u & 1)
    const int run = lane % LANES_PER_ROW, sub = lane / LANES_PER_ROW;
    // this lane's accumulators of block column j are unit 4j + lane/16 of their row
    const int q = lane >> 4;
    const int wr_lane = lane::acc_col(lane) * PITCH + 16 * ((q >> 1) + (UNITS / 2) * (q & 1));
#pragma unroll
    for (int pass = 0; pass < MT / 2; ++pass) {
#pragma unroll
        for (int ii = 0; ii < 2; ++ii)
#pragma unroll
            for (int j = 0; j < NT; ++j)
                *reinterpret_cast<f32x4*>(patch + wr_lane + lane::kBlock * ii * PITCH + 32 * j) = acc.acc[2 * pass + ii][j];
        f32x4 lo[ITERS], hi[ITERS];
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const char* rd = patch + (it * ROWS_PER_ITER + sub) * PITCH;
            lo[it] = *reinterpret_cast<const f32x4*>(rd + 16 * run);                 // unit 2*run   -> position run
            hi[it] = *reinterpret_cast<const f32x4*>(rd + 16 * (run + UNITS / 2));   // unit 2*run+1 -> position run + UNITS/2
        }
#pragma unroll
        for (int it = 0; it < ITERS; ++it) sink(kDrainRows * pass + it * ROWS_PER_ITER, sub, lo[it], hi[it]);
        __builtin_amdgcn_sched_barrier(0);  // one pass at a time keeps the register need small
    }
}

// Drain without LDS for a wave tile whose block columns are paired (lane::paired_tile_row):
// every lane already holds runs of eight consecutive n.  sink(row_uniform, col_uniform, lo, hi)
// receives the run of row row_uniform + lane % 16, columns col_uniform + 8 * (lane / 16) .. +7
// of the wave tile, once for every block row and pair of block columns.
template <int MT, int NT, typename TileT, typename Sink>
__device__ __forceinline__ void drain_pairs(persp::Wave, const TileT& acc, Sink&& sink)
{
    static_assert(NT % 2 == 0, "block columns come in pairs");
#pragma unroll
    for (int i = 0; i < MT; ++i) {
#pragma unroll
        for (int s = 0; s < NT / 2; ++s) {
            // (taken from the accumulation registers here and no earlier: without this the moves
            // of all blocks drift to the top of the epilogue and spill)
            f32x4 lo = acc.acc[i][2 * s], hi = acc.acc[i][2 * s + 1];
            asm volatile("" : "+a"(lo), "+a"(hi));
            sink(lane::kBlock * i, 32 * s, lo, hi);
        }
        __builtin_amdgcn_sched_barrier(0);  // one block row at a time keeps the register need small
    }
}

// Drain for a 16-bit result of a wave tile with paired block columns.  Every lane finishes its
// runs of eight consecutive n itself: pack(row_uniform, col_uniform, lo, hi) returns the 16
// bytes of the run of row row_uniform + lane % 16, columns col_uniform + 8 * (lane / 16) .. +7.
// The pieces of one block row (16 rows of 32 * NT bytes) pass through the wave's LDS patch and
// come back row by row, so that store(row_uniform, row_lane, byte_in_row, piece) writes whole
// rows of the wave tile (16 consecutive lanes hold 256 contiguous bytes).  Four times less LDS
// traffic than draining the fp32 accumulators, and full cache lines per store instruction.
// `patch` is this wave's, kRowsPatchBytes(NT) long; the padding of 16 bytes per row spreads
// both the writes (16 rows, one piece each) and the reads over all banks.
constexpr int rows_patch_bytes(int nt) { return lane::kBlock * (2 * lane::kBlock * nt + 16); }
template <int MT, int NT, typename TileT, typename Pack, typename Store>
__device__ __forceinline__ void drain_rows(persp::Wave, const TileT& acc, char* patch, int lane, Pack&& pack, Store&& store)
{
    static_assert(NT % 2 == 0, "block columns come in pairs");
    constexpr int ROW_BYTES = 2 * lane::kBlock * NT, PITCH = ROW_BYTES + 16;
    constexpr int PIECES = ROW_BYTES / 16;        // lanes that share a row on the way out
    constexpr int ROWS_PER_ITER = 64 / PIECES, ITERS = lane::kBlock / ROWS_PER_ITER;
    char* wr = patch + (lane & 15) * PITCH + 16 * (lane >> 4);
    const int piece = lane % PIECES, sub = lane / PIECES;
    const char* rd = patch + sub * PITCH + 16 * piece;
#pragma unroll
    for (int i = 0; i < MT; ++i) {
#pragma unroll
        for (int s = 0; s < NT / 2; ++s) {
            f32x4 lo = acc.acc[i][2 * s], hi = acc.acc[i][2 * s + 1];
            asm volatile("" : "+a"(lo), "+a"(hi));  // taken from the accumulation registers here and no earlier
            *reinterpret_cast<u32x4*>(wr + 64 * s) = pack(lane::kBlock * i, 32 * s, lo, hi);
        }
        u32x4 out[ITERS];
#pragma unroll
        for (int it = 0; it < ITERS; ++it) out[it] = *reinterpret_cast<const u32x4*>(rd + it * ROWS_PER_ITER * PITCH);
#pragma unroll
        for (int it = 0; it < ITERS; ++it) store(lane::kBlock * i + it * ROWS_PER_ITER, sub, 16 * piece, out[it]);
        __builtin_amdgcn_sched_barrier(0);  // one block row at a time keeps the register need small
    }
}

// ------------------------------------------------------------------------------------
// Pipelined main loop: direct-to-LDS copies, STAGES slots.  An operand is K-contiguous
// (its LDS tile is BM or BN rows of BK elements) or contiguous along its other index
// (A_MK: A along m, B_KN: B along n; the LDS tile is then BK k-rows of BM or BN elements,
// copied as it lies in memory, and the fragments, which need consecutive k per lane, are
// fetched with the transposing LDS read of gfx950, two per fragment).
// ------------------------------------------------------------------------------------
template <typename T, int BM, int BN, int BK, int WAVES_M, int WAVES_N, int STAGES, bool B_KN = false, bool A_MK = false>
struct Pipeline {
    using L = lane::TileLayout<BK>;
    static constexpr int ES = Frag<T>::kElemBytes;
    static constexpr int K_PER_STEP = L::kRowBytes / ES;  // elements of K one step consumes (BK counts 2-byte units)
    // (A 256x256 form of the k-row variants was built twice; beside 256 accumulators it spills
    // several hundred registers and runs at half the speed of the 128x128 form.)
    static_assert(!B_KN || (BK == 64 && BN == 128), "n-contiguous B: k-rows of 128 elements");
    static_assert(!A_MK || (BK == 64 && BM == 128), "m-contiguous A: k-rows of 128 elements");
    static_assert(!(A_MK && B_KN) || BM == BN, "both operands as k-rows: square tile");
    // A K-contiguous B is dealt to the LDS rows in the paired order (lane::paired_tile_row), so
    // that the epilogue can store from the registers; the k-row form keeps the plain order.
    static constexpr bool PAIRED_N = !B_KN;
    static constexpr int NW = WAVES_M * WAVES_N;
    static constexpr int THREADS = NW * 64;
    static constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
    static constexpr int MT = WTM / lane::kBlock, NT = WTN / lane::kBlock;
    static constexpr int KSUB = BK / lane::kBlockK;
    static constexpr int A_BYTES = BM * L::kRowBytes, B_BYTES = BN * L::kRowBytes;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int LDS_BYTES = STAGES * STAGE_BYTES;
    // LDS: the A tiles of all slots first, then the B tiles.  A lane's fragment addresses are then
    // one base per operand and sub-step plus constants below 64 KiB (block, slot), which fit the
    // offset field of the LDS read: no address arithmetic inside the K loop.
    static constexpr int a_slot(int stage) { return stage * A_BYTES; }
    static constexpr int b_slot(int stage) { return STAGES * A_BYTES + stage * B_BYTES; }
    static constexpr int COPY_ROWS = 1024 / L::kRowBytes;  // rows moved by one wave-wide copy
    static constexpr int A_COPIES = BM / COPY_ROWS / NW, B_COPIES = BN / COPY_ROWS / NW;  // per wave per K step
    static constexpr int COPIES = A_COPIES + B_COPIES;
    static_assert(BM % (COPY_ROWS * NW) == 0 && BN % (COPY_ROWS * NW) == 0, "tile rows must split over the waves");
    static_assert((NW * COPY_ROWS) % 16 == 0, "the swizzle of a lane's row must not depend on the copy index");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile is made of pairs of 16x16 blocks");
    static_assert(LDS_BYTES <= 163840, "LDS budget of one gfx950 compute unit");
    static_assert(NW * drain_patch_bytes(NT) <= LDS_BYTES, "epilogue patches reuse the operand slots");
    static_assert(STAGES >= 2 && (STAGES - 1) * COPIES <= 63, "vmcnt range");

    using tile_t = wave::Tile<T, MT, NT>;
    using frag_t = typename Frag<T>::type;

    // a_tile / b_tile: uniform byte pointers to element (first row of the tile,
    // first k of the slice); a_ld / b_ld: row pitch in bytes; a_rows / b_rows:
    // rows of the tile that exist (>= 1; missing rows re-read the last one and
    // their results are never stored).  ksteps >= 1 steps of BK k each.
    //
    // Schedule of one K step (KSUB sub-steps of 32 k, NM = MT*NT MFMAs each):
    //   sub-steps 0 .. KSUB-2 : MFMAs of sub-step s, the fragment reads of
    //                           sub-step s+1 dealt one by one between them;
    //   sub-step KSUB-1       : wait for my copies of the next step, barrier,
    //                           then the MFMAs with the copies of step
    //                           t+STAGES (into the slot just retired) and the
    //                           fragment reads of (t+1, 0) dealt between them.
    // Every piece is pinned with a scheduling fence so the matrix pipe always
    // has the next MFMA queued while the memory instructions issue.
    __device__ __forceinline__ static void run(persp::Workgroup wgp, tile_t& acc, const char* a_tile, uint32_t a_ld, int a_rows,
                               const char* b_tile, uint32_t b_ld, int b_rows, int ksteps,
                               char* lds, int wave, int lane, uint64_t* stamps = nullptr)
    {
        const persp::Wave wv = wgp.wave();  // every wave of the workgroup runs this code
        constexpr int PARTS = wave::mfma_parts(frag_t{});  // matrix instructions per block and sub-step
        constexpr int NM = MT * NT * PARTS;                // MFMAs per sub-step
        constexpr int A_READS = A_MK && ES == 2 ? 2 : 1, B_READS = B_KN && ES == 2 ? 2 : 1;  // LDS reads per fragment
        constexpr int NR = A_READS * MT + B_READS * NT;                // fragment reads per sub-step
        // -- per-lane copy offsets: wave-copy i moves row block (i*NW + wave) of COPY_ROWS rows;
        //    a lane fills one chunk position of one row with the logical chunk the swizzle wants.
        // (row pitches in bytes stay below 2^24 and rows below 2^8 -- the host refuses larger
        // pitches for this kernel -- so the full-rate 24-bit multiply gives the exact product)
        const int sub_row = lane / L::kChunksPerRow;
        const int chunk = (lane % L::kChunksPerRow) ^ L::swizzle(wave * COPY_ROWS + sub_row);
        uint32_t g_off[COPIES];
        // An operand kept as k-rows: a k-row of the tile is 128 elements and a wave-wide copy
        // moves 1024 bytes of them.  16-bit types: the 16-byte chunk c of k-row k sits at position
        // c ^ 2*(k%4), so that the four k-rows a transposing read touches fall on four different
        // 32-byte bank groups.  fp32: at position c ^ 4*((k/4)%2), so that the four k-rows of a
        // 4-byte gather (k = 4g + e for lane group g) alternate between the two halves of the
        // banks.  `cols` counts the elements of a k-row that exist (whole chunks); chunks beyond
        // them re-read the last one that exists and only feed results that are never stored.
        constexpr int KN_WIDTH = B_KN ? BN : BM;  // elements of a k-row (with both operands as k-rows BM == BN)
        constexpr int KN_ROW_BYTES = KN_WIDTH * ES, KN_CHUNKS = KN_ROW_BYTES / lane::kChunkBytes, KN_ROWS = 1024 / KN_ROW_BYTES;
        constexpr int PER_CHUNK = lane::kChunkBytes / ES;
        auto k_row_offset = [&](int i, uint32_t ld, int cols) __attribute__((always_inline)) {
            const int k_row = (i * NW + wave) * KN_ROWS + lane / KN_CHUNKS;
            const int swz = ES == 2 ? (k_row & 3) << 1 : ((k_row >> 2) & 1) << 2;
            int c = (lane % KN_CHUNKS) ^ swz;
            const int last = (cols - 1) / PER_CHUNK;
            c = c < last ? c : last;
            return __umul24(static_cast<uint32_t>(k_row), ld) + c * lane::kChunkBytes;
        };
#pragma unroll
        for (int i = 0; i < A_COPIES; ++i) {
            if constexpr (!A_MK) {
                int row = (i * NW + wave) * COPY_ROWS + sub_row;
                row = row < a_rows ? row : a_rows - 1;
                g_off[i] = __umul24(static_cast<uint32_t>(row), a_ld) + chunk * lane::kChunkBytes;
            } else {
                g_off[i] = k_row_offset(i, a_ld, a_rows);
            }
        }
#pragma unroll
        for (int i = 0; i < B_COPIES; ++i) {
            if constexpr (!B_KN) {
                int row = lane::paired_tile_row((i * NW + wave) * COPY_ROWS + sub_row);
                row = row < b_rows ? row : b_rows - 1;
                g_off[A_COPIES + i] = __umul24(static_cast<uint32_t>(row), b_ld) + chunk * lane::kChunkBytes;
            } else {
                g_off[A_COPIES + i] = k_row_offset(i, b_ld, b_rows);
            }
        }
        const uint32_t lds0 = lds_address(lds) + wave * 1024;

        // copy number c (0 .. COPIES-1) of K step `step` into slot `stage`
        auto copy = [&](int c, int step, int stage) __attribute__((always_inline)) {
            const int64_t k_bytes = static_cast<int64_t>(step) * L::kRowBytes;
            const int64_t a_bytes = A_MK ? static_cast<int64_t>(step) * K_PER_STEP * a_ld : k_bytes;
            const int64_t b_bytes = B_KN ? static_cast<int64_t>(step) * K_PER_STEP * b_ld : k_bytes;
            // (the slot's offset goes into the instruction's constant when the slot is known at compile time,
            // as in the steady loop, and into the base otherwise)
            const char* src = c < A_COPIES ? a_tile + a_bytes : b_tile + b_bytes;
            const int slot = c < A_COPIES ? a_slot(stage) : b_slot(stage);
            const int in_slot = (c < A_COPIES ? c : c - A_COPIES) * NW * 1024;
            if (__builtin_constant_p(stage)) copy_async_16(wv, src, g_off[c], lds0, slot + in_slot);
            else copy_async_16(wv, src, g_off[c], lds0 + slot, in_slot);
        };
        // -- prologue, first part: fill the slots.  The copies go out before the addressing of the
        //    fragment reads is worked out: that arithmetic then runs while the first bytes travel.
#pragma unroll
        for (int s = 0; s < STAGES; ++s)
            if (s < ksteps) {
#pragma unroll
                for (int c = 0; c < COPIES; ++c) copy(c, s, s);
            }
        __builtin_amdgcn_sched_barrier(0);

        // 16-bit operands kept as k-rows: fragments come from the transposing LDS read, see
        // wave::read_k_rows_half; four per-lane address parts serve all reads.
        uint32_t k_rows_part[4];
#pragma unroll
        for (int jl = 0; jl < 4; ++jl) k_rows_part[jl] = wave::k_rows_lane_part<KN_ROW_BYTES>(wv, jl, lane);
        auto read_k_rows = [&](const char* tile, int row0, int j, int ksub, int h) __attribute__((always_inline)) {
            return wave::read_k_rows_half<KN_ROW_BYTES>(wv, tile, row0, j, ksub, h, k_rows_part);
        };
        // fp32 fragment from k-rows: element e of lane (x, g) is the value at k-row 16*ksub + 4g + e,
        // element first + x; nothing to transpose, four 4-byte reads.
        auto gather_k_rows = [&](const char* tile, int first, int ksub) __attribute__((always_inline)) {
            const int n = first + (lane & 15), g = lane >> 4;
            const char* src = tile + (16 * ksub + 4 * g) * KN_ROW_BYTES + (((n >> 2) ^ ((g & 1) << 2)) * lane::kChunkBytes) + (n & 3) * 4;
            f32x4 v;
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = *reinterpret_cast<const float*>(src + e * KN_ROW_BYTES);
            return v;
        };

        const int wave_m = wave / WAVES_N, wave_n = wave % WAVES_N;
        const int a_row0 = wave_m * WTM, b_row0 = wave_n * WTN;
        using v4s = wave::v4s;
        static_assert(WTM % 8 == 0 && WTN % 8 == 0 && lane::kBlock % 8 == 0, "row blocks start at multiples of 8 rows");
        // The lane's share of a fragment address, one per operand and sub-step: wave tile's first
        // row, the lane's row and chunk inside a block, and for B the start of the B tiles.  Every
        // read of the K loop is one of these plus a constant (block, slot) below 64 KiB.
        uint32_t fa_off[KSUB], fb_off[KSUB];
#pragma unroll
        for (int ks = 0; ks < KSUB; ++ks) {
            const uint32_t part = lane::fragment_lane_part<BK>(wv.lane(), ks, lane);
            fa_off[ks] = a_row0 * L::kRowBytes + part;
            fb_off[ks] = b_slot(0) + b_row0 * L::kRowBytes + part;
            asm volatile("" : "+v"(fa_off[ks]), "+v"(fb_off[ks]));  // kept in registers, not re-derived per read
        }
        frag_t fa[2][MT], fb[2][NT];
        v4s fah[2][MT][2], fbh[2][NT][2];  // operands kept as k-rows: the two halves of every fragment
        // read number r (0 .. NR-1) of sub-step ksub of slot `stage` into buffer `buf`;
        // order: a0, all b, remaining a -- what the first MFMAs of the next group need first
        auto read_a = [&](int x, int buf, int stage, int ksub) __attribute__((always_inline)) {  // x: fragment * A_READS + half
            const char* st = lds + a_slot(stage);
            if constexpr (A_MK && ES == 2) fah[buf][x / 2][x % 2] = read_k_rows(st, a_row0, x / 2, ksub, x % 2);
            else if constexpr (A_MK) fa[buf][x] = __builtin_bit_cast(frag_t, gather_k_rows(st, a_row0 + lane::kBlock * x, ksub));
            else fa[buf][x] = lane::load_fragment_at<T>(wv.lane(), st + lane::kBlock * x * L::kRowBytes, fa_off[ksub]);
        };
        auto read_b = [&](int x, int buf, int stage, int ksub) __attribute__((always_inline)) {
            const char* st = lds + b_slot(stage);
            if constexpr (B_KN && ES == 2) fbh[buf][x / 2][x % 2] = read_k_rows(st, b_row0, x / 2, ksub, x % 2);
            else if constexpr (B_KN) fb[buf][x] = __builtin_bit_cast(frag_t, gather_k_rows(st, b_row0 + lane::kBlock * x, ksub));
            else fb[buf][x] = lane::load_fragment_at<T>(wv.lane(), st - b_slot(0) + lane::kBlock * x * L::kRowBytes, fb_off[ksub]);
        };
        auto read = [&](int r, int buf, int stage, int ksub) __attribute__((always_inline)) {
            if (r < A_READS) read_a(r, buf, stage, ksub);
            else if (r < A_READS + B_READS * NT) read_b(r - A_READS, buf, stage, ksub);
            else read_a(r - B_READS * NT, buf, stage, ksub);
        };
        auto whole = [](v4s lo, v4s hi) __attribute__((always_inline)) {
            if constexpr (ES == 2) return __builtin_bit_cast(frag_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
            else return frag_t{};
        };
        auto mfma = [&](int m, int buf) __attribute__((always_inline)) {
            const int e = m / (MT * NT), blk = m % (MT * NT), i = blk / NT, j = blk % NT;
            frag_t a, b;
            if constexpr (A_MK && ES == 2) a = whole(fah[buf][i][0], fah[buf][i][1]);
            else a = fa[buf][i];
            if constexpr (B_KN && ES == 2) b = whole(fbh[buf][j][0], fbh[buf][j][1]);
            else b = fb[buf][j];
            acc.acc[i][j] = wave::mfma_part(wv, b, a, e, acc.acc[i][j]);
        };

        // -- prologue, second part: wait for step 0, fetch its first fragments
        if (ksteps >= STAGES) wait_counts<(STAGES - 1) * COPIES, 0>();
        else wait_counts<0, 0>();
        barrier(wgp);
        asm volatile("" ::: "memory");
#pragma unroll
        for (int r = 0; r < NR; ++r) read(r, 0, 0, 0);
        PRISM_PARANOID_SYNC(wgp);
        stamp(stamps, STAMP_FIRST_FRAGMENTS);

        // MFMA slots of the memory instructions of a group: reads on the even slots, copies on
        // the odd ones, so no MFMA has more than one of them in its 16-cycle shadow.
        // Read r sits on slot READ_SPACING*r, head copy c on slot 2c+1, tail copy c on slot
        // TAIL_SPACING*c+1.  The first TAILN copies of a step are issued right after the slot
        // is released, the last HEADN at the start of the following step.  (The slot of an
        // instruction is computed from the slot index, not searched for: the loops below are
        // unrolled in full, and their size before unrolling is limited.)
        // (All copies go out right after the release when a slot every fourth MFMA is enough for
        // them: with the sustained clock that is as fast on 4096^3 and 2 % faster on 8192^3.)
        constexpr int HEADN = 4 * (COPIES - 1) + 1 < NM ? 0 : COPIES / 4, TAILN = COPIES - HEADN;
        constexpr int TAIL_SPACING = 4 * (TAILN - 1) + 1 < NM ? 4 : 2;
        constexpr int READ_SPACING = 2 * NR <= NM ? 2 : 1;  // reads share slots with copies only when they must
        static_assert(NR <= NM && 2 * HEADN <= NM && TAIL_SPACING * (TAILN - 1) + 1 < NM,
                      "every memory instruction of a group needs an MFMA slot");

        // One K step t on slot `stage`.
        //   HEAD: the last HEADN copies of step t+1 are issued in sub-step 0
        //   TAIL: the first TAILN copies of step t+2 are issued after the hand-over
        //   LAST: no step follows (no hand-over)
        // Issuing most copies as early as the slot allows gives them a whole K step to land
        // (rows 16 KiB apart miss the L2 and the address translation caches far more often
        // than the MFMAs of half a step can hide); spreading them keeps every MFMA slot down
        // to one memory instruction, which is what a wave can issue in the shadow of one MFMA.
        auto k_step = [&](auto head_c, auto tail_c, auto last_c, int t, int stage, int next) __attribute__((always_inline)) {
            constexpr bool HEAD = decltype(head_c)::value;
            constexpr bool TAIL = decltype(tail_c)::value;
            constexpr bool LAST = decltype(last_c)::value;
#pragma unroll
            for (int ks = 0; ks < KSUB; ++ks) {
                const int cur = ks & 1, nxt = cur ^ 1;
                if (ks + 1 < KSUB) {
#pragma unroll
                    for (int m = 0; m < NM; ++m) {
                        if (m % READ_SPACING == 0 && m / READ_SPACING < NR) read(m / READ_SPACING, nxt, stage, ks + 1);
                        if (HEAD && ks == 0 && m % 2 == 1 && m / 2 < HEADN) copy(TAILN + m / 2, t + 1, next);
                        __builtin_amdgcn_sched_barrier(0);  // memory instructions stay in front of their MFMA
                        mfma(m, cur);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                } else if (!LAST) {
                    // Hand-over: my copies for step t+1 have landed and my reads of this
                    // slot are done; after the barrier that holds for every wave.
                    wait_counts<0, 0>();
                    barrier(wgp);
                    asm volatile("" ::: "memory");  // keep what follows on this side of the barrier
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int m = 0; m < NM; ++m) {
                        if (m % READ_SPACING == 0 && m / READ_SPACING < NR) read(m / READ_SPACING, nxt, next, 0);
                        if (TAIL && m % TAIL_SPACING == 1 && m / TAIL_SPACING < TAILN) copy(m / TAIL_SPACING, t + 2, stage);
                        __builtin_amdgcn_sched_barrier(0);  // memory instructions stay in front of their MFMA
                        mfma(m, cur);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                } else {
#pragma unroll
                    for (int m = 0; m < NM; ++m) mfma(m, cur);
                }
                PRISM_PARANOID_SYNC(wgp);
            }
        };
        static_assert(KSUB % 2 == 0, "fragment buffers must return to slot 0 at the end of a K step");
        static_assert(STAGES == 2 && COPIES % 2 == 0, "the copy schedule below is written for two slots");

        using yes = std::integral_constant<bool, true>;
        using no = std::integral_constant<bool, false>;
        // step t's copies: the first TAILN issued after the hand-over of step t-2, the rest in
        // sub-step 0 of step t-1; steps 0 and 1 came whole from the prologue.
        int t = 0;
        if (ksteps == 1) {
            k_step(no{}, no{}, yes{}, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            return;
        }
        if (ksteps > 2) k_step(no{}, yes{}, no{}, 0, 0, 1);
        else k_step(no{}, no{}, no{}, 0, 0, 1);
        // steady state, two steps per trip so that the slot of a step is a compile-time constant
        // (LDS addresses fold into instruction offsets instead of being recomputed every step)
        for (t = 1; t + 3 < ksteps; t += 2) {
            k_step(yes{}, yes{}, no{}, t, 1, 0);
            k_step(yes{}, yes{}, no{}, t + 1, 0, 1);
        }
        if (t + 2 < ksteps) {  // t is odd here
            k_step(yes{}, yes{}, no{}, t, 1, 0);
            ++t;
        }
        if (t + 1 < ksteps) {  // t == ksteps - 2 >= 1: step t+1 >= 2 still needs its second half
            k_step(yes{}, no{}, no{}, t, t & 1, (t & 1) ^ 1);
            ++t;
        }
        k_step(no{}, no{}, yes{}, t, t & 1, t & 1);
        __builtin_amdgcn_sched_barrier(0);  // nothing of the epilogue moves up into the K loop
    }
};

// drain_runs with one 16-row block per pass and no padding: the patch is 16 rows of
// 16*NT floats (8 KiB for a 128-wide wave tile).  Instead of padding, the 16-byte unit at
// position p of row r is kept at position p ^ r (positions as in drain_runs: even units
// first), which spreads the 16 rows of a write and the 16 units of a read over the banks.
template <int MT, int NT, typename TileT, typename Sink>
__device__ __forceinline__ void drain_runs16(persp::Wave, const TileT& acc, char* patch, int lane, Sink&& sink)
{
    constexpr int WTN = lane::kBlock * NT;
    constexpr int UNITS = WTN / 4;
    constexpr int PITCH = WTN * 4;            // bytes
    constexpr int LANES_PER_ROW = WTN / 8;
    constexpr int ROWS_PER_ITER = 64 / LANES_PER_ROW;
    constexpr int ITERS = lane::kBlock / ROWS_PER_ITER;
    static_assert(UNITS / 2 >= 16 || UNITS / 2 == 8, "the row index is folded into the low position bits");
    constexpr int FOLD = UNITS / 2 >= 16 ? 15 : 7;  // bits of the row folded into the position
    const int run = lane % LANES_PER_ROW, sub = lane / LANES_PER_ROW;
    const int q = lane >> 4, r = lane::acc_col(lane);
    const int pos_q = (q >> 1) + (UNITS / 2) * (q & 1);  // plus 2j for block column j
    char* wr = patch + r * PITCH;
#pragma unroll
    for (int i = 0; i < MT; ++i) {
#pragma unroll
        for (int j = 0; j < NT; ++j)
            *reinterpret_cast<f32x4*>(wr + 16 * ((pos_q + 2 * j) ^ (r & FOLD))) = acc.acc[i][j];
        f32x4 lo[ITERS], hi[ITERS];
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int row = it * ROWS_PER_ITER + sub;
            const char* rd = patch + row * PITCH;
            lo[it] = *reinterpret_cast<const f32x4*>(rd + 16 * (run ^ (row & FOLD)));
            hi[it] = *reinterpret_cast<const f32x4*>(rd + 16 * ((run + UNITS / 2) ^ (row & FOLD)));
        }
#pragma unroll
        for (int it = 0; it < ITERS; ++it) sink(lane::kBlock * i + it * ROWS_PER_ITER, sub, lo[it], hi[it]);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// ------------------------------------------------------------------------------------
// Persistent form of the pipeline: one workgroup walks a sequence of 256x256 tiles and
// treats their K steps as one stream.  The copies issued in the last two steps of a tile
// already belong to the next tile, so its first operands sit in LDS when its first MFMA
// issues, and the fixed cost of starting a tile (first loads from memory) disappears for
// every tile but the first.  This is the tile loop of the paper's persistent hgemm kernel
// (code appendix, `while(true)` over tiles) with the loads of the next tile pipelined
// under the tail of the current one.
//
// LDS: two operand slots (128 KiB) and, behind them, one 8 KiB epilogue patch per wave,
// which together are exactly the 160 KiB of a compute unit; the patches are separate so
// that the epilogue of a tile can run while the slots already hold the next tile.
// ------------------------------------------------------------------------------------
template <typename T, int HEADN = 0>  // copies of a step left for the start of the next one (0: measured best)
struct PersistentPipe {
    using L = lane::TileLayout<64>;
    static constexpr int BM = 256, BN = 256, BK = 64, WAVES_M = 2, WAVES_N = 2, NW = 4, THREADS = 256;
    static constexpr bool PAIRED_N = true;  // B rows in the paired order, as in Pipeline
    static constexpr int WTM = 128, WTN = 128, MT = WTM / lane::kBlock, NT = WTN / lane::kBlock;
    static constexpr int KSUB = BK / lane::kBlockK, NM = MT * NT, NR = MT + NT;
    static constexpr int A_BYTES = BM * L::kRowBytes, B_BYTES = BN * L::kRowBytes, STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int a_slot(int stage) { return stage * A_BYTES; }              // A tiles of both slots first,
    static constexpr int b_slot(int stage) { return 2 * A_BYTES + stage * B_BYTES; }  // then the B tiles (see Pipeline)
    static constexpr int PATCH_BYTES = lane::kBlock * WTN * 4;
    static constexpr int PATCH_BASE = 2 * STAGE_BYTES;
    static constexpr int LDS_BYTES = PATCH_BASE + NW * PATCH_BYTES;
    static constexpr int COPY_ROWS = 8, A_COPIES = BM / COPY_ROWS / NW, COPIES = 2 * A_COPIES;
    static constexpr int TAILN = COPIES - HEADN;
    static_assert(HEADN >= 0 && HEADN <= COPIES && 4 * (TAILN - 1) + 1 < MT * NT && 2 * (MT + NT) <= MT * NT,
                  "every memory instruction of a group needs an MFMA slot of its own kind");
    static_assert(LDS_BYTES <= 163840 && KSUB == 2 && BM == BN, "written for the 256x256x64 tile");

    using tile_t = wave::Tile<T, MT, NT>;
    using frag_t = typename Frag<T>::type;

    // Operand rows of one tile: a / b point at (first row of the tile, first k of the slice).
    struct Source {
        const char* a;
        const char* b;
        uint32_t a_ld, b_ld;  // row pitch in bytes
        int a_rows, b_rows;   // rows that exist (>= 1)
    };

    // Walks the tiles of one workgroup.
    //   first / first_ksteps: operands and K steps (even, >= 2) of the first tile
    //   peek(Source&, int& ksteps) -> bool: describes the tile after the current one, false if none
    //   finish(tile_t&): epilogue of the current tile (its accumulators are complete)
    //   advance(): the tile described by the last peek becomes the current one
    template <typename Peek, typename Finish, typename Advance>
    __device__ __forceinline__ static void run(persp::Workgroup wgp, char* lds, int wave, int lane, Source first, int first_ksteps,
                                               Peek&& peek, Finish&& finish, Advance&& advance)
    {
        const persp::Wave wv = wgp.wave();  // every wave of the workgroup runs this code
        tile_t acc;
        frag_t fa[2][MT], fb[2][NT];
        uint32_t g_off[COPIES];
        const uint32_t lds0 = lds_address(lds) + wave * 1024;
        const int a_row0 = (wave / WAVES_N) * WTM, b_row0 = (wave % WAVES_N) * WTN;

        // per-lane copy offsets for a tile (rows beyond the matrix re-read the last row)
        auto set_offsets = [&](const Source& s) __attribute__((always_inline)) {
            const int sub_row = lane / L::kChunksPerRow;
            const int chunk = (lane % L::kChunksPerRow) ^ L::swizzle(wave * COPY_ROWS + sub_row);
#pragma unroll
            for (int i = 0; i < A_COPIES; ++i) {
                const int row = (i * NW + wave) * COPY_ROWS + sub_row, row_b = lane::paired_tile_row(row);
                const int ra = row < s.a_rows ? row : s.a_rows - 1;
                const int rb = row_b < s.b_rows ? row_b : s.b_rows - 1;
                g_off[i] = __umul24(static_cast<uint32_t>(ra), s.a_ld) + chunk * lane::kChunkBytes;
                g_off[A_COPIES + i] = __umul24(static_cast<uint32_t>(rb), s.b_ld) + chunk * lane::kChunkBytes;
                // (kept as they are in registers: left to itself the compiler splits every offset into a
                // uniform and a per-lane part and adds them again in front of each copy of the K loop)
                asm volatile("" : "+v"(g_off[i]), "+v"(g_off[A_COPIES + i]));
            }
        };
        // copy number c of the K step whose operands start at a_src / b_src, into slot `stage`
        auto copy = [&](int c, const char* a_src, const char* b_src, int stage) __attribute__((always_inline)) {
            if (c < A_COPIES) copy_async_16(wv, a_src, g_off[c], lds0, a_slot(stage) + c * NW * 1024);
            else copy_async_16(wv, b_src, g_off[c], lds0, b_slot(stage) + (c - A_COPIES) * NW * 1024);
        };
        uint32_t fa_off[KSUB], fb_off[KSUB];  // the lane's share of a fragment address per operand and sub-step (see Pipeline)
#pragma unroll
        for (int ks = 0; ks < KSUB; ++ks) {
            const uint32_t part = lane::fragment_lane_part<BK>(wv.lane(), ks, lane);
            fa_off[ks] = a_row0 * L::kRowBytes + part;
            fb_off[ks] = b_slot(0) + b_row0 * L::kRowBytes + part;
            asm volatile("" : "+v"(fa_off[ks]), "+v"(fb_off[ks]));
        }
        auto read = [&](int r, int buf, int stage, int ksub) __attribute__((always_inline)) {
            const char* sa = lds + a_slot(stage);
            const char* sb = lds + b_slot(stage) - b_slot(0);
            if (r == 0) fa[buf][0] = lane::load_fragment_at<T>(wv.lane(), sa, fa_off[ksub]);
            else if (r <= NT) fb[buf][r - 1] = lane::load_fragment_at<T>(wv.lane(), sb + lane::kBlock * (r - 1) * L::kRowBytes, fb_off[ksub]);
            else fa[buf][r - NT] = lane::load_fragment_at<T>(wv.lane(), sa + lane::kBlock * (r - NT) * L::kRowBytes, fa_off[ksub]);
        };
        auto mfma = [&](int m, int buf) __attribute__((always_inline)) {
            const int i = m / NT, j = m % NT;
            acc.acc[i][j] = wave::mfma_block(wv, fb[buf][j], fa[buf][i], acc.acc[i][j]);
        };
        constexpr int TAIL_SPACING = 4;  // read r on slot 2r, head copy c on 2c+1, tail copy c on 4c+1

        // One K step computing from slot `stage`.  After the hand-over (wait, barrier, first
        // fragments of the next step) this slot is free, and sub-step 1 issues the first TAILN
        // copies of the step after next (from a2 / b2) into it; the remaining HEADN copies of
        // that step follow in sub-step 0 of the next step (here: from a1 / b1 into the other
        // slot).  "Next" steps past the end of a tile are the first steps of the following
        // tile, so the loop never drains; switch_now loads that tile's copy offsets between
        // the two halves.
        auto k_step = [&](auto stage_c, const char* a1, const char* b1, bool switch_now, const Source& to,
                          const char* a2, const char* b2) __attribute__((always_inline)) {
            constexpr int stage = decltype(stage_c)::value, next = stage ^ 1;
#pragma unroll
            for (int m = 0; m < NM; ++m) {
                if (m % 2 == 0 && m / 2 < NR) read(m / 2, 1, stage, 1);
                if (m % 2 == 1 && m / 2 < HEADN) copy(TAILN + m / 2, a1, b1, next);
                __builtin_amdgcn_sched_barrier(0);
                mfma(m, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
            PRISM_PARANOID_SYNC(wgp);
            if (switch_now) set_offsets(to);
            wait_counts<0, 0>();
            barrier(wgp);
            asm volatile("" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int m = 0; m < NM; ++m) {
                if (m % 2 == 0 && m / 2 < NR) read(m / 2, 0, next, 0);
                if (m % TAIL_SPACING == 1 && m / TAIL_SPACING < TAILN) copy(m / TAIL_SPACING, a2, b2, stage);
                __builtin_amdgcn_sched_barrier(0);
                mfma(m, 1);
                __builtin_amdgcn_sched_barrier(0);
            }
            PRISM_PARANOID_SYNC(wgp);
        };
        constexpr int STEP = L::kRowBytes;  // bytes one K step advances in a row
        // Keeps every accumulator block in the accumulation registers at the edges of the K
        // loop, so that the register allocator does not rotate blocks through VGPRs inside it.
        auto pin_acc = [&]() __attribute__((always_inline)) {
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < NT; ++j) asm volatile("" : "+a"(acc.acc[i][j]));
        };

        // -- before the first tile: step 0 whole, the first TAILN copies of step 1, the first fragments
        Source sc = first;
        int ksteps = first_ksteps;
        set_offsets(sc);
#pragma unroll
        for (int c = 0; c < COPIES; ++c) copy(c, sc.a, sc.b, 0);
#pragma unroll
        for (int c = 0; c < TAILN; ++c) copy(c, sc.a + STEP, sc.b + STEP, 1);
        wait_counts<TAILN, 0>();
        barrier(wgp);
        asm volatile("" ::: "memory");
#pragma unroll
        for (int r = 0; r < NR; ++r) read(r, 0, 0, 0);

        using slot0 = std::integral_constant<int, 0>;
        using slot1 = std::integral_constant<int, 1>;
        for (;;) {
            // Without a following tile the copies past the end re-read this tile's last two
            // steps (just fetched, so they come from the cache) into slots nobody reads again:
            // no branch around any copy and no traffic to memory.
            Source sn = sc;
            int next_ksteps = ksteps;
            const bool has_next = peek(sn, next_ksteps);
            if (!has_next) {
                sn.a = sc.a + static_cast<int64_t>(ksteps - 2) * L::kRowBytes;
                sn.b = sc.b + static_cast<int64_t>(ksteps - 2) * L::kRowBytes;
            }
            acc.clear();
            pin_acc();
            // Every tile has an even number of K steps, so a trip of two steps always starts on
            // slot 0 and slots are compile-time constants.  Past the end of the tile the copies
            // continue with the first two steps of the next one.
            for (int t = 0; t < ksteps; t += 2) {
                const bool last = t + 2 == ksteps;
                const char* a1 = sc.a + static_cast<int64_t>(t + 1) * STEP;
                const char* b1 = sc.b + static_cast<int64_t>(t + 1) * STEP;
                const char* a2 = last ? sn.a : sc.a + static_cast<int64_t>(t + 2) * STEP;
                const char* b2 = last ? sn.b : sc.b + static_cast<int64_t>(t + 2) * STEP;
                k_step(slot0{}, a1, b1, last, sn, a2, b2);
                k_step(slot1{}, a2, b2, false, sn, a2 + STEP, b2 + STEP);
            }
            pin_acc();
            finish(acc);
            if (!has_next) break;
            advance();
            sc = sn;
            ksteps = next_ksteps;
        }
        wait_counts<0, 0>();  // the copies issued past the end of the last tile
    }
};

// ------------------------------------------------------------------------------------
// Staged main loop: any element strides and alignments, 16-bit or fp32 operands.  The
// operands of a K step pass through registers, are zero-filled outside the matrix and
// written to one LDS slot; the loads of step t+1 are in flight while step t computes.
// A K step is 128 bytes of every operand row (64 elements of a 16-bit type, 32 of fp32).
// This is the paper's sgemm structure (section 6.1: block tile staged in shared memory,
// then warp- and thread-level tiles), with the thread-level tile replaced by MFMA blocks.
// ------------------------------------------------------------------------------------
template <typename T>
struct Staged {
    using L = lane::TileLayout<64>;  // rows of 128 bytes
    static constexpr int ES = Frag<T>::kElemBytes, EPC = lane::kChunkBytes / ES;  // elements per chunk
    static constexpr int BM = 128, BN = 128, BK = L::kRowBytes / ES, NW = 4, THREADS = 256;
    static constexpr int WTM = 64, WTN = 64, MT = WTM / lane::kBlock, NT = WTN / lane::kBlock;
    static constexpr int KSUB = L::kChunksPerRow / 4;  // a fragment read covers 4 chunks of a row
    static constexpr int A_BYTES = BM * L::kRowBytes, B_BYTES = BN * L::kRowBytes;
    static constexpr int DRAIN_BYTES = NW * drain_patch_bytes(NT);
    static constexpr int LDS_BYTES = A_BYTES + B_BYTES > DRAIN_BYTES ? A_BYTES + B_BYTES : DRAIN_BYTES;
    static constexpr int CHUNKS = BM * L::kChunksPerRow / THREADS;  // per thread per operand

    using tile_t = wave::Tile<T, MT, NT>;
    using frag_t = typename Frag<T>::type;
    using elem_t = typename std::conditional<ES == 2, uint16_t, uint32_t>::type;

    // One thread's share of a 128-row operand tile as CHUNKS 16-byte chunks.
    // base: element (row 0 of the tile, k 0 of the matrix); s_row / s_k: element
    // strides; rows: rows that exist; k0: first k of this step; k_end: end of
    // the slice.  vec: rows are K-contiguous and every chunk is 16-byte aligned.
    // With K-contiguous rows consecutive threads take consecutive chunks of a row,
    // otherwise consecutive rows of one chunk, so that either way they read
    // neighbouring addresses.
    __device__ __forceinline__ static void gather(u32x4 (&regs)[CHUNKS], const char* base, int64_t s_row, int64_t s_k,
                                  int rows, int k0, int k_end, bool vec, int tid)
    {
        const bool k_fast = s_k == 1;
#pragma unroll
        for (int i = 0; i < CHUNKS; ++i) {
            const int q = tid + THREADS * i;
            const int row = k_fast ? q / L::kChunksPerRow : q % BM;
            const int c = k_fast ? q % L::kChunksPerRow : q / BM;
            const int k = k0 + EPC * c;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (row < rows && k < k_end) {
                const char* src = base + ES * (row * s_row + k * s_k);
                if (vec && k + EPC <= k_end) {
                    v = *reinterpret_cast<const u32x4*>(src);
                } else {
                    uint32_t h[EPC];
#pragma unroll
                    for (int e = 0; e < EPC; ++e)
                        h[e] = (k + e < k_end) ? *reinterpret_cast<const elem_t*>(src + ES * e * s_k) : 0u;
                    if constexpr (ES == 2)
                        v = u32x4{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
                    else
                        v = u32x4{h[0], h[1], h[2], h[3]};
                }
            }
            regs[i] = v;
        }
    }

    // Where one thread's chunks of a whole K step come from, for an operand whose chunks can be
    // fetched without looking at k: byte offsets from the step's first element (rows beyond the
    // matrix re-read the last row and are zeroed in commit).  Valid when the operand is
    // K-contiguous with aligned chunks, or contiguous along its rows.
    struct Regular {
        uint32_t off[CHUNKS];
        bool inside[CHUNKS];
    };
    __device__ __forceinline__ static Regular regular(int64_t s_row, int64_t s_k, int rows, int tid)
    {
        Regular r;
        const bool k_fast = s_k == 1;
#pragma unroll
        for (int i = 0; i < CHUNKS; ++i) {
            const int q = tid + THREADS * i;
            const int row = k_fast ? q / L::kChunksPerRow : q % BM;
            const int c = k_fast ? q % L::kChunksPerRow : q / BM;
            r.inside[i] = row < rows;
            r.off[i] = static_cast<uint32_t>(ES * ((row < rows ? row : rows - 1) * s_row + EPC * c * s_k));
        }
        return r;
    }
    // All chunks of a K step that lies wholly inside the slice; step0 points at (row 0, first k
    // of the step).  No address arithmetic per lane: uniform base plus the fixed offsets.
    __device__ __forceinline__ static void gather_regular(u32x4 (&regs)[CHUNKS], const char* step0, int64_t s_k,
                                                          const Regular& r)
    {
        if (s_k == 1) {
#pragma unroll
            for (int i = 0; i < CHUNKS; ++i) regs[i] = *reinterpret_cast<const u32x4*>(step0 + r.off[i]);
        } else {
            const int64_t pitch = ES * s_k;
#pragma unroll
            for (int i = 0; i < CHUNKS; ++i) {
                uint32_t h[EPC];
#pragma unroll
                for (int e = 0; e < EPC; ++e) h[e] = *reinterpret_cast<const elem_t*>(step0 + e * pitch + r.off[i]);
                if constexpr (ES == 2)
                    regs[i] = u32x4{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
                else
                    regs[i] = u32x4{h[0], h[1], h[2], h[3]};
            }
        }
    }

    __device__ __forceinline__ static void commit(const u32x4 (&regs)[CHUNKS], const bool (&inside)[CHUNKS], char* tile,
                                                  bool k_fast, int tid)
    {
#pragma unroll
        for (int i = 0; i < CHUNKS; ++i) {
            const int q = tid + THREADS * i;
            const int row = k_fast ? q / L::kChunksPerRow : q % BM;
            const int c = k_fast ? q % L::kChunksPerRow : q / BM;
            *reinterpret_cast<u32x4*>(tile + L::offset(row, c)) = inside[i] ? regs[i] : u32x4{0u, 0u, 0u, 0u};
        }
    }

    __device__ __forceinline__ static void run(persp::Workgroup wgp, tile_t& acc, const char* a_tile, int64_t a_sm, int64_t a_sk, int a_rows, bool a_vec,
                               const char* b_tile, int64_t b_sn, int64_t b_sk, int b_rows, bool b_vec,
                               int k_begin, int k_end, char* lds, int wave, int lane)
    {
        const persp::Wave wv = wgp.wave();  // every wave of the workgroup runs this code
        const int tid = wave * 64 + lane;
        const int wave_m = wave >> 1, wave_n = wave & 1;
        // Whole K steps of "regular" operands take the cheap fetch; the last, partial step and
        // operands with other strides or alignments take the general one.
        auto is_regular = [](int64_t s_row, int64_t s_k, bool vec) {
            const int64_t reach = (BM - 1) * (s_row < 0 ? -s_row : s_row) + (BK - 1) * (s_k < 0 ? -s_k : s_k);
            return (s_k == 1 ? vec : s_row == 1) && s_row >= 0 && s_k >= 0 && reach * ES < (int64_t{1} << 31);
        };
        const bool all_regular = is_regular(a_sm, a_sk, a_vec) && is_regular(b_sn, b_sk, b_vec);
        const Regular pa = regular(a_sm, a_sk, a_rows, tid), pb = regular(b_sn, b_sk, b_rows, tid);
        u32x4 ra[CHUNKS], rb[CHUNKS];
        auto fetch = [&](int k0) __attribute__((always_inline)) {
            if (all_regular && k0 + BK <= k_end) {
                gather_regular(ra, a_tile + ES * k0 * a_sk, a_sk, pa);
                gather_regular(rb, b_tile + ES * k0 * b_sk, b_sk, pb);
            } else {
                gather(ra, a_tile, a_sm, a_sk, a_rows, k0, k_end, a_vec, tid);
                gather(rb, b_tile, b_sn, b_sk, b_rows, k0, k_end, b_vec, tid);
            }
        };
        fetch(k_begin);
        for (int k0 = k_begin; k0 < k_end; k0 += BK) {
            sync(wgp);  // the previous step's fragment reads are finished
            commit(ra, pa.inside, lds, a_sk == 1, tid);
            commit(rb, pb.inside, lds + A_BYTES, b_sk == 1, tid);
            sync(wgp);
            if (k0 + BK < k_end) fetch(k0 + BK);  // next step's operands travel while this one computes
#pragma unroll
            for (int ks = 0; ks < KSUB; ++ks) {
                frag_t fa[MT], fb[NT];
                wave::load_fragments<T, 64, MT>(wv, fa, lds, wave_m * WTM, ks, lane);
                wave::load_fragments<T, 64, NT>(wv, fb, lds + A_BYTES, wave_n * WTN, ks, lane);
                acc.mma(wv, fa, fb);
            }
        }
    }
};

}  // namespace wg
}  // namespace prism
