// Device kernels: thin __global__ shells that place a workgroup on its tile
// (grid layer), run a workgroup main loop and hand the accumulators to the
// epilogue.  All arithmetic of the matrix product happens here on the GPU.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "grid.hpp"
#include "lane.hpp"
#include "launch.hpp"
#include "wave.hpp"
#include "workgroup.hpp"

namespace prism {

const PipeConfig kPipeConfigs[kNumPipeConfigs] = {
    {0, 256, 256, 64, 4, 2, "256x256x64_w4"},
    {1, 128, 128, 64, 4, 2, "128x128x64_w4"},
    {2, 128, 128, 64, 4, 2, "128x128x64_w4_b_along_n"},
    {3, 128, 128, 64, 4, 2, "128x128x64_w4_a_along_m"},
    {4, 128, 128, 64, 4, 2, "128x128x64_w4_a_along_m_b_along_n"},
    {5, 128, 128, 32, 4, 2, "f32_128x128x32_w4"},
    {6, 128, 128, 32, 4, 2, "f32_128x128x32_w4_b_along_n"},
    {7, 128, 128, 32, 4, 2, "f32_128x128x32_w4_a_along_m"},
    {8, 128, 128, 32, 4, 2, "f32_128x128x32_w4_a_along_m_b_along_n"},
};

namespace {

struct Placement {
    int batch, slice, m0, n0, k_begin, k_end;
};

template <int BM, int BN>
__device__ __forceinline__ Placement place(const GemmParams& p, int wg)
{
    const grid::TileCoord c = grid::schedule(wg, p.tiles_m, p.tiles_n, p.batch * p.split_k);
    Placement q;
    q.batch = c.unit / p.split_k;
    q.slice = c.unit - q.batch * p.split_k;
    q.m0 = c.tile_m * BM;
    q.n0 = c.tile_n * BN;
    q.k_begin = q.slice * p.k_slice;
    q.k_end = q.k_begin + p.k_slice < p.K ? q.k_begin + p.k_slice : p.K;
    return q;
}

// Accumulators of one wave tile -> C or the split-K scratch.
// OWN_PATCH false: the patches reuse the operand slots; workgroup-collective, every wave
// must call it (it starts with a barrier that retires the slots).  OWN_PATCH true: `patch`
// is this wave's private 16-row patch outside the slots; no barrier, 16 rows per pass.
// Partial sums of the same workgroup tile computed elsewhere (stream-K): `count` row-major
// 256 x 256 fp32 tiles, kPartialTile floats apart, added to the accumulators on their way out.
constexpr int kPartialSide = 256, kPartialTile = kPartialSide * kPartialSide;
struct Addends {
    const float* first = nullptr;
    int count = 0;
};

template <typename TileT, int MT, int NT, bool OWN_PATCH = false, bool PAIRED = false, bool ADD = false>
__device__ __forceinline__ void epilogue(persp::Workgroup wgp, const GemmParams& p, const Placement& q, const TileT& acc,
                                         int m_wave, int n_wave, char* lds, int wave, int lane, Addends add = Addends{})
{
    const persp::Wave wv = wgp.wave();
    const int esize = p.c_dtype == DT_F32 ? 4 : 2;
    char* c_problem = p.C + static_cast<int64_t>(q.batch) * p.batch_c * esize;
    const bool inside = m_wave + lane::kBlock * MT <= p.M && n_wave + lane::kBlock * NT <= p.N;
    const bool fast = p.split_k == 1 && inside && p.c_vec8 && p.beta == 0.0f && !(p.bias && p.bias_along_m);
    auto out_type = [&](auto&& run) {
        if (p.c_dtype == DT_BF16) run(std::integral_constant<int, DT_BF16>{});
        else if (p.c_dtype == DT_F16) run(std::integral_constant<int, DT_F16>{});
        else run(std::integral_constant<int, DT_F32>{});
    };
    char* patch = lds;
    if constexpr (!OWN_PATCH) {
        wg::sync(wgp);  // every wave has finished with the operand slots: they become patches
        patch = lds + wave * wg::drain_patch_bytes(NT);
    }
    if constexpr (PAIRED) {
        if (fast) {
            // Common case: whole wave tile inside C, aligned rows, nothing to read back.  Every
            // lane holds runs of eight consecutive n of row lane % 16 of each block row and
            // finishes them itself.  A 16-bit result then passes through the patch once, to leave
            // as whole rows (full cache lines per store instruction, written past the caches'
            // retention: C is not read again by this kernel); an fp32 result goes straight out.
            constexpr int RUNS = NT / 2;
            const int n_lane = n_wave + 8 * (lane >> 4);
            const int64_t row_bytes = p.ldc * esize;
            const float* add_lane = add.first + (m_wave - q.m0 + (lane & 15)) * kPartialSide + (n_lane - q.n0);
            auto run = [&](auto out_c, auto bias_c) {
                constexpr int OUT = decltype(out_c)::value;
                constexpr bool BIAS = decltype(bias_c)::value;
                float bias[BIAS ? RUNS : 1][8];
                if constexpr (BIAS) {
#pragma unroll
                    for (int s = 0; s < RUNS; ++s) {
                        const f32x4 b0 = *reinterpret_cast<const f32x4*>(p.bias + n_lane + 32 * s);
                        const f32x4 b1 = *reinterpret_cast<const f32x4*>(p.bias + n_lane + 32 * s + 4);
                        bias[s][0] = b0[0]; bias[s][1] = b0[1]; bias[s][2] = b0[2]; bias[s][3] = b0[3];
                        bias[s][4] = b1[0]; bias[s][5] = b1[1]; bias[s][6] = b1[2]; bias[s][7] = b1[3];
                    }
                }
                auto addends = [&](int r_uniform, int c_uniform, f32x4& lo, f32x4& hi) {
                    if constexpr (ADD) {
                        const float* a = add_lane + r_uniform * kPartialSide + c_uniform;
                        for (int k = 0; k < add.count; ++k, a += kPartialTile) {
                            lo += *reinterpret_cast<const f32x4*>(a);
                            hi += *reinterpret_cast<const f32x4*>(a + 4);
                        }
                    }
                };
                if constexpr (OUT == DT_F32) {
                    char* lane_base = c_problem + (m_wave + (lane & 15)) * row_bytes + static_cast<int64_t>(n_lane) * 4;
                    wg::drain_pairs<MT, NT>(wv, acc, [&](int r_uniform, int c_uniform, f32x4 lo, f32x4 hi) {
                        addends(r_uniform, c_uniform, lo, hi);
                        grid::finish_run<OUT, BIAS>(lane_base + r_uniform * row_bytes + c_uniform * 4, p.alpha, bias[BIAS ? c_uniform / 32 : 0], lo, hi);
                    });
                } else {
                    char* wave_base = c_problem + m_wave * row_bytes + static_cast<int64_t>(n_wave) * 2;
                    wg::drain_rows<MT, NT>(
                        wv, acc, patch, lane,
                        [&](int r_uniform, int c_uniform, f32x4 lo, f32x4 hi) {
                            addends(r_uniform, c_uniform, lo, hi);
                            return grid::pack_run<OUT, BIAS>(p.alpha, bias[BIAS ? c_uniform / 32 : 0], lo, hi);
                        },
                        [&](int r_uniform, int r_lane, int byte_in_row, u32x4 piece) {
                            __builtin_nontemporal_store(piece, reinterpret_cast<u32x4*>(wave_base + (r_uniform + r_lane) * row_bytes + byte_in_row));
                        });
                }
            };
            out_type([&](auto out_c) {
                if (p.bias) run(out_c, std::true_type{});
                else run(out_c, std::false_type{});
            });
            return;
        }
    }
    if constexpr (PAIRED) {
        if (p.split_k > 1 && inside && p.p_vec) {  // raw partial sums of a K slice, the same way
            float* slab = p.partial + (static_cast<int64_t>(q.batch) * p.split_k + q.slice) * p.M * p.N;
            float* lane_base = slab + static_cast<int64_t>(m_wave + (lane & 15)) * p.N + n_wave + 8 * (lane >> 4);
            wg::drain_pairs<MT, NT>(wv, acc, [&](int r_uniform, int c_uniform, f32x4 lo, f32x4 hi) {
                float* dst = lane_base + static_cast<int64_t>(r_uniform) * p.N + c_uniform;
                *reinterpret_cast<f32x4*>(dst) = lo;
                *reinterpret_cast<f32x4*>(dst + 4) = hi;
            });
            return;
        }
    }
    auto drain_any = [&](auto&& sink) {
        if constexpr (OWN_PATCH) wg::drain<MT, NT, 16, 0, PAIRED>(wv, acc, patch, lane, sink);
        else wg::drain<MT, NT, wg::kDrainRows, 4, PAIRED>(wv, acc, patch, lane, sink);
    };
    if (p.split_k > 1) {
        float* slab = p.partial + (static_cast<int64_t>(q.batch) * p.split_k + q.slice) * p.M * p.N;
        drain_any([&](int r, int c, f32x4 v) { grid::partial4(p, slab, m_wave + r, n_wave + c, v); });
        return;
    }
    if constexpr (!PAIRED) {
        if (fast) {
            // Common case for the plain column order: the accumulators pass through the patch and
            // come back as runs of eight consecutive n.
            const int n_run = n_wave + 8 * (lane % (2 * NT));
            float bias[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            if (p.bias) {
                const f32x4 b0 = *reinterpret_cast<const f32x4*>(p.bias + n_run);
                const f32x4 b1 = *reinterpret_cast<const f32x4*>(p.bias + n_run + 4);
                bias[0] = b0[0]; bias[1] = b0[1]; bias[2] = b0[2]; bias[3] = b0[3];
                bias[4] = b1[0]; bias[5] = b1[1]; bias[6] = b1[2]; bias[7] = b1[3];
            }
            // the bias must be in registers before the first store is issued: stores and loads
            // share one in-order counter, so a later wait for the bias would wait for stores too
            wg::wait_counts<0, 15>();
            const int64_t row_bytes = p.ldc * esize;
            char* lane_base = c_problem + m_wave * row_bytes + static_cast<int64_t>(n_run) * esize;
            out_type([&](auto out_c) {
                constexpr int OUT = decltype(out_c)::value;
                auto sink = [&](int r_uniform, int r_lane, f32x4 lo, f32x4 hi) {
                    grid::finish_run<OUT, true>(lane_base + (r_uniform + r_lane) * row_bytes, p.alpha, bias, lo, hi);
                };
                if constexpr (OWN_PATCH) wg::drain_runs16<MT, NT>(wv, acc, patch, lane, sink);
                else wg::drain_runs<MT, NT>(wv, acc, patch, lane, sink);
            });
            return;
        }
    }
    drain_any([&](int r, int c, f32x4 v) {
        if constexpr (ADD) {
            const float* a = add.first + (m_wave - q.m0 + r) * kPartialSide + (n_wave - q.n0 + c);
            for (int k = 0; k < add.count; ++k, a += kPartialTile) v += *reinterpret_cast<const f32x4*>(a);
        }
        grid::finish4_any(p, c_problem, m_wave + r, n_wave + c, v);
    });
}

// One wave's accumulators (paired block columns) into a row-major 256 x 256 fp32 tile (`slot`),
// as runs of eight consecutive n straight from the registers.  row0 / col0: the wave tile's place.
template <typename TileT, int MT, int NT>
__device__ __forceinline__ void store_partial_tile(persp::Wave wv, const TileT& acc, int lane, float* slot, int row0, int col0)
{
    float* base = slot + (row0 + (lane & 15)) * kPartialSide + col0 + 8 * (lane >> 4);
    wg::drain_pairs<MT, NT>(wv, acc, [&](int r_uniform, int c_uniform, f32x4 lo, f32x4 hi) {
        float* dst = base + r_uniform * kPartialSide + c_uniform;
        *reinterpret_cast<f32x4*>(dst) = lo;
        *reinterpret_cast<f32x4*>(dst + 4) = hi;
    });
}

template <typename P, int BM, int BN, int BK, int WAVES_N>
__global__ __launch_bounds__(P::THREADS) void gemm_pipelined(const GemmParams p)
{
    const persp::Workgroup wgp = persp::Grid::at_kernel_entry().workgroup();
    __shared__ __attribute__((aligned(1024))) char lds[P::LDS_BYTES];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const Placement q = place<BM, BN>(p, blockIdx.x);

    constexpr int ES = P::ES;
    const char* a_tile = p.A + ES * (q.batch * p.batch_a + q.m0 * p.a_sm + q.k_begin * p.a_sk);
    const char* b_tile = p.B + ES * (q.batch * p.batch_b + q.n0 * p.b_sn + q.k_begin * p.b_sk);
    const int a_rows = p.M - q.m0 < BM ? p.M - q.m0 : BM;
    const int b_rows = p.N - q.n0 < BN ? p.N - q.n0 : BN;
    // pitch of a row of an LDS tile: a row of the matrix (K-contiguous operand) or a k-row
    const uint32_t a_ld = static_cast<uint32_t>(ES * (p.a_sk == 1 ? p.a_sm : p.a_sk));
    const uint32_t b_ld = static_cast<uint32_t>(ES * (p.b_sk == 1 ? p.b_sn : p.b_sk));

    typename P::tile_t acc;
    acc.clear();
    P::run(wgp, acc, a_tile, a_ld, a_rows, b_tile, b_ld, b_rows,
           (q.k_end - q.k_begin) / P::K_PER_STEP, lds, wave, lane);

    // The epilogue's per-lane addressing is computed after the K loop: kept live across it, it
    // would not fit in registers beside the accumulators and fragments.
    int lane_now = lane;
    asm volatile("" : "+v"(lane_now));
    epilogue<typename P::tile_t, P::MT, P::NT, false, P::PAIRED_N>(wgp, p, q, acc, q.m0 + (wave / WAVES_N) * P::WTM,
                                                                   q.n0 + (wave % WAVES_N) * P::WTN, lds, wave, lane_now);
}

// Persistent form for the 256x256x64 tile: workgroup w takes tiles w, w + gridDim.x, ...
// and streams their K steps through wg::PersistentPipe.  Every unit must have an even number
// of K steps, at least two (the host guarantees it).
template <typename T>
__global__ __launch_bounds__(256) void gemm_persistent(const GemmParams p, const int total)
{
    const persp::Workgroup wgp = persp::Grid::at_kernel_entry().workgroup();
    using P = wg::PersistentPipe<T>;
    __shared__ __attribute__((aligned(1024))) char lds[P::LDS_BYTES];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    auto source = [&](const Placement& q) {
        typename P::Source s;
        s.a = p.A + 2 * (q.batch * p.batch_a + q.m0 * p.a_sm + q.k_begin);
        s.b = p.B + 2 * (q.batch * p.batch_b + q.n0 * p.b_sn + q.k_begin);
        s.a_ld = static_cast<uint32_t>(2 * p.a_sm);
        s.b_ld = static_cast<uint32_t>(2 * p.b_sn);
        s.a_rows = p.M - q.m0 < P::BM ? p.M - q.m0 : P::BM;
        s.b_rows = p.N - q.n0 < P::BN ? p.N - q.n0 : P::BN;
        return s;
    };
    int tile = blockIdx.x;
    Placement cur = place<P::BM, P::BN>(p, tile), nxt = cur;
    P::run(
        wgp, lds, wave, lane, source(cur), (cur.k_end - cur.k_begin) / P::BK,
        [&](typename P::Source& s, int& ksteps) {
            if (tile + static_cast<int>(gridDim.x) >= total) return false;
            nxt = place<P::BM, P::BN>(p, tile + gridDim.x);
            s = source(nxt);
            ksteps = (nxt.k_end - nxt.k_begin) / P::BK;
            return true;
        },
        [&](typename P::tile_t& acc) {
            // The epilogue's per-lane addressing is recomputed for every tile: kept live across
            // the K loop it would not fit in registers beside the accumulators and fragments.
            int lane_now = lane;
            asm volatile("" : "+v"(lane_now));
            epilogue<typename P::tile_t, P::MT, P::NT, true, P::PAIRED_N>(wgp, p, cur, acc, cur.m0 + (wave / P::WAVES_N) * P::WTM,
                                                                          cur.n0 + (wave % P::WAVES_N) * P::WTN,
                                                                          lds + P::PATCH_BASE + wave * P::PATCH_BYTES, wave, lane_now);
        },
        [&]() {
            cur = nxt;
            tile += gridDim.x;
        });
}

// Stream-K form of the persistent kernel, for tile counts that fill the last round of compute
// units badly.  The K steps of all tiles form one sequence per die (the die's run of tiles in
// the locality order, tile after tile); the 32 workgroups of a die take equal, contiguous
// pieces of it in the order of a per-die ticket, so a workgroup computes the end of one tile,
// some whole tiles and the beginning of another.  A workgroup that does not reach the end of a
// tile writes its fp32 accumulators to its slot of the workspace and raises its flag; the one
// that reaches the end adds the slots of the tickets before it that worked on the tile, in
// ticket order (so the sum is the same in every run), and does the epilogue.  It only waits
// for lower tickets of its own die, and those workgroups are already running; as every piece
// is walked from its end, they wrote their slot at the very start.  The wait is
// bounded; a give-up sets the error word of the workspace.  p.partial is the workspace.
__global__ __launch_bounds__(256) void streamk_init(uint32_t* header)
{
    for (int i = threadIdx.x; i < kStreamKHeaderBytes / 4; i += blockDim.x) header[i] = 0u;
}

template <typename T>
__global__ __launch_bounds__(256) void gemm_streamk(const GemmParams p)
{
    const persp::Workgroup wgp = persp::Grid::at_kernel_entry().workgroup();
    using P = wg::PersistentPipe<T>;
    __shared__ __attribute__((aligned(1024))) char lds[P::LDS_BYTES];
    uint32_t* s_ticket = reinterpret_cast<uint32_t*>(lds + P::PATCH_BASE);  // the LDS is full: borrowed before the first epilogue
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    char* ws = reinterpret_cast<char*>(p.partial);
    uint32_t* header = reinterpret_cast<uint32_t*>(ws);
    uint32_t* flags = reinterpret_cast<uint32_t*>(ws + kStreamKFlagsOffset);
    const int die = blockIdx.x % grid::kDies, per_die = gridDim.x / grid::kDies;

    if (threadIdx.x == 0) *s_ticket = __hip_atomic_fetch_add(header + die, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    wg::sync(wgp);
    const int ticket = __builtin_amdgcn_readfirstlane(*s_ticket);  // 0 .. per_die-1 within the die
    wg::sync(wgp);                                                 // everyone has read it before the patch is used
    const int slot = die * per_die + ticket;
    float* my_slot = reinterpret_cast<float*>(ws + kStreamKHeaderBytes + slot * kStreamKSlotBytes);

    const int ksteps = p.K / P::BK;                                // even, the host guarantees it
    int first_tile, n_tiles;
    grid::die_run(die, p.tiles_m * p.tiles_n, first_tile, n_tiles);
    const int steps = n_tiles * ksteps;
    int piece = (steps + per_die - 1) / per_die;
    piece += piece & 1;                                            // pieces of an even number of K steps
    const int begin = ticket * piece, end = begin + piece < steps ? begin + piece : steps;
    if (begin >= end) return;                                      // uniform: the whole workgroup leaves

    struct Segment {
        int tile, k0, k1, m0, n0;                                  // K steps [k0, k1) of tile `tile` of the die's run
    };
    // the piece is walked from its end to its beginning (K ascending inside a segment): the part
    // of a tile that a lower ticket owns is then computed first thing, and is long there when
    // the ticket that ends the tile, last thing, comes to fetch it
    auto segment_ending_at = [&](int stop) {
        Segment g;
        g.tile = (stop - 1) / ksteps;
        g.k1 = stop - g.tile * ksteps;
        g.k0 = g.k1 - (stop - begin) > 0 ? g.k1 - (stop - begin) : 0;
        int tm, tn;
        grid::tile_at(first_tile + g.tile, p.tiles_m, p.tiles_n, tm, tn);
        g.m0 = tm * P::BM;
        g.n0 = tn * P::BN;
        return g;
    };
    auto source = [&](const Segment& g) {
        typename P::Source s;
        s.a = p.A + 2 * (g.m0 * p.a_sm + static_cast<int64_t>(g.k0) * P::BK);
        s.b = p.B + 2 * (g.n0 * p.b_sn + static_cast<int64_t>(g.k0) * P::BK);
        s.a_ld = static_cast<uint32_t>(2 * p.a_sm);
        s.b_ld = static_cast<uint32_t>(2 * p.b_sn);
        s.a_rows = p.M - g.m0 < P::BM ? p.M - g.m0 : P::BM;
        s.b_rows = p.N - g.n0 < P::BN ? p.N - g.n0 : P::BN;
        return s;
    };

    int stop = end;  // the part of the piece not yet computed is [begin, stop)
    Segment cur = segment_ending_at(stop), nxt = cur;
    P::run(
        wgp, lds, wave, lane, source(cur), cur.k1 - cur.k0,
        [&](typename P::Source& s, int& n) {
            const int next_stop = stop - (cur.k1 - cur.k0);
            if (next_stop <= begin) return false;
            nxt = segment_ending_at(next_stop);
            s = source(nxt);
            n = nxt.k1 - nxt.k0;
            return true;
        },
        [&](typename P::tile_t& acc) {
            int lane_now = lane;
            asm volatile("" : "+v"(lane_now));
            char* patch = lds + P::PATCH_BASE + wave * P::PATCH_BYTES;
            const int row0 = (wave / P::WAVES_N) * P::WTM, col0 = (wave % P::WAVES_N) * P::WTN;
            if (cur.k1 < ksteps) {
                // the tile is finished by a higher ticket: hand the partial sums over
                store_partial_tile<typename P::tile_t, P::MT, P::NT>(wgp.wave(), acc, lane_now, my_slot, row0, col0);
                __threadfence();
                wg::sync(wgp);
                if (threadIdx.x == 0) __hip_atomic_store(flags + slot, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
                return;
            }
            Addends add;
            if (cur.k0 > 0) {
                // the tile was begun by lower tickets: the one whose piece holds its first step,
                // and every ticket between that one and this
                const int first_ticket = (cur.tile * ksteps) / piece;
                for (int t = first_ticket; t < ticket; ++t) {
                    uint32_t polls = 0;
                    while (__hip_atomic_load(flags + die * per_die + t, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) == 0u) {
                        if (++polls > (1u << 22)) {
                            __hip_atomic_store(header + kStreamKErrorOffset / 4, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            break;
                        }
                        __builtin_amdgcn_s_sleep(2);
                    }
                }
                add.first = reinterpret_cast<const float*>(ws + kStreamKHeaderBytes + (die * per_die + first_ticket) * kStreamKSlotBytes);
                add.count = ticket - first_ticket;
            }
            Placement q;
            q.batch = 0; q.slice = 0; q.m0 = cur.m0; q.n0 = cur.n0; q.k_begin = 0; q.k_end = p.K;
            epilogue<typename P::tile_t, P::MT, P::NT, true, P::PAIRED_N, true>(wgp, p, q, acc, cur.m0 + (wave / P::WAVES_N) * P::WTM,
                                                                                cur.n0 + (wave % P::WAVES_N) * P::WTN,
                                                                                patch, wave, lane_now, add);
        },
        [&]() {
            stop -= cur.k1 - cur.k0;
            cur = nxt;
        });
}

template <typename T>
__global__ __launch_bounds__(256) void gemm_staged(const GemmParams p)
{
    const persp::Workgroup wgp = persp::Grid::at_kernel_entry().workgroup();
    using S = wg::Staged<T>;
    __shared__ __attribute__((aligned(1024))) char lds[S::LDS_BYTES];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const Placement q = place<S::BM, S::BN>(p, blockIdx.x);

    const char* a_tile = p.A + S::ES * (q.batch * p.batch_a + q.m0 * p.a_sm);
    const char* b_tile = p.B + S::ES * (q.batch * p.batch_b + q.n0 * p.b_sn);
    const int a_rows = p.M - q.m0 < S::BM ? p.M - q.m0 : S::BM;
    const int b_rows = p.N - q.n0 < S::BN ? p.N - q.n0 : S::BN;

    typename S::tile_t acc;
    acc.clear();
    S::run(wgp, acc, a_tile, p.a_sm, p.a_sk, a_rows, p.a_vec != 0, b_tile, p.b_sn, p.b_sk, b_rows, p.b_vec != 0,
           q.k_begin, q.k_end, lds, wave, lane);

    epilogue<typename S::tile_t, S::MT, S::NT>(wgp, p, q, acc, q.m0 + (wave >> 1) * S::WTM,
                                               q.n0 + (wave & 1) * S::WTN, lds, wave, lane);
}

// One thread per group of four consecutive n.  Slices are added in order
// 0, 1, ..., split_k-1 so the result does not depend on scheduling.
__global__ __launch_bounds__(256) void splitk_reduce(const GemmParams p)
{
    const int groups_n = (p.N + 3) / 4;
    const int64_t total = static_cast<int64_t>(p.batch) * p.M * groups_n;
    const int64_t slab = static_cast<int64_t>(p.M) * p.N;
    for (int64_t idx = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x; idx < total;
         idx += static_cast<int64_t>(gridDim.x) * blockDim.x) {
        const int g = static_cast<int>(idx % groups_n);
        const int64_t bm = idx / groups_n;
        const int m = static_cast<int>(bm % p.M);
        const int b = static_cast<int>(bm / p.M);
        const int n0 = 4 * g;
        f32x4 sum = {0.f, 0.f, 0.f, 0.f};
        const float* src = p.partial + static_cast<int64_t>(b) * p.split_k * slab + static_cast<int64_t>(m) * p.N + n0;
        for (int s = 0; s < p.split_k; ++s, src += slab) {
            if (p.p_vec && n0 + 3 < p.N) {
                sum += *reinterpret_cast<const f32x4*>(src);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (n0 + e < p.N) sum[e] += src[e];
            }
        }
        const int esize = p.c_dtype == DT_F32 ? 4 : 2;
        char* c_problem = p.C + static_cast<int64_t>(b) * p.batch_c * esize;
        grid::finish4_any(p, c_problem, m, n0, sum);
    }
}

template <typename P, int BM, int BN, int BK, int WAVES_N>
hipError_t launch_pipe(const GemmParams& p, int workgroups, hipStream_t stream)
{
    hipLaunchKernelGGL((gemm_pipelined<P, BM, BN, BK, WAVES_N>), dim3(workgroups), dim3(P::THREADS), 0, stream, p);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_pipe_config(int config, const GemmParams& p, int workgroups, hipStream_t stream)
{
    switch (config) {
    case 0: return launch_pipe<wg::Pipeline<T, 256, 256, 64, 2, 2, 2>, 256, 256, 64, 2>(p, workgroups, stream);
    case 1: return launch_pipe<wg::Pipeline<T, 128, 128, 64, 2, 2, 2>, 128, 128, 64, 2>(p, workgroups, stream);
    case 2: return launch_pipe<wg::Pipeline<T, 128, 128, 64, 2, 2, 2, true>, 128, 128, 64, 2>(p, workgroups, stream);
    case 3: return launch_pipe<wg::Pipeline<T, 128, 128, 64, 2, 2, 2, false, true>, 128, 128, 64, 2>(p, workgroups, stream);
    case 4: return launch_pipe<wg::Pipeline<T, 128, 128, 64, 2, 2, 2, true, true>, 128, 128, 64, 2>(p, workgroups, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t launch_pipelined(int config, int ab_dtype, const GemmParams& p, int workgroups, hipStream_t stream)
{
    if (ab_dtype == DT_F32) {  // fp32 operands: 128x128 tiles, the four layout pairs
        switch (config) {
        case 5: return launch_pipe<wg::Pipeline<f32_t, 128, 128, 64, 2, 2, 2>, 128, 128, 64, 2>(p, workgroups, stream);
        case 6: return launch_pipe<wg::Pipeline<f32_t, 128, 128, 64, 2, 2, 2, true>, 128, 128, 64, 2>(p, workgroups, stream);
        case 7: return launch_pipe<wg::Pipeline<f32_t, 128, 128, 64, 2, 2, 2, false, true>, 128, 128, 64, 2>(p, workgroups, stream);
        case 8: return launch_pipe<wg::Pipeline<f32_t, 128, 128, 64, 2, 2, 2, true, true>, 128, 128, 64, 2>(p, workgroups, stream);
        default: return hipErrorInvalidValue;
        }
    }
    return ab_dtype == DT_BF16 ? launch_pipe_config<bf16_t>(config, p, workgroups, stream)
                               : launch_pipe_config<f16_t>(config, p, workgroups, stream);
}

hipError_t launch_streamk(int ab_dtype, const GemmParams& p, hipStream_t stream)
{
    hipLaunchKernelGGL(streamk_init, dim3(1), dim3(256), 0, stream, reinterpret_cast<uint32_t*>(p.partial));
    if (ab_dtype == DT_BF16)
        hipLaunchKernelGGL(gemm_streamk<bf16_t>, dim3(kStreamKWorkgroups), dim3(256), 0, stream, p);
    else
        hipLaunchKernelGGL(gemm_streamk<f16_t>, dim3(kStreamKWorkgroups), dim3(256), 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_persistent(int ab_dtype, const GemmParams& p, int total, int workgroups, hipStream_t stream)
{
    if (ab_dtype == DT_BF16)
        hipLaunchKernelGGL(gemm_persistent<bf16_t>, dim3(workgroups), dim3(256), 0, stream, p, total);
    else
        hipLaunchKernelGGL(gemm_persistent<f16_t>, dim3(workgroups), dim3(256), 0, stream, p, total);
    return hipGetLastError();
}

hipError_t launch_staged(int ab_dtype, const GemmParams& p, int workgroups, hipStream_t stream)
{
    if (ab_dtype == DT_BF16)
        hipLaunchKernelGGL(gemm_staged<bf16_t>, dim3(workgroups), dim3(256), 0, stream, p);
    else if (ab_dtype == DT_F16)
        hipLaunchKernelGGL(gemm_staged<f16_t>, dim3(workgroups), dim3(256), 0, stream, p);
    else
        hipLaunchKernelGGL(gemm_staged<f32_t>, dim3(workgroups), dim3(256), 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_reduce(const GemmParams& p, hipStream_t stream)
{
    const int64_t total = static_cast<int64_t>(p.batch) * p.M * ((p.N + 3) / 4);
    int64_t blocks = (total + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(splitk_reduce, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, stream, p);
    return hipGetLastError();
}

}  // namespace prism
