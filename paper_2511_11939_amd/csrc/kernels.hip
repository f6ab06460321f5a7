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
    q.batch = p.split_k == 1 ? c.unit : grid::uniform_quotient(c.unit, p.split_k);
    q.slice = c.unit - q.batch * p.split_k;
    q.m0 = c.tile_m * BM;
    q.n0 = c.tile_n * BN;
    q.k_begin = q.slice * p.k_slice;
    q.k_end = q.k_begin + p.k_slice < p.K ? q.k_begin + p.k_slice : p.K;
    // uniform values: held in scalar registers, so that the tile addresses derived from them
    // are computed by the scalar unit
    q.batch = __builtin_amdgcn_readfirstlane(q.batch);
    q.slice = __builtin_amdgcn_readfirstlane(q.slice);
    q.m0 = __builtin_amdgcn_readfirstlane(q.m0);
    q.n0 = __builtin_amdgcn_readfirstlane(q.n0);
    q.k_begin = __builtin_amdgcn_readfirstlane(q.k_begin);
    q.k_end = __builtin_amdgcn_readfirstlane(q.k_end);
    return q;
}

// Accumulators of one wave tile -> C or the split-K scratch.
// OWN_PATCH false: the patches reuse the operand slots; workgroup-collective, every wave
// must call it (it starts with a barrier that retires the slots).  OWN_PATCH true: `patch`
// is this wave's private 16-row patch outside the slots; no barrier, 16 rows per pass.
template <typename TileT, int MT, int NT, bool OWN_PATCH = false, bool PAIRED = false>
__device__ __forceinline__ void epilogue(persp::Workgroup wgp, const GemmParams& p, const Placement& q, const TileT& acc,
                                         int m_wave, int n_wave, char* lds, int wave, int lane)
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
                if constexpr (OUT == DT_F32) {
                    char* lane_base = c_problem + (m_wave + (lane & 15)) * row_bytes + static_cast<int64_t>(n_lane) * 4;
                    wg::drain_pairs<MT, NT>(wv, acc, [&](int r_uniform, int c_uniform, f32x4 lo, f32x4 hi) {
                        grid::finish_run<OUT, BIAS>(lane_base + r_uniform * row_bytes + c_uniform * 4, p.alpha, bias[BIAS ? c_uniform / 32 : 0], lo, hi);
                    });
                } else {
                    char* wave_base = c_problem + m_wave * row_bytes + static_cast<int64_t>(n_wave) * 2;
                    wg::drain_rows<MT, NT>(
                        wv, acc, patch, lane,
                        [&](int r_uniform, int c_uniform, f32x4 lo, f32x4 hi) {
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
    drain_any([&](int r, int c, f32x4 v) { grid::finish4_any(p, c_problem, m_wave + r, n_wave + c, v); });
}

template <typename P, int BM, int BN, int BK, int WAVES_N>
__global__ __launch_bounds__(P::THREADS) void gemm_pipelined(const GemmParams p)
{
    const persp::Workgroup wgp = persp::Grid::at_kernel_entry().workgroup();
    __shared__ __attribute__((aligned(1024))) char lds[P::LDS_BYTES];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    stamp(p.stamps, STAMP_ENTRY);
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
           (q.k_end - q.k_begin) / P::K_PER_STEP, lds, wave, lane, p.stamps);
    stamp(p.stamps, STAMP_K_LOOP_DONE);

    // The epilogue's per-lane addressing is computed after the K loop: kept live across it, it
    // would not fit in registers beside the accumulators and fragments.
    int lane_now = lane;
    asm volatile("" : "+v"(lane_now));
    epilogue<typename P::tile_t, P::MT, P::NT, false, P::PAIRED_N>(wgp, p, q, acc, q.m0 + (wave / WAVES_N) * P::WTM,
                                                                   q.n0 + (wave % WAVES_N) * P::WTN, lds, wave, lane_now);
    if (p.stamps) {  // the last stamp is taken when this wave's stores have been acknowledged
        wg::wait_counts<0, 0>();
        stamp(p.stamps, STAMP_STORES_DONE);
    }
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
