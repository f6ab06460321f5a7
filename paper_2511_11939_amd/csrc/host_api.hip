// Host side of the C ABI: argument validation, the choice of kernel, tile shape
// and K split, and the launches.  No arithmetic of the matrix product happens
// here; everything numeric runs in the device kernels.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>

#include "../../include/prism_gemm.h"
#include "grid.hpp"
#include "launch.hpp"

namespace {

using prism::GemmParams;

constexpr int kComputeUnits = 256;
constexpr int kPersistentMaxSteps = 16;  // longest K loop (in K steps) the persistent kernel is chosen for
constexpr int kMaxSplit = 64;
constexpr int kVeryLongK = 512;              // K steps from which few 256x256 tiles with many slices beat small tiles
constexpr int kMinSliceStepsStaged = 8;      // shortest K loop (in K steps) a slice of the staged kernel gets
constexpr int64_t kIntMax = 2147483647;

struct Problem {
    GemmParams p;
    prism_gemm_plan_t plan;
    int ab_dtype;
    int pipe_config;  // index into kPipeConfigs when plan.kernel is 2 or 3
    int total_units;  // (tile, unit) pairs the persistent kernel walks
};

bool valid_dtype_ab(int v) { return v == PRISM_DTYPE_BF16 || v == PRISM_DTYPE_F16 || v == PRISM_DTYPE_F32; }
bool valid_dtype_c(int v) { return v == PRISM_DTYPE_BF16 || v == PRISM_DTYPE_F16 || v == PRISM_DTYPE_F32; }
bool valid_layout(int v) { return v == PRISM_ROW_MAJOR || v == PRISM_COL_MAJOR; }
bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Elements spanned by a rows x cols matrix with leading dimension ld.
int64_t span(int layout, int64_t rows, int64_t cols, int64_t ld)
{
    if (rows == 0 || cols == 0) return 0;
    return layout == PRISM_ROW_MAJOR ? (rows - 1) * ld + cols : (cols - 1) * ld + rows;
}

bool overlaps(const void* a, int64_t a_bytes, const void* b, int64_t b_bytes)
{
    if (!a || !b || a_bytes <= 0 || b_bytes <= 0) return false;
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
    return a0 < b0 + static_cast<uintptr_t>(b_bytes) && b0 < a0 + static_cast<uintptr_t>(a_bytes);
}

// Hooks for tests and experiments, read from the environment once (at the first call that
// needs them, or again on prism_reread_environment) and kept:
//   PRISM_GEMM_CONFIG=<index>  pins the pipeline's tile configuration (0: 256x256, 1: 128x128)
//   PRISM_PERSISTENT=0|1       never / whenever possible use the persistent kernel
//   PRISM_LOG=1                one line per launch on stderr: problem, kernel, tile, split
struct Hooks {
    int pipe_config = -1;  // -1: the library decides
    int persistent = -1;   // -1: the library decides, 0: never, 1: whenever possible
    bool log = false;
};
Hooks g_hooks;
bool g_hooks_loaded = false;
std::mutex g_hooks_mutex;

void load_hooks_locked()
{
    Hooks h;
    if (const char* e = std::getenv("PRISM_GEMM_CONFIG"); e && *e) {
        const int v = std::atoi(e);
        if (v >= 0 && v < prism::kNumPipeConfigs) h.pipe_config = v;
    }
    if (const char* e = std::getenv("PRISM_PERSISTENT"); e && (e[0] == '0' || e[0] == '1')) h.persistent = e[0] - '0';
    if (const char* e = std::getenv("PRISM_LOG"); e && e[0] == '1') h.log = true;
    g_hooks = h;
    g_hooks_loaded = true;
}

Hooks hooks()
{
    std::lock_guard<std::mutex> lock(g_hooks_mutex);
    if (!g_hooks_loaded) load_hooks_locked();
    return g_hooks;
}

// Validates everything, normalises to a row-major C and chooses the launch.
prism_status_t make_problem(const prism_gemm_desc_t* d, int64_t M, int64_t N, int64_t K,
                            const void* A, int64_t lda, int64_t strideA, const void* B, int64_t ldb,
                            int64_t strideB, const void* C, int64_t ldc, int64_t strideC, int64_t batch,
                            bool need_pointers, Problem* out)
{
    if (!d || !out) return PRISM_ERR_INVALID_ARG;
    if (!valid_dtype_ab(d->ab_dtype) || !valid_dtype_c(d->c_dtype) || !valid_layout(d->layout_a) ||
        !valid_layout(d->layout_b) || !valid_layout(d->layout_c))
        return PRISM_ERR_UNSUPPORTED;
    if (d->ab_dtype == PRISM_DTYPE_F32 && d->c_dtype != PRISM_DTYPE_F32) return PRISM_ERR_UNSUPPORTED;
    if (d->reserved != 0) return PRISM_ERR_INVALID_ARG;
    if (M < 0 || N < 0 || K < 0 || batch < 0 || d->split_k < 0) return PRISM_ERR_INVALID_ARG;
    if (M > kIntMax || N > kIntMax || K > kIntMax - 64 || batch > kIntMax) return PRISM_ERR_INVALID_ARG;
    if (lda < 1 || ldb < 1 || ldc < 1) return PRISM_ERR_INVALID_ARG;
    if (lda < (d->layout_a == PRISM_ROW_MAJOR ? K : M)) return PRISM_ERR_INVALID_ARG;
    if (ldb < (d->layout_b == PRISM_ROW_MAJOR ? N : K)) return PRISM_ERR_INVALID_ARG;
    if (ldc < (d->layout_c == PRISM_ROW_MAJOR ? N : M)) return PRISM_ERR_INVALID_ARG;
    if (!(d->alpha == d->alpha) || !(d->beta == d->beta)) return PRISM_ERR_INVALID_ARG;  // NaN scales

    std::memset(out, 0, sizeof(*out));
    const Hooks hk = hooks();
    prism_gemm_plan_t& plan = out->plan;
    plan.split_k = 1;
    const bool empty = M == 0 || N == 0 || batch == 0;
    if (empty) return PRISM_OK;  // plan.kernel == 0: nothing to do

    const int64_t c_span = span(d->layout_c, M, N, ldc);
    const int64_t a_span = span(d->layout_a, M, K, lda), b_span = span(d->layout_b, K, N, ldb);
    const int c_esize = d->c_dtype == PRISM_DTYPE_F32 ? 4 : 2;
    const int ab_esize = d->ab_dtype == PRISM_DTYPE_F32 ? 4 : 2;
    const int epc = 16 / ab_esize;  // operand elements per 16-byte chunk
    if (need_pointers) {
        if (!C || (K > 0 && (!A || !B))) return PRISM_ERR_INVALID_ARG;
    }
    if (batch > 1) {
        const int64_t sc = strideC < 0 ? -strideC : strideC;
        if (sc < c_span) return PRISM_ERR_INVALID_ARG;  // C matrices of the batch would overlap
    }
    if (batch == 1 || (strideA >= 0 && strideB >= 0 && strideC >= 0)) {
        // C must not share memory with A or B (checked over the whole batch extent)
        const int64_t nb = batch - 1;
        const int64_t c_bytes = (nb * strideC + c_span) * c_esize;
        if (overlaps(C, c_bytes, A, (nb * strideA + a_span) * ab_esize) ||
            overlaps(C, c_bytes, B, (nb * strideB + b_span) * ab_esize))
            return PRISM_ERR_INVALID_ARG;
    }

    // ---- normalise: a column-major C is the row-major C^T = B^T A^T
    GemmParams& p = out->p;
    int64_t a_sm = d->layout_a == PRISM_ROW_MAJOR ? lda : 1, a_sk = d->layout_a == PRISM_ROW_MAJOR ? 1 : lda;
    int64_t b_sk = d->layout_b == PRISM_ROW_MAJOR ? ldb : 1, b_sn = d->layout_b == PRISM_ROW_MAJOR ? 1 : ldb;
    if (d->layout_c == PRISM_COL_MAJOR) {
        plan.swapped = 1;
        p.A = static_cast<const char*>(B); p.a_sm = b_sn; p.a_sk = b_sk; p.batch_a = strideB;
        p.B = static_cast<const char*>(A); p.b_sn = a_sm; p.b_sk = a_sk; p.batch_b = strideA;
        p.M = static_cast<int>(N); p.N = static_cast<int>(M);
        p.bias_along_m = 1;
    } else {
        p.A = static_cast<const char*>(A); p.a_sm = a_sm; p.a_sk = a_sk; p.batch_a = strideA;
        p.B = static_cast<const char*>(B); p.b_sn = b_sn; p.b_sk = b_sk; p.batch_b = strideB;
        p.M = static_cast<int>(M); p.N = static_cast<int>(N);
        p.bias_along_m = 0;
    }
    p.K = static_cast<int>(K);
    p.C = static_cast<char*>(const_cast<void*>(C));
    p.ldc = ldc;
    p.batch_c = strideC;
    p.batch = static_cast<int>(batch);
    p.bias = d->bias;
    p.alpha = d->alpha;
    p.beta = d->beta;
    p.c_dtype = d->c_dtype;
    out->ab_dtype = d->ab_dtype;

    // ---- alignment facts
    const bool a_kfast = p.a_sk == 1, b_kfast = p.b_sk == 1;
    p.a_vec = a_kfast && aligned(p.A, 16) && p.a_sm % epc == 0 && (p.batch == 1 || p.batch_a % epc == 0);
    p.b_vec = b_kfast && aligned(p.B, 16) && p.b_sn % epc == 0 && (p.batch == 1 || p.batch_b % epc == 0);
    const size_t c_align = 4 * static_cast<size_t>(c_esize);
    p.c_vec = aligned(p.C, c_align) && p.ldc % 4 == 0 && (p.batch == 1 || p.batch_c % 4 == 0) &&
              (!p.bias || p.bias_along_m || aligned(p.bias, 4));
    p.p_vec = p.N % 4 == 0 && aligned(d->workspace, 16);
    p.c_vec8 = aligned(p.C, 16) && p.ldc % 8 == 0 && (p.batch == 1 || p.batch_c % 8 == 0) &&
               (!p.bias || aligned(p.bias, 16));

    if (K == 0) {  // C <- bias + beta*C: only the epilogue kernel runs
        plan.kernel = 0;
        p.split_k = 0;
        p.tiles_m = p.tiles_n = 0;
        return PRISM_OK;
    }

    // ---- kernel and tile shape
    const int64_t step_k = 128 / ab_esize;  // a K step is 128 bytes of every operand row
    const int64_t ksteps = ceil_div(K, step_k);
    const bool pitch_ok = p.a_sm < (int64_t{1} << 21) && p.b_sn < (int64_t{1} << 21) && p.a_sk < (int64_t{1} << 21) &&
                          p.b_sk < (int64_t{1} << 21);
    // An operand contiguous along m (column-major A) or n (row-major B): whole, aligned 16-byte
    // chunks of every k-row
    const bool a_along_m = p.a_sm == 1 && p.a_sk != 1 && aligned(p.A, 16) && p.a_sk % epc == 0 && p.M % epc == 0 &&
                           (p.batch == 1 || p.batch_a % epc == 0);
    const bool b_along_n = p.b_sn == 1 && p.b_sk != 1 && aligned(p.B, 16) && p.b_sk % epc == 0 && p.N % epc == 0 &&
                           (p.batch == 1 || p.batch_b % epc == 0);
    const bool pipe_ok = (p.a_vec || a_along_m) && (p.b_vec || b_along_n) && K % step_k == 0 && pitch_ok;
    int tile_m = prism::kStagedTileM, tile_n = prism::kStagedTileN, waves = prism::kStagedWaves;
    plan.kernel = 1;
    if (pipe_ok) {
        plan.kernel = 2;
        int cfg = hk.pipe_config;
        if (cfg > 1) cfg = -1;  // the hook names a tile size (0: 256x256, 1: 128x128)
        if (cfg < 0) {
            // Big tiles when they give at least half of the compute units a workgroup, or for a
            // very long K (the split then needs fewer slices); else small tiles, two workgroups
            // per compute unit.  Measured: 128x128 tiles win on square problems up to 2560^3
            // (2048^3: 26 against 40 us) and on 1024x1024x8192 (30 against 38 us), 256x256 tiles
            // from 3072^3 on and on 1024x1024x32768.
            const int64_t big = ceil_div(p.M, 256) * ceil_div(p.N, 256) * batch;
            cfg = (big >= kComputeUnits / 2 || ksteps >= kVeryLongK) ? 0 : 1;
        }
        // an operand that is not K-contiguous: 128x128 tiles, that operand kept as k-rows in LDS
        if (!p.a_vec || !p.b_vec) cfg = !p.a_vec ? (!p.b_vec ? 4 : 3) : 2;
        // fp32 operands: 128x128 tiles in all four layout pairs
        if (ab_esize == 4) cfg = 5 + (p.b_vec ? 0 : 1) + (p.a_vec ? 0 : 2);
        out->pipe_config = cfg;
        tile_m = prism::kPipeConfigs[cfg].tile_m;
        tile_n = prism::kPipeConfigs[cfg].tile_n;
        waves = prism::kPipeConfigs[cfg].waves;
    }
    const int64_t tiles_m = ceil_div(p.M, tile_m), tiles_n = ceil_div(p.N, tile_n);
    if (tiles_m * tiles_n > kIntMax / 64 || tiles_m * tiles_n * batch > kIntMax / 64) return PRISM_ERR_INVALID_ARG;

    // ---- K split: explicit request, or enough slices to give every compute unit a workgroup
    int64_t want = d->split_k;
    const int64_t units = tiles_m * tiles_n * batch;
    const size_t slab_bytes = static_cast<size_t>(batch) * p.M * p.N * sizeof(float);
    if (want == 0) {
        want = 1;
        // A split costs a round trip of fp32 partial sums and a second kernel: it pays only for
        // a long K loop, and every slice must keep a K loop of its own.  Small tiles run two
        // workgroups per compute unit, so they are split until there are about twice as many
        // workgroups as compute units (measured: 512x512x16384 23 us with 16 slices, 28 with
        // 8 or 32).
        const bool small_tiles = plan.kernel != 2 || out->pipe_config != 0;
        const int64_t slots = small_tiles ? 2 * kComputeUnits : kComputeUnits;
        // (a K step of fp32 operands holds four times the matrix instructions of a 16-bit one)
        const bool short_steps = plan.kernel == 2 && ab_esize == 2;
        const int64_t min_slice = !short_steps ? kMinSliceStepsStaged : (small_tiles ? 16 : 32);
        const int64_t min_k = !short_steps ? 4 * kMinSliceStepsStaged : 64;
        if (units * 2 <= slots && ksteps >= min_k) {
            want = slots / units;
            if (want > ksteps / min_slice) want = ksteps / min_slice;
            if (small_tiles && want > 32) want = 32;
            if (want > kMaxSplit) want = kMaxSplit;
            if (want < 1) want = 1;
        }
    }
    if (want > ksteps) want = ksteps;
    int64_t slice_steps = ceil_div(ksteps, want);
    int64_t split = ceil_div(ksteps, slice_steps);  // no empty slices
    size_t ws_need = split > 1 ? slab_bytes * static_cast<size_t>(split) : 0;
    if (split > 1 && need_pointers && (!d->workspace || d->workspace_bytes < ws_need)) {
        if (d->split_k > 1) return PRISM_ERR_WORKSPACE;
        split = 1; slice_steps = ksteps; ws_need = 0;  // library's own choice: fall back quietly
    }
    p.split_k = static_cast<int>(split);
    p.k_slice = static_cast<int>(slice_steps * step_k);
    p.partial = split > 1 ? static_cast<float*>(d->workspace) : nullptr;
    p.tiles_m = static_cast<int>(tiles_m);
    p.tiles_n = static_cast<int>(tiles_n);

    plan.tile_m = tile_m; plan.tile_n = tile_n; plan.waves = waves;
    plan.tile_k = plan.kernel >= 2 ? prism::kPipeConfigs[out->pipe_config].tile_k : static_cast<int32_t>(step_k);
    plan.split_k = static_cast<int32_t>(split);
    plan.tiles_m = tiles_m; plan.tiles_n = tiles_n;
    plan.workgroups = units * split;
    // More (tile, unit) pairs than compute units, each with a short K loop: 256x256 tiles whose
    // slices all have two or more K steps go to the persistent kernel, one workgroup per
    // compute unit walking several pairs with the next pair's operands loaded under the tail of
    // the current one.  With long K loops the start of a tile is a small share of its time and
    // the hardware's own dealing of workgroups to free compute units balances better than the
    // fixed assignment of the persistent kernel (measured).
    {
        const bool never = hk.persistent == 0, always = hk.persistent == 1;
        const int64_t last_slice_steps = ksteps - (split - 1) * slice_steps;
        const bool possible = plan.kernel == 2 && out->pipe_config == 0 && slice_steps >= 2 && last_slice_steps >= 2 &&
                              slice_steps % 2 == 0 && last_slice_steps % 2 == 0;  // it walks K two steps at a time
        const bool pays = units * split > kComputeUnits && slice_steps <= kPersistentMaxSteps;
        if (possible && !never && (always || pays)) {
            plan.kernel = 3;
            out->total_units = static_cast<int>(units * split);
            if (plan.workgroups > kComputeUnits) plan.workgroups = kComputeUnits;
        }
    }
    plan.workspace_bytes = ws_need;
    if (plan.workgroups > kIntMax) return PRISM_ERR_INVALID_ARG;
    return PRISM_OK;
}

prism_status_t run(const Problem& pr, hipStream_t stream)
{
    const GemmParams& p = pr.p;
    if (p.M == 0 || p.N == 0 || p.batch == 0) return PRISM_OK;
    hipError_t e = hipSuccess;
    if (pr.plan.kernel == 3)
        e = prism::launch_persistent(pr.ab_dtype, p, pr.total_units, static_cast<int>(pr.plan.workgroups), stream);
    else if (pr.plan.kernel == 2)
        e = prism::launch_pipelined(pr.pipe_config, pr.ab_dtype, p, static_cast<int>(pr.plan.workgroups), stream);
    else if (pr.plan.kernel == 1)
        e = prism::launch_staged(pr.ab_dtype, p, static_cast<int>(pr.plan.workgroups), stream);
    if (e != hipSuccess) return PRISM_ERR_LAUNCH;
    if (hooks().log) {
        static const char* const names[] = {"none", "gemm_staged", "gemm_pipelined", "gemm_persistent"};
        std::fprintf(stderr, "prism_gemm: M=%d N=%d K=%d batch=%d%s kernel=%s tile=%dx%dx%d waves=%d split_k=%d workgroups=%lld\n",
                     p.M, p.N, p.K, p.batch, pr.plan.swapped ? " (run as C^T = B^T A^T)" : "",
                     names[pr.plan.kernel >= 0 && pr.plan.kernel <= 3 ? pr.plan.kernel : 0], pr.plan.tile_m, pr.plan.tile_n,
                     pr.plan.tile_k, pr.plan.waves, pr.plan.split_k, static_cast<long long>(pr.plan.workgroups));
    }
    if (p.split_k != 1) {  // K == 0 (split_k == 0) or a real split: the reduction writes C
        e = prism::launch_reduce(p, stream);
        if (e != hipSuccess) return PRISM_ERR_LAUNCH;
    }
    return PRISM_OK;
}

}  // namespace

extern "C" {

prism_status_t prism_gemm_batched(const prism_gemm_desc_t* d, int64_t M, int64_t N, int64_t K,
                                  const void* A, int64_t lda, int64_t strideA, const void* B, int64_t ldb,
                                  int64_t strideB, void* C, int64_t ldc, int64_t strideC, int64_t batch,
                                  void* hip_stream)
{
    Problem pr;
    const prism_status_t s =
        make_problem(d, M, N, K, A, lda, strideA, B, ldb, strideB, C, ldc, strideC, batch, true, &pr);
    if (s != PRISM_OK) return s;
    return run(pr, static_cast<hipStream_t>(hip_stream));
}

prism_status_t prism_gemm_batched_stamped(const prism_gemm_desc_t* d, int64_t M, int64_t N, int64_t K,
                                          const void* A, int64_t lda, int64_t strideA, const void* B, int64_t ldb,
                                          int64_t strideB, void* C, int64_t ldc, int64_t strideC, int64_t batch,
                                          uint64_t* stamps, size_t stamp_bytes, void* hip_stream)
{
    Problem pr;
    const prism_status_t s =
        make_problem(d, M, N, K, A, lda, strideA, B, ldb, strideB, C, ldc, strideC, batch, true, &pr);
    if (s != PRISM_OK) return s;
    if (pr.plan.kernel != 2) return PRISM_ERR_UNSUPPORTED;  // only the pipelined kernel leaves stamps
    if (!stamps || reinterpret_cast<uintptr_t>(stamps) % 8 != 0) return PRISM_ERR_INVALID_ARG;
    if (stamp_bytes < static_cast<size_t>(pr.plan.workgroups) * PRISM_STAMP_BYTES_PER_WORKGROUP) return PRISM_ERR_WORKSPACE;
    static_assert(PRISM_STAMP_BYTES_PER_WORKGROUP == prism::kStampWords * sizeof(uint64_t), "stamp layout");
    pr.p.stamps = stamps;
    return run(pr, static_cast<hipStream_t>(hip_stream));
}

prism_status_t prism_gemm(const prism_gemm_desc_t* d, int64_t M, int64_t N, int64_t K, const void* A,
                          int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc, void* hip_stream)
{
    return prism_gemm_batched(d, M, N, K, A, lda, 0, B, ldb, 0, C, ldc, 0, 1, hip_stream);
}

prism_status_t prism_gemm_plan(const prism_gemm_desc_t* d, int64_t M, int64_t N, int64_t K, const void* A,
                               int64_t lda, int64_t strideA, const void* B, int64_t ldb, int64_t strideB,
                               const void* C, int64_t ldc, int64_t strideC, int64_t batch,
                               prism_gemm_plan_t* plan_out)
{
    if (!plan_out) return PRISM_ERR_INVALID_ARG;
    Problem pr;
    const prism_status_t s =
        make_problem(d, M, N, K, A, lda, strideA, B, ldb, strideB, C, ldc, strideC, batch, false, &pr);
    if (s != PRISM_OK) return s;
    *plan_out = pr.plan;
    return PRISM_OK;
}

prism_status_t prism_gemm_workspace_size(const prism_gemm_desc_t* d, int64_t M, int64_t N, int64_t K,
                                         int64_t batch, size_t* bytes_out)
{
    if (!d || !bytes_out) return PRISM_ERR_INVALID_ARG;
    // Leading dimensions and strides do not influence the split; use the packed ones.
    const int64_t lda = d->layout_a == PRISM_ROW_MAJOR ? K : M, ldb = d->layout_b == PRISM_ROW_MAJOR ? N : K;
    const int64_t ldc = d->layout_c == PRISM_ROW_MAJOR ? N : M;
    Problem pr;
    const prism_status_t s =
        make_problem(d, M, N, K, nullptr, lda < 1 ? 1 : lda, M * K, nullptr, ldb < 1 ? 1 : ldb, K * N, nullptr,
                     ldc < 1 ? 1 : ldc, M * N, batch, false, &pr);
    if (s != PRISM_OK) return s;
    *bytes_out = pr.plan.workspace_bytes;
    return PRISM_OK;
}

prism_status_t prism_sched_map(int64_t wg, int64_t tiles_m, int64_t tiles_n, int64_t units, int64_t* tile_m,
                               int64_t* tile_n, int64_t* unit)
{
    if (!tile_m || !tile_n || !unit || tiles_m < 1 || tiles_n < 1 || units < 1) return PRISM_ERR_INVALID_ARG;
    if (tiles_m > kIntMax || tiles_n > kIntMax || units > kIntMax) return PRISM_ERR_INVALID_ARG;
    if (tiles_m * tiles_n > kIntMax || tiles_m * tiles_n * units > kIntMax) return PRISM_ERR_INVALID_ARG;
    if (wg < 0 || wg >= tiles_m * tiles_n * units) return PRISM_ERR_INVALID_ARG;
    const prism::grid::TileCoord c = prism::grid::schedule(static_cast<int>(wg), static_cast<int>(tiles_m),
                                                           static_cast<int>(tiles_n), static_cast<int>(units));
    *tile_m = c.tile_m;
    *tile_n = c.tile_n;
    *unit = c.unit;
    return PRISM_OK;
}

const char* prism_status_string(prism_status_t s)
{
    switch (s) {
    case PRISM_OK: return "PRISM_OK";
    case PRISM_ERR_INVALID_ARG: return "PRISM_ERR_INVALID_ARG";
    case PRISM_ERR_UNSUPPORTED: return "PRISM_ERR_UNSUPPORTED";
    case PRISM_ERR_WORKSPACE: return "PRISM_ERR_WORKSPACE";
    case PRISM_ERR_LAUNCH: return "PRISM_ERR_LAUNCH";
    }
    return "PRISM_ERR_UNKNOWN";
}

int prism_version(void) { return 200; }

void prism_reread_environment(void)
{
    {
        std::lock_guard<std::mutex> lock(g_hooks_mutex);
        load_hooks_locked();
    }
    prism::scan_reread_environment();
}

}  // extern "C"
