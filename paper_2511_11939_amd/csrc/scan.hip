// Single-pass inclusive prefix sum over uint32 with decoupled look-back (the paper's scan
// benchmark, section 6.1 and its code appendix `scan_kernel`; the scheme is Merrill and
// Garland's).  Layered like the GEMM code: lane-level sums of four consecutive elements,
// a wave-level scan with cross-lane moves, a workgroup-level combine through LDS, and a
// grid-level chain of per-tile status words.
//
// What differs from the paper's kernel, written for 32-wide warps and 16 warps per block:
// its tile of 16384 elements is handled by four 64-wide waves, every lane owning sixteen
// 16-byte vectors held in registers (loads and stores are whole cache lines per wave, and
// the data never passes through LDS); the sixteen per-lane partial sums are scanned
// together, so a tile needs one barrier for the combine and one for the prefix;
// the look-back is done by a whole wave, 64 predecessors per poll; a status word carries
// flag and value in one 64-bit store, so no fence separates them.
#include <hip/hip_runtime.h>

#include <cstdlib>
#include <mutex>

#include "../../include/prism_scan.h"
#include "launch.hpp"
#include "persp.hpp"

namespace prism {
namespace scan {

constexpr int kThreads = 256, kWaves = 4, kVec = 4, kChunks = 16;
constexpr int kTile = kThreads * kVec * kChunks;  // 16384 elements per workgroup, the tile of the paper's kernel
constexpr int64_t kMaxN = int64_t{1} << 43;
constexpr size_t kHeaderBytes = 64;               // [0] tile counter, [1] error word
constexpr uint32_t kDefaultSpinLimit = 1u << 20;  // polls of one status word; a real wait is a few dozen

enum : uint32_t { kInvalid = 0, kAggregate = 1, kPrefix = 2 };

using u32x4 = __attribute__((ext_vector_type(4))) uint32_t;

__device__ __forceinline__ uint64_t pack(uint32_t flag, uint32_t value)
{
    return (static_cast<uint64_t>(flag) << 32) | value;
}

// ---- workgroup level
__device__ __forceinline__ void sync(persp::Workgroup) { __syncthreads(); }

// ---- wave level: all 64 lanes converged -------------------------------------------------
// Inclusive sum over the lanes of a wave (lane l receives the sum of lanes 0..l), with the
// data-parallel-primitive lane moves of the vector ALU instead of LDS permutes: four shifts
// inside each row of 16 lanes (lanes without a source add zero), then the last lane of a row
// is broadcast into the next row (rows 1 and 3), then lane 31 into rows 2 and 3.  This is
// the gfx950 counterpart of the shuffle-up loop of the paper's `scan_warps`.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t lanes_moved(uint32_t v)
{
    return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), CTRL, ROW_MASK, 0xF, ROW_MASK == 0xF));
}
__device__ __forceinline__ uint32_t wave_inclusive_sum(persp::Wave, uint32_t v)
{
    constexpr int kRowShr = 0x110, kRowBcast15 = 0x142, kRowBcast31 = 0x143;
    v += lanes_moved<kRowShr + 1, 0xF>(v);
    v += lanes_moved<kRowShr + 2, 0xF>(v);
    v += lanes_moved<kRowShr + 4, 0xF>(v);
    v += lanes_moved<kRowShr + 8, 0xF>(v);
    v += lanes_moved<kRowBcast15, 0xA>(v);
    v += lanes_moved<kRowBcast31, 0xC>(v);
    return v;
}

// ---- grid level: the chain of tile status words ------------------------------------------
// Called by one whole wave of tile `tile` (> 0) after its aggregate is published.  Returns,
// in every lane, the sum of all elements before the tile.  Lane l looks at tile
// (window_end - l); the nearest predecessor whose full prefix is known ends the walk.
__device__ __forceinline__ uint32_t look_back(persp::Wave, const uint64_t* status, uint32_t tile, int lane, uint32_t spin_limit,
                                              uint32_t* error_word)
{
    uint32_t exclusive = 0;
    int64_t window_end = static_cast<int64_t>(tile) - 1;
    for (;;) {
        const int64_t idx = window_end - lane;
        uint32_t flag = kPrefix, value = 0;  // positions before tile 0 contribute nothing
        if (idx >= 0) {
            uint64_t s = __hip_atomic_load(status + idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            uint32_t polls = 0;
            while (static_cast<uint32_t>(s >> 32) == kInvalid && polls < spin_limit) {
                __builtin_amdgcn_s_sleep(1);
                s = __hip_atomic_load(status + idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                ++polls;
            }
            flag = static_cast<uint32_t>(s >> 32);
            value = static_cast<uint32_t>(s);
            if (flag == kInvalid) {  // gave up: terminate with a wrong result and say so
                __hip_atomic_store(error_word, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                flag = kPrefix;
                value = 0;
            }
        }
        const uint64_t has_prefix = __ballot(flag == kPrefix);
        // lanes up to and including the first one with a full prefix take part in the sum
        const int first = has_prefix ? __builtin_ctzll(has_prefix) : 63;
        uint32_t part = lane <= first ? value : 0u;
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) part += __shfl_xor(part, d, 64);
        exclusive += part;
        if (has_prefix) return exclusive;
        window_end -= 64;
    }
}

// Clears what a scan needs cleared: the header, one status word per tile and the error word
// (the header's own, or a word of the caller's).
__global__ __launch_bounds__(64) void scan_init(uint32_t* header, uint64_t* status, int64_t tiles, uint32_t* error_word)
{
    const int64_t i = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x;
    if (i < tiles) status[i] = pack(kInvalid, 0);
    if (i < static_cast<int64_t>(kHeaderBytes / 4)) header[i] = 0u;
    if (i == 0) *error_word = 0u;
}

template <bool VEC_IN, bool VEC_OUT>
__global__ __launch_bounds__(256) void scan_lookback(const uint32_t* in, uint32_t* out, int64_t n, uint32_t* header,
                                                     uint64_t* status, uint32_t spin_limit, uint32_t* error_word)
{
    const persp::Workgroup wgp = persp::Grid::at_kernel_entry().workgroup();
    const persp::Wave wv = wgp.wave();
    __shared__ uint32_t s_tile, s_exclusive;
    __shared__ uint32_t s_wave_total[kChunks][kWaves];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // Tiles are numbered in the order workgroups start, so every tile this one will wait
    // for has been taken by a workgroup that is already running.
    if (tid == 0) s_tile = __hip_atomic_fetch_add(header, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    sync(wgp);
    const uint32_t tile = s_tile;
    const int64_t base = static_cast<int64_t>(tile) * kTile;
    const bool whole = base + kTile <= n;

    // ---- lane level: chunk j of the tile is 1024 consecutive elements, 4 per lane (one vector)
    uint32_t x[kChunks][kVec];
#pragma unroll
    for (int j = 0; j < kChunks; ++j) {
        const int64_t at = base + (j * kThreads + tid) * kVec;
        if (VEC_IN && whole) {
            // every element is read once and written once: streaming accesses (no retention in
            // the caches asked for) measured 6 % faster at 2^28 elements than plain ones
            const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(in + at));
            x[j][0] = v[0]; x[j][1] = v[1]; x[j][2] = v[2]; x[j][3] = v[3];
        } else {
#pragma unroll
            for (int e = 0; e < kVec; ++e) x[j][e] = at + e < n ? in[at + e] : 0u;
        }
        x[j][1] += x[j][0];
        x[j][2] += x[j][1];
        x[j][3] += x[j][2];
    }

    // ---- wave level: scan the lanes' sums of each chunk
    uint32_t before[kChunks];  // sum of the chunk's elements in lower lanes of this wave
#pragma unroll
    for (int j = 0; j < kChunks; ++j) {
        const uint32_t incl = wave_inclusive_sum(wv, x[j][kVec - 1]);
        before[j] = incl - x[j][kVec - 1];
        if (lane == 63) s_wave_total[j][wave] = incl;
    }
    sync(wgp);

    // ---- workgroup level: chunks in order, waves in order inside a chunk
    uint32_t running = 0;
#pragma unroll
    for (int j = 0; j < kChunks; ++j) {
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const uint32_t t = s_wave_total[j][w];
            if (w == wave) before[j] += running;
            running += t;
        }
    }
    const uint32_t aggregate = running;

    // ---- grid level
    if (wave == 0) {
        uint32_t exclusive = 0;
        if (tile == 0) {
            if (lane == 0)
                __hip_atomic_store(status, pack(kPrefix, aggregate), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else {
            if (lane == 0)
                __hip_atomic_store(status + tile, pack(kAggregate, aggregate), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            exclusive = look_back(wv, status, tile, lane, spin_limit, error_word);
            if (lane == 0)
                __hip_atomic_store(status + tile, pack(kPrefix, exclusive + aggregate), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
        }
        if (lane == 0) s_exclusive = exclusive;
    }
    sync(wgp);
    const uint32_t exclusive = s_exclusive;

#pragma unroll
    for (int j = 0; j < kChunks; ++j) {
        const int64_t at = base + (j * kThreads + tid) * kVec;
        const uint32_t add = exclusive + before[j];
        if (VEC_OUT && whole) {
            __builtin_nontemporal_store(u32x4{x[j][0] + add, x[j][1] + add, x[j][2] + add, x[j][3] + add},
                                        reinterpret_cast<u32x4*>(out + at));
        } else {
#pragma unroll
            for (int e = 0; e < kVec; ++e)
                if (at + e < n) out[at + e] = x[j][e] + add;
        }
    }
}

}  // namespace scan
}  // namespace prism

namespace {

bool aligned_to(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// Test hook: PRISM_SCAN_SPIN_LIMIT=<polls> shortens the bounded wait of the look-back.  Read
// once and kept; prism_reread_environment reads it again.
std::mutex g_spin_mutex;
bool g_spin_loaded = false;
uint32_t g_spin_limit = prism::scan::kDefaultSpinLimit;

void load_spin_limit_locked()
{
    g_spin_limit = prism::scan::kDefaultSpinLimit;
    if (const char* e = std::getenv("PRISM_SCAN_SPIN_LIMIT"); e && *e) {
        const long v = std::atol(e);
        g_spin_limit = v < 0 ? 0u : static_cast<uint32_t>(v);
    }
    g_spin_loaded = true;
}

uint32_t spin_limit()
{
    std::lock_guard<std::mutex> lock(g_spin_mutex);
    if (!g_spin_loaded) load_spin_limit_locked();
    return g_spin_limit;
}

// in / out of a non-empty scan: present, 4-byte aligned, the same array or disjoint ones.
prism_status_t check_data(const uint32_t* in, const uint32_t* out, int64_t n)
{
    if (!in || !out || !aligned_to(in, 4) || !aligned_to(out, 4)) return PRISM_ERR_INVALID_ARG;
    if (in != out) {
        const uintptr_t a = reinterpret_cast<uintptr_t>(in), b = reinterpret_cast<uintptr_t>(out);
        const uintptr_t bytes = static_cast<uintptr_t>(n) * 4;
        if (a < b + bytes && b < a + bytes) return PRISM_ERR_INVALID_ARG;
    }
    return PRISM_OK;
}

bool shares_memory(const void* w, size_t w_bytes, const uint32_t* data, int64_t n)
{
    const uintptr_t a = reinterpret_cast<uintptr_t>(w), b = reinterpret_cast<uintptr_t>(data);
    return a < b + static_cast<uintptr_t>(n) * 4 && b < a + w_bytes;
}

// The two launches of a scan: clear the workspace (a kernel, so that the call can be captured
// into a graph), then the single pass.  `workspace` holds the header and the status words.
prism_status_t enqueue(const uint32_t* in, uint32_t* out, int64_t n, void* workspace, uint32_t* error_word, hipStream_t stream)
{
    using namespace prism::scan;
    const int64_t tiles = (n + kTile - 1) / kTile;
    uint32_t* header = static_cast<uint32_t*>(workspace);
    uint64_t* status = reinterpret_cast<uint64_t*>(static_cast<char*>(workspace) + kHeaderBytes);
    const int64_t init_items = tiles > 16 ? tiles : 16;
    hipLaunchKernelGGL(scan_init, dim3(static_cast<unsigned>((init_items + 63) / 64)), dim3(64), 0, stream, header, status,
                       tiles, error_word);
    if (hipGetLastError() != hipSuccess) return PRISM_ERR_LAUNCH;
    const bool vin = aligned_to(in, 16), vout = aligned_to(out, 16);
    const dim3 grid(static_cast<unsigned>(tiles)), block(kThreads);
    const uint32_t limit = spin_limit();
    if (vin && vout) hipLaunchKernelGGL((scan_lookback<true, true>), grid, block, 0, stream, in, out, n, header, status, limit, error_word);
    else if (vin) hipLaunchKernelGGL((scan_lookback<true, false>), grid, block, 0, stream, in, out, n, header, status, limit, error_word);
    else if (vout) hipLaunchKernelGGL((scan_lookback<false, true>), grid, block, 0, stream, in, out, n, header, status, limit, error_word);
    else hipLaunchKernelGGL((scan_lookback<false, false>), grid, block, 0, stream, in, out, n, header, status, limit, error_word);
    return hipGetLastError() == hipSuccess ? PRISM_OK : PRISM_ERR_LAUNCH;
}

// ---- the scratch of prism_scan_u32_static ---------------------------------------------------
// One array per GPU, part of the loaded code object, for callers that must not allocate.  Its
// name is only a host-side handle: the address a kernel can use is asked for once per device,
// with that device current, and kept; every later use goes through the kept pointer.
constexpr int64_t kStaticMaxN = int64_t{1} << 30;
constexpr size_t kStaticScratchBytes = prism::scan::kHeaderBytes + static_cast<size_t>(kStaticMaxN / prism::scan::kTile) * sizeof(uint64_t);
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
void* g_scratch_of_device[kMaxDevices] = {};
std::mutex g_scratch_mutex;

void* static_scratch_of_current_device()
{
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_of_device[device]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
        g_scratch_of_device[device] = ptr;
    }
    return g_scratch_of_device[device];
}

}  // namespace

namespace prism {
void scan_reread_environment()
{
    std::lock_guard<std::mutex> lock(g_spin_mutex);
    load_spin_limit_locked();
}
}  // namespace prism

extern "C" {

prism_status_t prism_scan_workspace_size(int64_t n, size_t* bytes_out)
{
    using namespace prism::scan;
    if (!bytes_out || n < 0 || n >= kMaxN) return PRISM_ERR_INVALID_ARG;
    const int64_t tiles = (n + kTile - 1) / kTile;
    *bytes_out = n == 0 ? 0 : kHeaderBytes + static_cast<size_t>(tiles) * sizeof(uint64_t);
    return PRISM_OK;
}

prism_status_t prism_scan_u32(const uint32_t* in, uint32_t* out, int64_t n, void* workspace, size_t workspace_bytes,
                              void* hip_stream)
{
    using namespace prism::scan;
    size_t need = 0;
    if (prism_scan_workspace_size(n, &need) != PRISM_OK) return PRISM_ERR_INVALID_ARG;
    if (n == 0) return PRISM_OK;
    const prism_status_t bad = check_data(in, out, n);
    if (bad != PRISM_OK) return bad;
    if (!workspace || workspace_bytes < need) return PRISM_ERR_WORKSPACE;
    if (!aligned_to(workspace, 8)) return PRISM_ERR_INVALID_ARG;
    if (shares_memory(workspace, need, in, n) || shares_memory(workspace, need, out, n)) return PRISM_ERR_INVALID_ARG;
    return enqueue(in, out, n, workspace, static_cast<uint32_t*>(workspace) + 1, static_cast<hipStream_t>(hip_stream));
}

prism_status_t prism_scan_u32_static(const uint32_t* in, uint32_t* out, int64_t n, uint32_t* gave_up, void* hip_stream)
{
    using namespace prism::scan;
    if (n < 0) return PRISM_ERR_INVALID_ARG;
    if (n > kStaticMaxN) return PRISM_ERR_WORKSPACE;  // beyond what the built-in scratch holds
    if (n == 0) return PRISM_OK;
    const prism_status_t bad = check_data(in, out, n);
    if (bad != PRISM_OK) return bad;
    if (gave_up && !aligned_to(gave_up, 4)) return PRISM_ERR_INVALID_ARG;
    if (gave_up && (shares_memory(gave_up, 4, in, n) || shares_memory(gave_up, 4, out, n))) return PRISM_ERR_INVALID_ARG;
    void* ws = static_scratch_of_current_device();
    if (!ws) return PRISM_ERR_LAUNCH;
    return enqueue(in, out, n, ws, gave_up ? gave_up : static_cast<uint32_t*>(ws) + 1, static_cast<hipStream_t>(hip_stream));
}

prism_status_t prism_scan_check(const void* workspace, void* hip_stream)
{
    if (!workspace) return PRISM_ERR_INVALID_ARG;
    uint32_t head[2] = {0u, 0u};
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (hipMemcpyAsync(head, workspace, sizeof(head), hipMemcpyDeviceToHost, stream) != hipSuccess) return PRISM_ERR_LAUNCH;
    if (hipStreamSynchronize(stream) != hipSuccess) return PRISM_ERR_LAUNCH;
    return head[1] == 0u ? PRISM_OK : PRISM_ERR_LAUNCH;
}

}  // extern "C"
