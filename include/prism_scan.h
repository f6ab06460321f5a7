/*
 * prism_scan.h -- C ABI of the single-pass prefix scan on one MI355X (gfx950).
 *
 * The paper's second benchmark (section 6.1): the inclusive prefix sum of an
 * array of 32-bit unsigned integers,
 *
 *     out[i] = (in[0] + in[1] + ... + in[i]) mod 2^32,
 *
 * computed in ONE pass over the data with the decoupled look-back scheme the
 * paper implements (every tile publishes its aggregate, then looks back over
 * the tiles before it until it meets one whose full prefix is known).  The
 * data is read once and written once: 8 bytes of HBM traffic per element.
 *
 * Ownership, streams and errors as in prism_gemm.h: device pointers belong to
 * the caller, the library allocates nothing, calls enqueue work on the given
 * HIP stream and return without synchronising, argument errors are found on
 * the host before anything is launched.
 */
#ifndef PRISM_SCAN_H
#define PRISM_SCAN_H

#include "prism_gemm.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Bytes of device workspace a scan of n elements needs (tile counter, error
 * word and one 8-byte status word per tile of 16384 elements).  n < 0 is
 * PRISM_ERR_INVALID_ARG.  Host arithmetic only.
 */
PRISM_API prism_status_t prism_scan_workspace_size(int64_t n, size_t* bytes_out);

/*
 * Inclusive prefix sum of n uint32 values.
 *
 * in, out      device, 4-byte aligned; out may be the same pointer as in (the
 *              scan then works in place, as the paper's kernel does); any other
 *              overlap is PRISM_ERR_INVALID_ARG.  16-byte aligned pointers take
 *              the vector path, others a slower element-wise one.
 * n            number of elements, 0 <= n < 2^43; n == 0 launches nothing.
 * workspace    device, 8-byte aligned, at least prism_scan_workspace_size(n)
 *              bytes (else PRISM_ERR_WORKSPACE); it is initialised by the call
 *              itself and may be reused by the next call on the same stream.
 *              Calls that overlap in time need separate workspaces.
 * hip_stream   a hipStream_t passed as void*; NULL is the default stream.
 *
 * A tile waits for the tiles before it with a bounded number of polls; if the
 * bound is ever hit (it is not in a working system: tiles take their numbers
 * from an atomic counter, so every tile waited for is already running) the
 * kernel still terminates, the result is wrong, and prism_scan_check reports it.
 */
PRISM_API prism_status_t prism_scan_u32(const uint32_t* in, uint32_t* out, int64_t n,
                                        void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The same scan for callers that can neither allocate nor bring a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  The status words live
 * in an array that is part of the library's code object (512 KiB + 64 bytes, held by every GPU
 * the library runs on until the process ends); the call allocates and frees nothing.
 *
 * in, out, n, hip_stream   as prism_scan_u32, with n <= 2^30; a larger n is refused with
 *              PRISM_ERR_WORKSPACE (use prism_scan_u32 with a workspace of your own).
 * gave_up      device, 4-byte aligned, or NULL: a word that the call clears and that a look-back
 *              which gave up waiting sets to 1 (what prism_scan_check reads from a workspace);
 *              the caller reads it after the stream has executed the work.
 *
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 * streams, two threads) race and give wrong results; calls on one stream, or otherwise
 * ordered, are fine, and each call clears what it needs with a kernel of its own (no memset
 * node, so the call can be captured).  The first call on a GPU looks the array's device
 * address up (hipGetSymbolAddress, once per GPU): make that call outside graph capture.
 */
PRISM_API prism_status_t prism_scan_u32_static(const uint32_t* in, uint32_t* out, int64_t n,
                                               uint32_t* gave_up, void* hip_stream);

/*
 * Synchronises the stream and reads the workspace's error word back:
 * PRISM_OK, or PRISM_ERR_LAUNCH when a look-back of the last scan that used
 * this workspace gave up waiting.
 */
PRISM_API prism_status_t prism_scan_check(const void* workspace, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* PRISM_SCAN_H */
