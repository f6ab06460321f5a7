/*
 * CPU oracle for the inclusive prefix sum over 32-bit unsigned integers
 * (test infrastructure only).
 *
 * The paper's second benchmark (section 6.1, "single-pass parallel prefix
 * scan with decoupled look-back") computes, for every position of an array,
 * the sum of all elements up to and including that position; its kernel works
 * on uint32_t, so sums wrap modulo 2^32.  The single-pass algorithm reaches
 * exactly that result (integer addition is associative), so the oracle is the
 * definition written out: one running sum, left to right.  It shares no code
 * with the GPU library and must never be linked into or called from the
 * product path.
 */
#include <stdint.h>
#include <stddef.h>

/* out[i] = (in[0] + ... + in[i]) mod 2^32 for 0 <= i < n.  in == out is allowed. */
int prism_oracle_inclusive_scan_u32(const uint32_t* in, uint32_t* out, int64_t n)
{
    if (n < 0 || (n > 0 && (!in || !out)))
        return -1;
    uint32_t running = 0u;
    for (int64_t i = 0; i < n; ++i) {
        running += in[i];   /* unsigned arithmetic wraps modulo 2^32 */
        out[i] = running;
    }
    return 0;
}
