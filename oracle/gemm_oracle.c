/*
 * CPU oracle for C <- alpha*A*B + bias + beta*C  (test infrastructure only).
 *
 * This file is the plain definition of the matrix product the paper's
 * evaluation computes (section 6.1: C <- alpha A B + beta C; section 6.2 and
 * the hgemm kernel in the code appendix: 16-bit inputs, wider accumulation),
 * written out as a triple loop in IEEE double precision.  It is deliberately
 * slow and has no tiling, no vector intrinsics and no reordering of the k
 * sum.  It shares no code with the GPU library and must never be linked into
 * or called from the product path: only the tests, the smoke check and the
 * benchmark's CPU-baseline leg use it.
 *
 * Besides the result it returns, for every entry, the magnitude sum
 *     mag = |alpha| * sum_k |a_ik * b_kj| + |bias_j| + |beta * c_ij|
 * that the acceptance bound of the GPU tests is scaled by.
 *
 * Products of two bf16 (8-bit significand) or two fp16 (11-bit significand)
 * values are exact in double; the only rounding is the double accumulation.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* bf16: 1 sign, 8 exponent (bias 127), 7 fraction bits. */
double prism_oracle_decode_bf16(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 7) & 0xFF;
    int f = h & 0x7F;
    double v;
    if (e == 0)
        v = ldexp((double)f, -126 - 7);            /* zero / subnormal */
    else if (e == 0xFF)
        v = f ? NAN : INFINITY;
    else
        v = ldexp((double)(128 + f), e - 127 - 7); /* 1.f * 2^(e-127) */
    return sign ? -v : v;
}

/* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits. */
double prism_oracle_decode_f16(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1F;
    int f = h & 0x3FF;
    double v;
    if (e == 0)
        v = ldexp((double)f, -14 - 10);
    else if (e == 0x1F)
        v = f ? NAN : INFINITY;
    else
        v = ldexp((double)(1024 + f), e - 15 - 10);
    return sign ? -v : v;
}

int prism_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * ab_dtype: 0 = bf16, 1 = fp16 (bit patterns in uint16).
 * Element (i,k) of A is A[i*a_si + k*a_sk]; element (k,j) of B is
 * B[k*b_sk + j*b_sj]  (strides in elements, so any layout is expressible).
 * bias: N floats or NULL.  c_in: M x N row-major doubles (ld = N) or NULL;
 * it is only read when beta != 0.
 * rows: list of n_rows row indices to evaluate, or NULL for all M rows
 * (then n_rows must equal M).  ref and mag receive n_rows x N row-major
 * doubles; c_in is indexed by the true row index.
 * Returns 0, or -1 on a bad argument.
 */
int prism_oracle_gemm(int ab_dtype, int64_t M, int64_t N, int64_t K,
                      const uint16_t* A, int64_t a_si, int64_t a_sk,
                      const uint16_t* B, int64_t b_sk, int64_t b_sj,
                      double alpha, double beta,
                      const float* bias, const double* c_in,
                      const int64_t* rows, int64_t n_rows,
                      double* ref, double* mag)
{
    static double dec[2][65536];
    if (M < 0 || N < 0 || K < 0 || n_rows < 0 || (ab_dtype != 0 && ab_dtype != 1))
        return -1;
    if (!rows && n_rows != M)
        return -1;
    if (beta != 0.0 && !c_in)
        return -1;

    /* value of every 16-bit pattern, from the decoders above */
    double* d = dec[ab_dtype];
    for (int h = 0; h < 65536; ++h)
        d[h] = ab_dtype == 0 ? prism_oracle_decode_bf16((uint16_t)h)
                             : prism_oracle_decode_f16((uint16_t)h);

#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t r = 0; r < n_rows; ++r) {
        for (int64_t j = 0; j < N; ++j) {
            int64_t i = rows ? rows[r] : r;
            double s = 0.0, m = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                double p = d[A[i * a_si + k * a_sk]] * d[B[k * b_sk + j * b_sj]];
                s += p;
                m += fabs(p);
            }
            double out = alpha * s;
            double om = fabs(alpha) * m;
            if (bias) {
                out += (double)bias[j];
                om += fabs((double)bias[j]);
            }
            if (beta != 0.0) {
                double t = beta * c_in[i * N + j];
                out += t;
                om += fabs(t);
            }
            ref[r * N + j] = out;
            mag[r * N + j] = om;
        }
    }
    return 0;
}

/*
 * The same definition for fp32 operands (the paper's sgemm, section 6.1:
 * C <- alpha A B + beta C on float matrices).  A float converts to double
 * exactly and the product of two floats (24-bit significands) is exact in
 * double, so again the only rounding is the double accumulation.
 * Arguments as prism_oracle_gemm, with A and B as floats.
 */
int prism_oracle_sgemm(int64_t M, int64_t N, int64_t K,
                       const float* A, int64_t a_si, int64_t a_sk,
                       const float* B, int64_t b_sk, int64_t b_sj,
                       double alpha, double beta,
                       const float* bias, const double* c_in,
                       const int64_t* rows, int64_t n_rows,
                       double* ref, double* mag)
{
    if (M < 0 || N < 0 || K < 0 || n_rows < 0)
        return -1;
    if (!rows && n_rows != M)
        return -1;
    if (beta != 0.0 && !c_in)
        return -1;

#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t r = 0; r < n_rows; ++r) {
        for (int64_t j = 0; j < N; ++j) {
            int64_t i = rows ? rows[r] : r;
            double s = 0.0, m = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                double p = (double)A[i * a_si + k * a_sk] * (double)B[k * b_sk + j * b_sj];
                s += p;
                m += fabs(p);
            }
            double out = alpha * s;
            double om = fabs(alpha) * m;
            if (bias) {
                out += (double)bias[j];
                om += fabs((double)bias[j]);
            }
            if (beta != 0.0) {
                double t = beta * c_in[i * N + j];
                out += t;
                om += fabs(t);
            }
            ref[r * N + j] = out;
            mag[r * N + j] = om;
        }
    }
    return 0;
}
