/*
 * prism_gemm.h -- C ABI of the MI355X (gfx950) dense matrix-multiply library.
 *
 * The library computes, on one GPU,
 *
 *     C  <-  alpha * A * B  +  bias  +  beta * C
 *
 * with 16-bit floating-point operands (bf16 or fp16) or fp32 operands, and
 * fp32 accumulation: the matrix product the paper's evaluation is built on
 * (section 6.1 defines C <- alpha A B + beta C for its fp32 sgemm study;
 * section 6.2 and the hgemm kernel of the code appendix use bf16 operands,
 * fp32 accumulators and a bf16 result).  The per-column bias and the split-K
 * reduction are additions of this library; the paper's kernels have neither.
 *
 * All pointers named "device" are HIP device pointers owned by the caller; the
 * library never allocates or frees memory and keeps no mutable global state
 * apart from its experiment hooks, read once from the environment (see
 * prism_reread_environment).  It is written for one MI355X: 256 compute
 * units in 8 dies.  Calls enqueue work on the given HIP stream and return
 * without synchronising; every buffer must stay valid until the stream has
 * executed the work.  Calls are re-entrant.  Every argument
 * error is detected on the host before anything is launched and reported as
 * a status code; the library never throws or aborts.
 */
#ifndef PRISM_GEMM_H
#define PRISM_GEMM_H

#include <stddef.h>
#include <stdint.h>

#if defined(__GNUC__)
#define PRISM_API __attribute__((visibility("default")))
#else
#define PRISM_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

typedef enum prism_status {
    PRISM_OK = 0,
    PRISM_ERR_INVALID_ARG = 1, /* null pointer, negative size, ld too small, overlap ... */
    PRISM_ERR_UNSUPPORTED = 2, /* dtype / layout value outside the enums below, or
                                  fp32 operands with a 16-bit result                  */
    PRISM_ERR_WORKSPACE = 3,   /* forced split_k > 1 but workspace missing / too small */
    PRISM_ERR_LAUNCH = 4       /* the HIP runtime refused the launch                   */
} prism_status_t;

typedef enum prism_dtype {
    PRISM_DTYPE_BF16 = 0, /* 1-8-7 brain float, 2 bytes          */
    PRISM_DTYPE_F16 = 1,  /* IEEE binary16, 2 bytes              */
    PRISM_DTYPE_F32 = 2   /* IEEE binary32, 4 bytes              */
} prism_dtype_t;

typedef enum prism_layout {
    PRISM_ROW_MAJOR = 0, /* element (r, c) at base[r * ld + c] */
    PRISM_COL_MAJOR = 1  /* element (r, c) at base[r + c * ld] */
} prism_layout_t;

/*
 * Problem descriptor.  A is the logical M x K matrix, B the logical K x N
 * matrix, C the logical M x N matrix.  Plain-old-data; the library reads it
 * during the call only.
 */
typedef struct prism_gemm_desc {
    int32_t ab_dtype;        /* prism_dtype_t of A and B alike; F32 operands need an
                                F32 result (else PRISM_ERR_UNSUPPORTED)                */
    int32_t c_dtype;         /* prism_dtype_t: BF16, F16 or F32                       */
    int32_t layout_a;        /* prism_layout_t                                        */
    int32_t layout_b;        /* prism_layout_t                                        */
    int32_t layout_c;        /* prism_layout_t                                        */
    float alpha;             /* scale of the product; 1.0f for plain C = A*B          */
    float beta;              /* 0.0f: C is write-only and never read                  */
    const float* bias;       /* device, N fp32 values added to every row, or NULL     */
    int32_t split_k;         /* 0 = library decides, 1 = never split, n > 1 = n slices */
    int32_t reserved;        /* must be 0                                             */
    void* workspace;         /* device scratch for split-K partial sums, or NULL      */
    size_t workspace_bytes;  /* size of that scratch                                  */
} prism_gemm_desc_t;

/*
 * What the library will launch for a problem: filled by prism_gemm_plan, pure
 * host arithmetic (usable without a GPU).
 */
typedef struct prism_gemm_plan {
    int32_t kernel;          /* 0 = nothing to launch, 1 = staged (any layout/alignment),
                                2 = direct-to-LDS pipeline (aligned operands),
                                3 = the same pipeline, persistent: used for more tiles
                                    than compute units with short K loops              */
    int32_t tile_m, tile_n, tile_k; /* workgroup tile                                */
    int32_t waves;           /* wavefronts per workgroup                              */
    int32_t split_k;         /* K slices actually used (>= 1)                         */
    int32_t swapped;         /* 1 if the problem is run as C^T = B^T A^T              */
    int32_t reserved;
    int64_t tiles_m, tiles_n;
    int64_t workgroups;      /* grid size of the main kernel (kernel 3: at most 256)  */
    size_t workspace_bytes;  /* scratch the chosen split needs (0 when split_k == 1)  */
} prism_gemm_plan_t;

/*
 * C <- alpha*A*B + bias + beta*C for one problem (paper section 6.1 / 6.2).
 *
 * d            host pointer to the descriptor.
 * M, N, K      logical sizes, each >= 0.
 * A, B         device; lda / ldb / ldc are leading dimensions in elements:
 *              row-major needs ld >= number of columns, column-major needs
 *              ld >= number of rows (ld >= 1 always).
 * C            device; written (and read when beta != 0).  C must not overlap
 *              A or B.
 * hip_stream   a hipStream_t passed as void*; NULL is the default stream.
 *
 * M == 0 or N == 0: nothing is written, PRISM_OK.  K == 0: C <- bias + beta*C.
 * Any positive sizes, leading dimensions and alignments are accepted.
 * Operands in either layout run on the fast pipeline when their rows (or
 * columns) start on 16-byte boundaries, K is a multiple of 128 bytes of
 * elements (64 of a 16-bit type, 32 of fp32) and, for an operand that is not
 * contiguous along K (column-major A, row-major B), M respectively N is a
 * multiple of 16 bytes of elements; everything else runs on a staged kernel
 * with the same arithmetic.  For a fixed problem, descriptor and GPU the result is
 * bit-for-bit reproducible: split-K partial sums are reduced in slice order.
 */
PRISM_API prism_status_t prism_gemm(const prism_gemm_desc_t* d, int64_t M, int64_t N, int64_t K,
                          const void* A, int64_t lda, const void* B, int64_t ldb,
                          void* C, int64_t ldc, void* hip_stream);

/*
 * `batch` independent problems of the same shape; problem b uses
 * A + b*strideA, B + b*strideB, C + b*strideC (strides in elements).  strideA
 * or strideB may be 0 to share an operand; |strideC| must be large enough that
 * the C matrices do not overlap.  The bias, alpha and beta are shared.
 * batch == 0 is a no-op.  Everything else as prism_gemm.
 */
PRISM_API prism_status_t prism_gemm_batched(const prism_gemm_desc_t* d, int64_t M, int64_t N, int64_t K,
                                  const void* A, int64_t lda, int64_t strideA,
                                  const void* B, int64_t ldb, int64_t strideB,
                                  void* C, int64_t ldc, int64_t strideC,
                                  int64_t batch, void* hip_stream);

/*
 * Bytes of device workspace the descriptor's split_k setting needs for this
 * shape: forced n > 1 gives n*batch*M*N*4, split_k == 1 gives 0, and
 * split_k == 0 gives what the library's own choice would use (it falls back to
 * no split when the caller passes a smaller workspace).  Host arithmetic only.
 */
PRISM_API prism_status_t prism_gemm_workspace_size(const prism_gemm_desc_t* d, int64_t M, int64_t N,
                                         int64_t K, int64_t batch, size_t* bytes_out);

/*
 * The launch plan for a problem, with the same validation and choices as
 * prism_gemm_batched (pointer alignment is taken from the pointers given; pass
 * the real device pointers or NULL to assume 16-byte alignment).  Host only.
 */
PRISM_API prism_status_t prism_gemm_plan(const prism_gemm_desc_t* d, int64_t M, int64_t N, int64_t K,
                               const void* A, int64_t lda, int64_t strideA,
                               const void* B, int64_t ldb, int64_t strideB,
                               const void* C, int64_t ldc, int64_t strideC,
                               int64_t batch, prism_gemm_plan_t* plan_out);

/*
 * The tile scheduler's map, evaluated on the host: workgroup `wg` of a grid of
 * `tiles_m * tiles_n * units` workgroups (units = batch * split_k) works on
 * output tile (*tile_m, *tile_n) of unit *unit.  The map is a bijection; it
 * deals consecutive workgroup ids round-robin over the 8 accelerator dies and
 * gives each die a compact block of neighbouring tiles (the role the super-tile
 * order plays in the paper's persistent hgemm scheduler).  Returns
 * PRISM_ERR_INVALID_ARG for an id outside the grid.
 */
PRISM_API prism_status_t prism_sched_map(int64_t wg, int64_t tiles_m, int64_t tiles_n, int64_t units,
                               int64_t* tile_m, int64_t* tile_n, int64_t* unit);

/*
 * Measurement aid: the ceiling of the matrix instructions alone.  Launches 256 workgroups of
 * four wavefronts that run the register-blocked wave tile of the GEMM kernels (8 x 8 blocks of
 * 16 x 16, the MFMA of paper section 6.2's "collective matrix-core instructions") `iterations`
 * times over operand fragments held in registers: no LDS and no memory traffic inside the
 * loop.  One iteration is the matrix work of one K step of the 256 x 256 x 64 tile, so
 * `iterations` = K / 64 mimics a GEMM's launch; a launch does
 * PRISM_MFMA_PROBE_FLOP_PER_ITERATION * iterations floating-point operations (half of that
 * for fp32 operands, whose K step is 32 elements).
 *
 * ab_dtype     BF16, F16 or F32: which matrix instruction.
 * operands     device, 16-byte aligned, PRISM_MFMA_PROBE_OPERAND_BYTES bytes of operand values
 *              (their distribution matters: the clock a GPU sustains depends on the data).
 * counters     device, 8-byte aligned, PRISM_MFMA_PROBE_COUNTER_BYTES bytes; wave w of workgroup
 *              g writes four uint64 at index 4 * (4 * g + w): shader-clock cycles of its loop,
 *              ticks of the constant 100 MHz counter over the same span, a checksum, iterations.
 * Too small a buffer is PRISM_ERR_WORKSPACE.  Enqueues on hip_stream; time it with events.
 */
#define PRISM_MFMA_PROBE_OPERAND_BYTES ((size_t)33554432)
#define PRISM_MFMA_PROBE_COUNTER_BYTES ((size_t)32768)
#define PRISM_MFMA_PROBE_FLOP_PER_ITERATION 2147483648.0 /* 256 x 4 waves x 128 MFMAs x 2 x 16 x 16 x 32 */
PRISM_API prism_status_t prism_mfma_probe(int32_t ab_dtype, const void* operands, size_t operand_bytes,
                                          int32_t iterations, uint64_t* counters, size_t counter_bytes,
                                          void* hip_stream);

/*
 * Measurement aid: prism_gemm_batched with time stamps.  The same launch (same kernel, same
 * result), in which the first thread of every workgroup of the main kernel records, at four
 * points, the shader-clock counter and the constant 100 MHz counter:
 *   stamps[8*g + 2*p], stamps[8*g + 2*p + 1]   cycles, 100 MHz ticks of workgroup g at point p
 *   p = 0 kernel entry, 1 first operand fragments in registers (start of the K loop),
 *       2 K loop done, 3 results stored and acknowledged.
 * Differences of cycles over differences of ticks give the clock the GPU sustained in a
 * phase; workgroup g runs on die g % 8.  Only problems that prism_gemm_plan sends to the
 * direct-to-LDS pipeline (plan.kernel == 2) can be stamped, others are PRISM_ERR_UNSUPPORTED.
 * stamps: device, 8-byte aligned, plan.workgroups * PRISM_STAMP_BYTES_PER_WORKGROUP bytes or
 * more (else PRISM_ERR_WORKSPACE).  Everything else as prism_gemm_batched.
 */
#define PRISM_STAMP_BYTES_PER_WORKGROUP ((size_t)64)
PRISM_API prism_status_t prism_gemm_batched_stamped(const prism_gemm_desc_t* d, int64_t M, int64_t N, int64_t K,
                                          const void* A, int64_t lda, int64_t strideA,
                                          const void* B, int64_t ldb, int64_t strideB,
                                          void* C, int64_t ldc, int64_t strideC, int64_t batch,
                                          uint64_t* stamps, size_t stamp_bytes, void* hip_stream);

/*
 * Test aid: shows, on the device, the two lane layouts the kernels are built on, through the
 * very device functions the kernels use (one wavefront, a few microseconds).
 *
 * PRISM_LAYOUT_ACCUMULATOR_BF16 / _F16: in0 = R, in1 = C, each a row-major 16 x 32 matrix of
 *   the 16-bit type; out = row-major 16 x 16 fp32 matrix that must equal R * C^T: one matrix
 *   instruction, its accumulator registers placed by the library's lane -> (row, column) map.
 * PRISM_LAYOUT_K_ROWS_READ: in0 = row-major 32 x 128 matrix of 16-bit values (k-rows of an
 *   operand that is not contiguous along K), in1 unused; out = row-major 128 x 32 matrix that must
 *   be its transpose: the transposing LDS reads of the pipeline, placed by the documented layout.
 * Pointers are device pointers, 16-byte aligned.  Other values of `what`: PRISM_ERR_UNSUPPORTED.
 */
#define PRISM_LAYOUT_ACCUMULATOR_BF16 0
#define PRISM_LAYOUT_ACCUMULATOR_F16 1
#define PRISM_LAYOUT_K_ROWS_READ 2
PRISM_API prism_status_t prism_layout_probe(int32_t what, const void* in0, const void* in1, void* out, void* hip_stream);

/* Static string for a status code ("PRISM_OK", ...); never NULL. */
PRISM_API const char* prism_status_string(prism_status_t s);

/* Library version, major*10000 + minor*100 + patch. */
PRISM_API int prism_version(void);

/*
 * The library reads its test and experiment hooks from the environment once, at the first call
 * that needs them, and keeps them: PRISM_GEMM_CONFIG=0|1 (pin 256x256 / 128x128 tiles of the
 * pipeline), PRISM_PERSISTENT=0|1 (never / whenever possible use the persistent kernel),
 * PRISM_LOG=1 (one line per launch on stderr: problem, kernel, tile, split),
 * PRISM_SCAN_SPIN_LIMIT=<polls> (bound of the scan's look-back wait).  This call reads them
 * again, for a process that changes its environment after the first call (tests do).
 */
PRISM_API void prism_reread_environment(void);

#ifdef __cplusplus
}
#endif
#endif /* PRISM_GEMM_H */
