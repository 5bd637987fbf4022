/*
 * srq.h - C ABI of the sparse-residual-compensated quantized GEMM for MI355X (gfx950).
 *
 * The library computes  D = alpha * (A.B, quantized and compensated) + beta * C  following
 * Algorithm 1 of Gu et al., "A method for accelerating low precision operations by sparse
 * matrix multiplication":  vector-wise symmetric quantization of A (one scale per row) and
 * B (one scale per column) (Sec. 3.2), an INT8 x INT8 -> INT32 product, dequantization by
 * the outer product of the scales (Eq. "quantized GEMM"), and a correction built from the
 * quantized residual matrices (Sec. 2.3, Eq. gemm_r) in which the operands are first
 * reduced to sparse matrices by the threshold rule of Eq. avgQuan (Sec. 3.1.1).
 *
 * Conventions (all entry points)
 *   - Every data pointer is a DEVICE pointer owned by the caller unless a comment says
 *     "host".  Matrices are row-major with an explicit leading dimension counted in
 *     elements.  The library never allocates or frees device memory; scratch space comes
 *     from the workspace the caller attaches to the handle.
 *   - `stream` is the caller's hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work and return without waiting, except where a comment says the
 *     call synchronises.
 *   - Every call returns an srq_status_t.  Arguments are validated before anything is
 *     launched; a non-zero status means nothing was enqueued (except SRQ_STATUS_CAPACITY,
 *     see srq_compensated_gemm).
 *   - qmax = 2^(bits-1) - 1 (Sec. 2.3, lambda = (2^(N-1)-1)/a_max); bits in 2..8, codes are
 *     always stored in int8 containers.  K * qmax^2 must stay below 2^31 so the INT32
 *     accumulators cannot overflow.
 *   - "Vector" means a quantization vector: a row for SRQ_AXIS_ROW, a column for
 *     SRQ_AXIS_COL.  Code matrices are stored either vector-major (code of element e of
 *     vector v at Q[v*ld + e]) or element-major (Q[e*ld + v]).  For SRQ_AXIS_ROW
 *     vector-major is the layout of X itself; for SRQ_AXIS_COL element-major is.
 *   - Inputs must be finite; a vector whose maximum magnitude is zero gets scale 0,
 *     lambda 0 and all-zero codes.
 */
#ifndef SRQ_H_
#define SRQ_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum srq_status_t {
  SRQ_STATUS_OK = 0,
  SRQ_STATUS_INVALID_ARG = 1,   /* null pointer, negative size, ld too small, bad enum     */
  SRQ_STATUS_UNSUPPORTED = 2,   /* bits outside 2..8; reduced operand of 2^31 or more elements */
  SRQ_STATUS_K_OVERFLOW = 3,    /* K * qmax^2 >= 2^31                                       */
  SRQ_STATUS_CAPACITY = 4,      /* compressed-storage capacity too small for the selection  */
  SRQ_STATUS_WORKSPACE = 5,     /* no workspace attached, or too small                      */
  SRQ_STATUS_HIP_ERROR = 6,     /* a HIP runtime call failed (see srq_last_hip_error)       */
  SRQ_STATUS_NO_DEVICE = 7      /* arguments are valid but the handle has no device         */
} srq_status_t;

typedef enum srq_axis_t { SRQ_AXIS_ROW = 0, SRQ_AXIS_COL = 1 } srq_axis_t;
typedef enum srq_layout_t { SRQ_LAYOUT_VECTOR_MAJOR = 0, SRQ_LAYOUT_ELEMENT_MAJOR = 1 } srq_layout_t;

/* Rounding of lambda*x to an integer (Eq. Quantization's TypeCast).  The paper's worked
 * examples truncate; nearest-even is the default used for every measured workload. */
typedef enum srq_round_t { SRQ_ROUND_NEAREST_EVEN = 0, SRQ_ROUND_TRUNC = 1 } srq_round_t;

/* How the sparse products of Algorithm 1's SPMM line are executed.  Every strategy returns
 * the same INT32 values. */
typedef enum srq_strategy_t {
  SRQ_STRATEGY_AUTO = 0,        /* pick per term from the measured density, on the device   */
  SRQ_STRATEGY_CSR_VALU = 1,    /* row-wise CSR x dense on the vector ALUs                   */
  SRQ_STRATEGY_CSR_MFMA = 2,    /* CSR expanded to zero-filled INT8 tiles, matrix cores      */
  SRQ_STRATEGY_CSR_SMFMAC = 3,  /* the reduced operand in 2:4 form (two operands: the first two */
                                /* and the third and fourth kept code of every four k), on    */
                                /* the sparse matrix-core instruction; needs M, N multiples   */
                                /* of 256 and K <= 32768, otherwise runs as CSR_MFMA          */
  SRQ_STRATEGY_COLBLOCK = 4     /* column-block split: the indices k kept in at least 90 % of */
                                /* an operand's vectors (up to 128 of them: whole outlier     */
                                /* columns) form a dense strip that runs on the matrix cores; */
                                /* the remaining entries run as CSR on the vector ALUs.  The  */
                                /* two parts are added to C one after the other, so C is      */
                                /* within rounding of the other paths; the INT32 sums are the */
                                /* same                                                        */
} srq_strategy_t;

/* Granularity of the first-level scales in srq_compensated_gemm.  VECTOR is the method of
 * Sec. 3.2 (one scale per row of A and per column of B); GLOBAL is the matrix-wide scale of
 * Sec. 2.3 / Eq. getlambda (a_max over the whole matrix), the setting of the paper's worked
 * 3x3 example.  Residual codes keep one scale per vector in both modes. */
typedef enum srq_scale_t { SRQ_SCALE_VECTOR = 0, SRQ_SCALE_GLOBAL = 1 } srq_scale_t;

typedef struct srq_context* srq_handle_t;

/* Statistics written to device memory by srq_compensated_gemm. */
typedef struct srq_stats_t {
  int64_t nnz_a;        /* entries kept in A' (Algorithm 1, getSparsity)                    */
  int64_t nnz_b;        /* entries kept in B'                                               */
  int32_t path_a;       /* 0 = term skipped (theta = inf), 1 = CSR_VALU, 2 = CSR_MFMA,      */
  int32_t path_b;       /* 3 = dense branch on the unreduced operand, 4 = CSR_SMFMAC,       */
                        /* 5 = COLBLOCK                                                     */
  int32_t overflow;     /* bit 0: A' kept more entries than the workspace's compressed      */
                        /* arrays hold, bit 1: the same for B'.  Non-zero means that NO      */
                        /* correction term was added: C holds the uncorrected first product  */
                        /* (alpha / beta not applied), as with SRQ_STATUS_CAPACITY           */
  int32_t reserved;     /* written as 0                                                     */
} srq_stats_t;

/* Optional extra outputs of srq_compensated_gemm for stage-by-stage checks; any member may
 * be NULL.  Each is a caller-owned device buffer of M*N elements, row-major, ld = N. */
typedef struct srq_debug_t {
  int32_t* D_int;       /* A_int . B_int                                                    */
  float*   D_F;         /* its dequantization, before any correction                        */
  int32_t* DR1_int;     /* A'_int . RB_int   (or A_int . RB_int on the dense branch)        */
  int32_t* DR2_int;     /* RA_int . B'_int   (or RA_int . B_int on the dense branch)        */
} srq_debug_t;

/* Device pointers INTO THE WORKSPACE to the intermediates of the last
 * srq_compensated_gemm call on this handle (valid until the next call or until the
 * workspace is replaced).  Code matrices: A-side M x K vector-major, B-side N x K
 * vector-major, both with leading dimension ld_codes = K rounded up to a multiple of 128
 * (the columns past K hold zeros, so that every row starts on a 128-byte boundary whatever K
 * is).  Element-major residual codes: RB_em is K x N (ld = N), RA_em is K x M (ld = M); they
 * are only filled when a term ran as CSR_VALU. */
typedef struct srq_intermediates_t {
  const int8_t *A_int, *B_int, *RA_int, *RB_int, *RA_em, *RB_em;
  const float *s_a, *lam_a, *s_ra, *s_b, *lam_b, *s_rb;   /* [M] resp. [N]                 */
  const float *drow, *dcol, *t_a, *t_b;                   /* [M] resp. [N]                 */
  const int32_t *a_ptr, *a_idx; const int8_t* a_val;      /* CSR of A'_int                  */
  const int32_t *b_ptr, *b_idx; const int8_t* b_val;      /* CSC of B'_int; idx and val are */
                                                          /* NULL for a dense-branch term   */
  int64_t capacity_a, capacity_b;                         /* entries that fit idx/val       */
  int64_t ld_codes;                                       /* see above                      */
} srq_intermediates_t;

/* ---- lifecycle -------------------------------------------------------------------- */

/* Creates a handle bound to HIP device `device` (host call).  device = -1 creates a handle
 * without a device: every entry point still validates its arguments and then returns
 * SRQ_STATUS_NO_DEVICE instead of launching (used to test validation on a CPU-only host). */
srq_status_t srq_create(srq_handle_t* handle, int device);
srq_status_t srq_destroy(srq_handle_t handle);

/* Bytes of workspace srq_compensated_gemm needs for an M x N x K problem when at most
 * `max_density` (0..1] of each operand's entries are kept.  Host call, no device needed. */
srq_status_t srq_workspace_bytes(int64_t M, int64_t N, int64_t K, double max_density, size_t* bytes);

/* Attaches caller-owned device memory (256-byte aligned) as the handle's workspace.  The
 * staged entry points below need at least srq_stage_workspace_bytes(M, N, K) bytes of it
 * for operands of an M x N x K problem (a workspace sized by srq_workspace_bytes for the
 * same problem is always enough). */
srq_status_t srq_set_workspace(srq_handle_t handle, void* workspace, size_t bytes);
srq_status_t srq_stage_workspace_bytes(int64_t M, int64_t N, int64_t K, size_t* bytes);

/* Selects the scale granularity (see srq_scale_t) that later srq_compensated_gemm calls on
 * this handle use; a new handle starts with SRQ_SCALE_VECTOR.  With SRQ_SCALE_GLOBAL the
 * exported s_a / lam_a / s_b / lam_b vectors hold the one matrix-wide value in every entry.
 * Host call; returns SRQ_STATUS_INVALID_ARG for an unknown mode. */
srq_status_t srq_set_scale_mode(srq_handle_t handle, srq_scale_t mode);

/* SRQ_STRATEGY_AUTO decides per term on the device, after the selection, whether the sparse
 * product runs on the vector ALUs (1) or on the matrix cores (2).  Some intermediates are laid
 * out for one or the other before that decision exists; the library writes them for the execution
 * named here (0 = no expectation: the matrix cores) and, if the decision then differs, once more
 * in the other layout.  The hint never changes a result, only the time of a call.  The handle
 * also learns by itself: the deciding kernel stores its choice into pinned host memory of the
 * handle (a plain store from the device, no synchronisation), and the next call on the handle
 * takes whatever it finds there as its expectation, so a sequence of calls on similar operands
 * needs no hint after the first.  A call recorded into a HIP graph keeps storing there on every
 * replay: the handle must outlive the graph.  Host call. */
srq_status_t srq_set_auto_hint(srq_handle_t handle, int path_a, int path_b);

/* Stage timing of srq_compensated_gemm (the per-stage time shares of Sec. 4.1.2).  When
 * enabled, the call records a pair of HIP events on `stream` around each stage;
 * srq_profile_read waits for them and writes to ms[SRQ_NUM_STAGES] (host array) the
 * milliseconds per stage, summed over the calls made since the previous read (or since
 * enabling): read after every call for the times of that call, or after a run of calls issued
 * back to back for their totals without a wait in between.  The events of the last 64 calls
 * are kept; earlier ones are forgotten.  0 for a stage that did not run.
 * `enable`: 0 = off, SRQ_PROFILE_ALL = every stage, SRQ_PROFILE_PRODUCTS = only the three
 * products (SRQ_STAGE_GEMM, SRQ_STAGE_TERM1, SRQ_STAGE_TERM2; the other entries read 0): an event
 * record costs the call about 3 microseconds, since the kernel after it cannot start under the
 * tail of the kernel before it. */
enum { SRQ_PROFILE_ALL = 1, SRQ_PROFILE_PRODUCTS = 2 };
enum {
  SRQ_STAGE_QUANTIZE = 0,   /* amax, scales, codes of A and B, max |residual|             */
  SRQ_STAGE_GEMM = 1,       /* INT8 product, dequantization, partial sums of |D_F|        */
  SRQ_STAGE_SELECT = 2,     /* means, thresholds, count / scan / scatter to CSR and CSC   */
  SRQ_STAGE_RESIDUAL = 3,   /* residual codes in the layouts the chosen paths read        */
  SRQ_STAGE_TERM1_PREP = 4, /* expansion of CSR(A') for the matrix-core path              */
  SRQ_STAGE_TERM1 = 5,      /* DR1 product + accumulate                                   */
  SRQ_STAGE_TERM2_PREP = 6,
  SRQ_STAGE_TERM2 = 7,
  SRQ_NUM_STAGES = 8
};
srq_status_t srq_profile_enable(srq_handle_t handle, int enable);
srq_status_t srq_profile_read(srq_handle_t handle, float* ms);

/* Last hipError_t seen by this handle as an int (0 = hipSuccess).  Host call. */
int srq_last_hip_error(srq_handle_t handle);
const char* srq_status_string(srq_status_t status);

/* ---- quantize: Algorithm 1 line 1 (Eq. Quantization, Eq. getlambda, Sec. 3.2) -------- */

/* For every vector v of X[rows x cols] (ldx >= cols):  amax = max|x|, lambda_v =
 * fl(qmax/amax), scale_v = fl(amax/qmax), code = clamp(round(fl(x*lambda_v)), -qmax, qmax).
 *   Q      out, int8, rows*cols codes in `layout` (ldq >= vector length for vector-major,
 *          >= number of vectors for element-major)
 *   scale  out, float[number of vectors]   (the dequantization factor 1/lambda)
 *   lambda out, float[number of vectors], may be NULL
 * rows or cols equal to 0 is a valid no-op. */
srq_status_t srq_quantize(srq_handle_t handle, const float* X, int64_t rows, int64_t cols, int64_t ldx,
                          srq_axis_t axis, int bits, srq_round_t round, srq_layout_t layout,
                          int8_t* Q, int64_t ldq, float* scale, float* lambda, void* stream);

/* ---- build_sparse_residual: Algorithm 1 lines 4-10 for one operand -------------------- */

/* Given X, its vector scales/lambdas (from srq_quantize) and a threshold per vector
 * (thresh_v = theta * mean|D_F| over the vector's row resp. column of D_F, Eq. avgQuan):
 *   1. residual r = fl(x - fl(float(code)*scale_v)) with code recomputed from X and lambda
 *      (Sec. 2.3), quantized again per vector -> Rq (layout `r_layout`, ld `ldr`), rscale;
 *   2. the reduced operand: entry kept iff |x| > thresh_v (strict); kept codes compacted
 *      vector by vector, ascending element index: ptr[int32, nvec+1], idx[int32], val[int8]
 *      (CSR of A' for SRQ_AXIS_ROW, CSC of B' for SRQ_AXIS_COL).  Kept entries whose code
 *      is 0 are stored.
 * `capacity` = entries idx/val can hold.  nnz_dev (device int64) receives the number of
 * kept entries; if it exceeds `capacity` only ptr is complete and idx/val hold the first
 * `capacity` entries - the caller checks after synchronising.  Rq/rscale may both be NULL
 * to skip step 1; ptr/idx/val may all be NULL to skip step 2. */
srq_status_t srq_build_sparse_residual(srq_handle_t handle, const float* X, int64_t rows, int64_t cols,
                                       int64_t ldx, srq_axis_t axis, const float* scale,
                                       const float* lambda, const float* thresh, int bits,
                                       srq_round_t round, int8_t* Rq, int64_t ldr, srq_layout_t r_layout,
                                       float* rscale, int32_t* ptr, int32_t* idx, int8_t* val,
                                       int64_t capacity, int64_t* nnz_dev, void* stream);

/* ---- staged products (Algorithm 1 lines 2-3, 7, 12, 16-17), used by parity tests and by
 *      callers that keep operands quantized ------------------------------------------------ */

/* D_int[i,j] = sum_k Qa[i*lda+k] * Qb[j*ldb+k]  (both operands vector-major, K contiguous);
 * D_F[i,j] = fl(fl(float(D_int)) * fl(sa[i]*sb[j])).  D_int (ld = ldd) may be NULL.
 * drow[M], dcol[N] receive the means of |D_F| over each row / column (Sec. 3.1.1), summed
 * in double in a fixed order; both may be NULL.
 * Any shape and alignment is accepted; the fast kernels need 16-byte aligned Qa, Qb, lda and ldb
 * multiples of 16 and K a multiple of 64 (pad K with zero codes to get there: they add nothing),
 * the persistent one in addition at least 256 whole tiles of 256 x 256 and K a multiple of 128 (it
 * then takes the block of whole tiles and the plain kernel the strips beside it), and the
 * pipelined small-tile one (problems below that) M, N and K multiples of 128. */
srq_status_t srq_gemm_i8(srq_handle_t handle, int64_t M, int64_t N, int64_t K, const int8_t* Qa, int64_t lda,
                         const float* sa, const int8_t* Qb, int64_t ldb, const float* sb, float* D_F,
                         int32_t* D_int, int64_t ldd, float* drow, float* dcol, void* stream);

/* srq_gemm_i8 for callers that cannot hand the library any memory of their own and may not
 * allocate: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, same results bit for bit; the handle's workspace is neither needed nor touched.
 * The partial sums of |D_F| (the only scratch memory the call needs, and only when drow / dcol are
 * given) go to a fixed array inside the library's code object, srq_static_scratch_bytes() bytes
 * (8 MiB) per GPU, held from the moment the library is loaded on that GPU until the process ends.
 * Limit: 8 * (ceil(N/128) * M + ceil(M/128) * N), each term rounded up to 256, must not exceed that
 * size (e.g. M = N = 8192, or 4096 x 14336); a larger problem is refused with
 * SRQ_STATUS_WORKSPACE before anything is launched.  The call allocates and frees nothing and
 * records no memset.  All calls on one GPU share that GPU's array: calls that overlap in time on
 * the same GPU (two streams, two threads) race and must be serialised by the caller; calls one
 * after the other need no clearing in between (every slot read was written by the same call).
 * Returns SRQ_STATUS_HIP_ERROR if the array's address could not be obtained when the handle was
 * created. */
srq_status_t srq_gemm_i8_static_scratch(srq_handle_t handle, int64_t M, int64_t N, int64_t K, const int8_t* Qa,
                                        int64_t lda, const float* sa, const int8_t* Qb, int64_t ldb,
                                        const float* sb, float* D_F, int32_t* D_int, int64_t ldd, float* drow,
                                        float* dcol, void* stream);
size_t srq_static_scratch_bytes(void);

/* C[i,j] += fl(fl(float(DR[i,j])) * fl(s_row[i]*s_col[j])) with DR the product of a
 * compressed operand and dense residual codes:
 *   side = SRQ_AXIS_ROW: DR = A'.RB, (ptr,idx,val) = CSR of A' (M vectors over K), Rq = RB codes;
 *   side = SRQ_AXIS_COL: DR = RA.B', (ptr,idx,val) = CSC of B' (N vectors over K), Rq = RA codes.
 * Rq layout: CSR_VALU wants the residual codes k-major (RB element-major K x N, ld >= N;
 * RA element-major K x M, ld >= M); CSR_MFMA wants them K-contiguous (RB vector-major
 * N x K; RA vector-major M x K; ld >= K).  SRQ_STRATEGY_AUTO, SRQ_STRATEGY_CSR_SMFMAC and SRQ_STRATEGY_COLBLOCK
 * (which needs both layouts) are not accepted here.
 * s_row[M] / s_col[N] are the scales paired with rows / columns of C for this term.
 * DR_int (ld = ldc) may be NULL. */
srq_status_t srq_spmm_accumulate(srq_handle_t handle, srq_axis_t side, srq_strategy_t strategy, int64_t M,
                                 int64_t N, int64_t K, const int32_t* ptr, const int32_t* idx,
                                 const int8_t* val, const int8_t* Rq, int64_t ldr, const float* s_row,
                                 const float* s_col, float* C, int32_t* DR_int, int64_t ldc, void* stream);

/* ---- compensated_gemm: the whole of Algorithm 1 ---------------------------------------- */

/* C[M x N] = alpha * ( D_F + dequant(DR1_int) + dequant(DR2_int) ) + beta * Cin.
 *   A [M x K] (lda >= K), B [K x N] (ldb >= N), C (ldc >= N): float, row-major.
 *   theta_a, theta_b   threshold factor of Eq. avgQuan for A resp. B (the paper has one
 *                      theta: pass it twice).  +inf keeps nothing: plain vector-wise
 *                      quantized GEMM.  0 keeps every non-zero entry: dense compensation.
 *   dense_fallback_density   Algorithm 1's limit "s": a term whose reduced operand has
 *                      density >= s runs as a dense product on the UNREDUCED codes.  Values
 *                      > 1 switch the branch off; values <= 0 send every term to the dense
 *                      branch.  A value in (0, 1] makes the call synchronise once on `stream`
 *                      to read the densities (the only synchronising mode).
 *   Cin                read only if beta != 0 (ldcin >= N); must not overlap C.
 *   stats_dev          device srq_stats_t, may be NULL.
 *   dbg                host pointer to a struct of device buffers, may be NULL.
 * An operand that is reduced (finite theta) must have fewer than 2^31 elements (INT32 row
 * pointers): SRQ_STATUS_UNSUPPORTED otherwise.
 * With dbg != NULL a CSR_SMFMAC term runs as CSR_MFMA (the 2:4 kernel has no raw-sum output).
 * With dense_fallback_density > 1 or <= 0 the call only enqueues kernels on `stream`, whatever the
 * strategy (SRQ_STRATEGY_AUTO takes its decision on the device): no allocation, no host
 * read-back, no memset node, so it may be recorded into a HIP graph by a capturing caller (the
 * workspace must be attached before).  srq_get_intermediates then reports only what exists
 * whatever the decision turns out to be (residual codes in the hinted layout).
 * Returns SRQ_STATUS_CAPACITY (after the first product and the selection ran: C then holds the
 * uncorrected D_F, no correction term was added) when a synchronising mode finds more kept
 * entries than the workspace was sized for.  A non-synchronising mode cannot know on the host:
 * it returns SRQ_STATUS_OK, every correction kernel checks the counts on the device and does
 * nothing when an operand overflowed, so that C again holds the uncorrected D_F (never a
 * correction from truncated arrays), and stats_dev->overflow is set: pass stats_dev and check
 * it after synchronising.  The compressed arrays themselves hold the first `capacity` entries. */
srq_status_t srq_compensated_gemm(srq_handle_t handle, int64_t M, int64_t N, int64_t K, const float* A,
                                  int64_t lda, const float* B, int64_t ldb, float theta_a, float theta_b,
                                  int bits, srq_round_t round, float dense_fallback_density,
                                  srq_strategy_t strategy, float alpha, float beta, const float* Cin,
                                  int64_t ldcin, float* C, int64_t ldc, srq_stats_t* stats_dev,
                                  const srq_debug_t* dbg, void* stream);

/* Fills `out` (host struct) with workspace pointers to the last call's intermediates. */
srq_status_t srq_get_intermediates(srq_handle_t handle, srq_intermediates_t* out);

#ifdef __cplusplus
}
#endif
#endif /* SRQ_H_ */
