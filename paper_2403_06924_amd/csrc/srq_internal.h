// Internal declarations shared by the translation units of libsrq (not part of the ABI).
#ifndef SRQ_INTERNAL_H_
#define SRQ_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "srq.h"

struct srq_context {
  int device;            // -1: no device (validation only)
  void* ws;              // caller-owned device workspace
  size_t ws_bytes;
  int last_hip_error;
  int64_t* host_nnz;     // pinned host buffer for the two counters read back in synchronising modes
  srq_intermediates_t last;
  int prof_enabled;
  unsigned prof_mask;                       // bit i: stage i is timed
  // stage events of the last kProfRing calls (slot = call number mod kProfRing)
  unsigned prof_used[64];                   // bit i: stage i ran in that call
  hipEvent_t prof_ev[64][2 * SRQ_NUM_STAGES];   // start/stop per stage, created on enable
  int prof_slot;                            // slot of the call being recorded
  int64_t prof_calls;                       // calls recorded since the last read
  int prof_created;
  int scale_mode;        // srq_scale_t of the next srq_compensated_gemm calls
  int last_path_a;       // execution the caller expects SRQ_STRATEGY_AUTO to pick for term 1 (srq_set_auto_hint;
  int last_path_b;       // 0: none given, the matrix cores are assumed), resp. for term 2
};

namespace srq {

inline int qmax_of_bits(int bits) { return (1 << (bits - 1)) - 1; }

// A launch that only matters for some outcomes of a decision taken on the device (which execution
// SRQ_STRATEGY_AUTO picks for a term): the kernel reads *value and does nothing unless bit *value
// of ok_mask is set.  value == null: unconditional.
struct RunIf {
  const int32_t* value;
  uint32_t ok_mask;
};
static __device__ __forceinline__ bool run_if_ok(const RunIf& r) { return !r.value || ((r.ok_mask >> *r.value) & 1u); }
constexpr RunIf kAlways = {nullptr, 0u};

constexpr int kSelChunk = 256;      // elements of a vector handled by one wave in count/scatter

// epilogue modes of the INT8 GEMM
enum GemmMode { kGemmFirst = 0, kGemmAccum = 1 };

struct GemmEpilogue {
  int mode;               // GemmMode
  const float* s_row;     // [M] scale paired with rows of the output
  const float* s_col;     // [N] scale paired with columns
  float* C;               // output / accumulator, row-major
  int64_t ldc;
  int32_t* D_int;         // optional raw INT32 product (ld = ldd), may be null
  int64_t ldd;
  float* D_F_copy;        // optional copy of the dequantized product before alpha/beta (ld = ldd)
  double* row_part;       // kGemmFirst: [tiles_n][M] partial sums of |D_F| (may be null)
  double* col_part;       // kGemmFirst: [tiles_m][N]
  int final_scale;        // apply alpha/beta after this term
  float alpha, beta;
  const float* Cin;
  int64_t ldcin;
  // Overflow guard of the non-synchronising modes: when set, a kernel that adds a correction
  // term (or applies alpha / beta after one) does nothing if the selection kept more entries
  // than the compressed arrays hold (guard_nnz[0] > guard_cap_a or guard_nnz[1] > guard_cap_b),
  // so that C stays the uncorrected first product instead of receiving a truncated correction.
  const int64_t* guard_nnz;   // device int64[2]: kept entries of A' and B' (null: no guard)
  int64_t guard_cap_a, guard_cap_b;
  // a product that only matters when a device-side count is non-zero (the dense strip of the
  // column-block execution): when set and *run_if_nonzero == 0 the kernel does nothing
  const int32_t* run_if_nonzero;
  int dint_add;               // vector-ALU kernels: add the raw sums to D_int instead of storing them
  // executions chosen on the device (SRQ_STRATEGY_AUTO): paths[0] / paths[1] hold the execution of
  // term 1 / term 2; the kernel runs only if both are among those it was launched for
  const int32_t* paths;       // device int32[2] (null: unconditional)
  uint32_t ok_a, ok_b;        // bit p set: path p of term 1 resp. term 2 is acceptable
  // strides of the partial sums (row_part[part * part_ld_m + row], col_part[part * part_ld_n + col]);
  // 0: the M resp. N of the launch.  Set when a launch covers a block of a larger product.
  int64_t part_ld_m, part_ld_n;
  // paired launches only: the two products are decided one by one (product t runs iff the path of
  // term t+1 is acceptable) instead of both or none; alpha / beta go with the second product only
  int each_product;
};

// true when the epilogue's overflow guard is set and tripped (wave-uniform: scalar loads)
static __device__ __forceinline__ bool guard_tripped(const GemmEpilogue& ep) {
  if (ep.run_if_nonzero && *ep.run_if_nonzero == 0) return true;
  if (ep.paths) {
    const bool run_a = (ep.ok_a >> ep.paths[0]) & 1u, run_b = (ep.ok_b >> ep.paths[1]) & 1u;
    if (ep.each_product ? !(run_a || run_b) : !(run_a && run_b)) return true;
  }
  return ep.guard_nnz && (ep.guard_nnz[0] > ep.guard_cap_a || ep.guard_nnz[1] > ep.guard_cap_b);
}

// first and last product (0 or 1) a paired launch runs (guard_tripped has dealt with "none")
static __device__ __forceinline__ void pair_range(const GemmEpilogue& ep, int nprod, int& lo, int& hi) {
  lo = 0;
  hi = nprod - 1;
  if (nprod == 2 && ep.paths && ep.each_product) {
    if (!((ep.ok_a >> ep.paths[0]) & 1u)) lo = 1;
    if (!((ep.ok_b >> ep.paths[1]) & 1u)) hi = 0;
  }
}

// Second product of a paired accumulate-mode launch of the persistent kernel: C += dequant(Qa.Qb^T)
// with its own scales, right after the first product of the same output tile (Qa == null: none).
// alpha / beta of the epilogue, if any, are applied after the second product.
struct GemmSecond {
  const int8_t* Qa;
  const int8_t* Qb;
  int64_t lda, ldb;
  const float* s_row;
  const float* s_col;
};

// ---- launchers (each returns the hipError_t of its launches) --------------------------
hipError_t launch_fill_u32(uint32_t* p, int64_t n, uint32_t v, hipStream_t st);

// amax of |x| per vector as float bits in amax_bits[nvec] (must be zero-filled for AXIS_COL)
hipError_t launch_amax(const float* X, int64_t rows, int64_t cols, int64_t ldx, int axis,
                       uint32_t* amax_bits, hipStream_t st);
// in place: amax bits -> scale = amax/qmax; lambda = qmax/amax (lambda may be null)
// every entry of the vector of non-negative float bit patterns becomes their maximum
hipError_t launch_broadcast_max(uint32_t* bits, int64_t n, hipStream_t st);
hipError_t launch_scales(uint32_t* amax_bits_then_scale, float* lambda, int64_t nvec, int qmax,
                         hipStream_t st);
// codes of X in `layout`; if ramax_bits != null also accumulates max|residual| per vector
hipError_t launch_quantize_tiles(const float* X, int64_t rows, int64_t cols, int64_t ldx, int axis,
                                 const float* scale, const float* lambda, int qmax, int trunc,
                                 int layout, int8_t* Q, int64_t ldq, uint32_t* ramax_bits,
                                 hipStream_t st);
// residual codes in up to two layouts (either output may be null)
hipError_t launch_residual_tiles(const float* X, int64_t rows, int64_t cols, int64_t ldx, int axis,
                                 const float* scale, const float* lambda, const float* rlambda,
                                 int qmax, int trunc, int8_t* R_vm, int64_t ld_vm, int8_t* R_em,
                                 int64_t ld_em, hipStream_t st, RunIf run = kAlways);

// selection: counts per (chunk, vector) -> offsets -> compacted arrays
hipError_t launch_select_count(const float* X, int64_t rows, int64_t cols, int64_t ldx, int axis,
                               const float* thresh, int32_t* cnt, hipStream_t st);
hipError_t launch_select_scan(int32_t* cnt_then_off, int64_t nvec, int64_t nchunks, int32_t* totals,
                              int32_t* ptr, int64_t* nnz_dev, hipStream_t st);
hipError_t launch_select_scatter(const float* X, int64_t rows, int64_t cols, int64_t ldx, int axis,
                                 const float* thresh, const float* lambda, int qmax, int trunc,
                                 const int32_t* ptr, const int32_t* off, int32_t* idx, int8_t* val,
                                 int64_t capacity, hipStream_t st);
inline int64_t select_chunks(int64_t veclen) { return (veclen + kSelChunk - 1) / kSelChunk; }
// exclusive scan of per-vector totals into ptr[nvec+1]; *nnz_dev = grand total
hipError_t launch_scan_totals(const int32_t* totals, int64_t nvec, int32_t* ptr, int64_t* nnz_dev,
                              hipStream_t st);

// ---- streaming fast paths (fused.hip); the *_ok predicates say whether shapes/alignment allow them
inline int64_t mask_words(int64_t veclen) { return (veclen + 63) / 64; }
bool rows_fused_ok(const float* X, int64_t cols, int64_t ldx, const int8_t* Q, int64_t ldq, const int8_t* Rq,
                   int64_t ldr);
// (rscale == null: no residual at all; Rq == null with rscale given: residual scales only;
//  given_scale / given_lambda: use these per-row values instead of deriving them from the row's
//  maximum, and leave scale / lambda unwritten; rlambda may be null)
// up to three arrays of 32-bit words that launch_rows_fused zeroes on the side
struct ClearList {
  uint32_t* a; int64_t na;
  uint32_t* b; int64_t nb;
  uint32_t* c; int64_t nc;
};
bool rows_fused_can_clear(int64_t rows, const ClearList& c);   // one word per thread and array
hipError_t launch_rows_fused(const float* X, int64_t rows, int64_t cols, int64_t ldx, int qmax, int trunc,
                             int8_t* Q, int64_t ldq, float* scale, float* lambda, int8_t* Rq, int64_t ldr,
                             float* rscale, float* rlambda, hipStream_t st, const float* given_scale = nullptr,
                             const float* given_lambda = nullptr,
                             const ClearList* clear = nullptr);
bool rows_resid_em_ok(const float* X, int64_t rows, int64_t cols, int64_t ldx, const float* scale,
                      const float* lambda, const float* rlambda, const int8_t* Rem, int64_t ldem);
hipError_t launch_rows_resid_em(const float* X, int64_t rows, int64_t cols, int64_t ldx, int qmax, int trunc,
                                const float* scale, const float* lambda, const float* rlambda, int8_t* Rem,
                                int64_t ldem, hipStream_t st, RunIf run = kAlways);
// that pass doubling as the selection pass of the operand (mask and counts as launch_rows_mask)
bool rows_mask_resid_em_ok(const float* X, int64_t rows, int64_t cols, int64_t ldx, const float* scale,
                           const float* lambda, const float* rlambda, const int8_t* Rem, int64_t ldem,
                           const float* thresh);
hipError_t launch_rows_mask_resid_em(const float* X, int64_t rows, int64_t cols, int64_t ldx, int qmax, int trunc,
                                     const float* scale, const float* lambda, const float* rlambda, int8_t* Rem,
                                     int64_t ldem, const float* thresh, uint64_t* mask, int32_t* counts,
                                     hipStream_t st);
bool cols_pass_ok(const float* X, int64_t cols, int64_t ldx);
hipError_t launch_cols_amax(const float* X, int64_t rows, int64_t cols, int64_t ldx, uint32_t* amax_bits,
                            hipStream_t st);
hipError_t launch_cols_codes(const float* X, int64_t rows, int64_t cols, int64_t ldx, int qmax, int trunc,
                             const float* scale, const float* lambda, int8_t* Qvm, int64_t ldvm, int8_t* Qem,
                             int64_t ldem, uint32_t* ramax_bits, hipStream_t st);
hipError_t launch_cols_codes_from_amax(const float* X, int64_t rows, int64_t cols, int64_t ldx, int qmax,
                                       int trunc, const uint32_t* amax_bits, float* scale, float* lambda,
                                       int8_t* Qvm, int64_t ldvm, uint32_t* ramax_bits, hipStream_t st);
hipError_t launch_cols_resid_from_amax(const float* X, int64_t rows, int64_t cols, int64_t ldx, int qmax,
                                       int trunc, const float* scale, const float* lambda,
                                       const uint32_t* ramax_bits, float* rscale, float* rlambda, int8_t* Rvm,
                                       int64_t ldvm, int8_t* Rem, int64_t ldem, hipStream_t st);
// zeroes columns [cols, ld) of up to six row-major byte matrices of `rows[i]` rows each (null: skipped)
hipError_t launch_zero_pad(int8_t* const* mats, const int64_t* rows, int n, int64_t cols, int64_t ld,
                           hipStream_t st);
// zero-fills up to three arrays of 32-bit words in one launch (null pointers are skipped)
hipError_t launch_fill3_u32(uint32_t* a, int64_t na, uint32_t* b, int64_t nb, uint32_t* c, int64_t nc,
                            hipStream_t st);
hipError_t launch_cols_resid(const float* X, int64_t rows, int64_t cols, int64_t ldx, int qmax, int trunc,
                             const float* scale, const float* lambda, const float* rlambda, int8_t* Rvm,
                             int64_t ldvm, int8_t* Rem, int64_t ldem, hipStream_t st, RunIf run = kAlways);
hipError_t launch_cols_mask(const float* X, int64_t rows, int64_t cols, int64_t ldx, const float* thresh,
                            uint64_t* mask, int32_t* counts, hipStream_t st);
hipError_t launch_cols_mask_resid(const float* X, int64_t rows, int64_t cols, int64_t ldx, int qmax, int trunc,
                                  const float* scale, const float* lambda, const uint32_t* ramax_bits,
                                  float* rscale, float* rlambda, int8_t* Rvm, int64_t ldvm, int8_t* Rem,
                                  int64_t ldem, const float* thresh, uint64_t* mask, int32_t* counts,
                                  hipStream_t st);
hipError_t launch_rows_mask(const float* X, int64_t rows, int64_t cols, int64_t ldx, const float* thresh,
                            uint64_t* mask, int32_t* counts, hipStream_t st);
// compaction from mask + codes; dense != null also writes the vector zero-filled to dense[v*ldd + e];
// nnz_hint: the number of kept entries if the host knows it (picks the variant for very sparse
// operands), else -1; dense_if: the expansion is written only if the device-side decision allows
hipError_t launch_scatter_mask(const uint64_t* mask, int64_t nvec, int64_t veclen, const int8_t* Q, int64_t ldq,
                               const int32_t* ptr, int32_t* idx, int8_t* val, int64_t capacity, int8_t* dense,
                               int64_t ldd, int64_t nnz_hint, hipStream_t st, RunIf dense_if = kAlways);
// two exclusive scans in one launch; a null totals pointer skips that half
// decide != null (paths set): one block scans both vectors, then writes SRQ_STRATEGY_AUTO's choice per
// term (as launch_decide_paths would from the totals z0 / z1: a term whose totals pointer is null
// does not exist) and, if stats != null, the call's statistics
struct ScanDecision {
  int32_t* paths;             // device int32[2]
  int32_t* seen;              // host-visible int32[2] or null
  int64_t min_mfma_a, min_mfma_b;
  srq_stats_t* stats;         // device, or null
  int64_t cap_a, cap_b;       // capacities the totals are compared with for stats->overflow
};
hipError_t launch_scan_pair(const int32_t* t0, int64_t n0, int32_t* p0, int64_t* z0, const int32_t* t1,
                            int64_t n1, int32_t* p1, int64_t* z1, hipStream_t st,
                            const ScanDecision* decide = nullptr);

// thresholds from the partial sums of the GEMM epilogue
hipError_t launch_reduce_means_pair(const double* part0, int64_t nparts0, int64_t n0, int64_t count0, float theta0,
                                    float* mean0, float* thresh0, const double* part1, int64_t nparts1,
                                    int64_t n1, int64_t count1, float theta1, float* mean1, float* thresh1,
                                    hipStream_t st);

// INT8 GEMM, both operands K-contiguous
int gemm_tile_m();                          // smallest tile extents (upper bound on tile counts)
int gemm_tile_n();
// number of partial sums launch_gemm_i8 leaves per row (parts_n) and per column (parts_m) of D_F
// for this problem: what the reduction after it has to add up
void gemm_sum_parts(int64_t M, int64_t N, int64_t K, const int8_t* Qa, int64_t lda, const int8_t* Qb, int64_t ldb,
                    const GemmEpilogue& ep, int64_t* parts_n, int64_t* parts_m);
int64_t gemm_tiles_m(int64_t M, int64_t N);  // tile counts of the configuration launch_gemm_i8 picks
int64_t gemm_tiles_n(int64_t M, int64_t N);
hipError_t launch_gemm_i8(int64_t M, int64_t N, int64_t K, const int8_t* Qa, int64_t lda,
                          const int8_t* Qb, int64_t ldb, const GemmEpilogue& ep, hipStream_t st);
// persistent-workgroup variant for full, aligned, large problems (chosen inside launch_gemm_i8)
hipError_t gemm_device_cus(int* cus);
// raises a kernel's dynamic-LDS limit to `bytes` once per (device, kernel); safe to call from
// several host threads
hipError_t ensure_dynamic_lds(const void* kernel, int bytes);
bool gemm_persistent_ok(int64_t M, int64_t N, int64_t K, const int8_t* Qa, int64_t lda, const int8_t* Qb,
                        int64_t ldb, const GemmEpilogue& ep);
// (second: accumulate mode only; both products must pass gemm_persistent_ok)
hipError_t launch_gemm_i8_persistent(int64_t M, int64_t N, int64_t K, const int8_t* Qa, int64_t lda,
                                     const int8_t* Qb, int64_t ldb, const GemmEpilogue& ep, hipStream_t st,
                                     const GemmSecond* second = nullptr);
// the kernel for aligned problems with fewer than 256 tiles of 256 x 256 (gemm_small.hip); same contract
bool gemm_small_ok(int64_t M, int64_t N, int64_t K, const int8_t* Qa, int64_t lda, const int8_t* Qb, int64_t ldb,
                   const GemmEpilogue& ep);
hipError_t launch_gemm_i8_small(int64_t M, int64_t N, int64_t K, const int8_t* Qa, int64_t lda, const int8_t* Qb,
                                int64_t ldb, const GemmEpilogue& ep, hipStream_t st,
                                const GemmSecond* second = nullptr);
// Both correction products in one accumulate-mode launch (first Qa.Qb^T with ep's scales, then sec):
// possible when both products fit the same one of the two kernels above.
bool gemm_pair_ok(int64_t M, int64_t N, int64_t K, const int8_t* Qa, int64_t lda, const int8_t* Qb, int64_t ldb,
                  const GemmSecond& sec, const GemmEpilogue& ep);
hipError_t launch_gemm_i8_pair(int64_t M, int64_t N, int64_t K, const int8_t* Qa, int64_t lda, const int8_t* Qb,
                               int64_t ldb, const GemmSecond& sec, const GemmEpilogue& ep, hipStream_t st);

// CSR (vector-major) -> zero-filled dense vector-major codes
hipError_t launch_densify(const int32_t* ptr, const int32_t* idx, const int8_t* val, int64_t nvec,
                          int64_t veclen, int64_t capacity, int8_t* dense, int64_t ld, hipStream_t st,
                          RunIf run = kAlways);

// VALU SpMM.  out[v, e] = sum_p val[p] * R[idx[p]*ldr + e];  side 0: C[v, e], side 1: C[e, v].
// Vector v owns the pairs [ptr[v], ptr_end[v]); ptr_end == null means plain CSR (ptr + 1).
hipError_t launch_spmm_valu(int side, int64_t nvec, int64_t nelem, int64_t K, const int32_t* ptr,
                            const int32_t* ptr_end, const int32_t* idx, const int8_t* val, int64_t capacity,
                            const int8_t* R, int64_t ldr, const GemmEpilogue& ep, hipStream_t st,
                            const uint32_t* kflag = nullptr);   // kflag: bitmap over k of entries to skip

// ---- column-block execution (colblock.hip): the k kept in at least min_keep_ratio of the vectors
// (at most kStripK of them) become a dense strip.  count: int32[mask_words(K) * 64] scratch;
// klist: int32[kStripK]; kflag: uint32[mask_words(K) * 2]; nstrip: int32[1]
constexpr int kStripK = 128;
hipError_t launch_colblock_pick(const uint64_t* mask, int64_t nvec, int64_t K, double min_keep_ratio,
                                int32_t* count, int32_t* klist, uint32_t* kflag, int32_t* nstrip,
                                hipStream_t st);
// strip[v][c] = Q[v][klist[c]] (only where the keep-bit is set, if a mask is given), zero-padded
// to kStripK columns
hipError_t launch_strip_gather(const int8_t* Q, int64_t ldq, const uint64_t* mask, int64_t K, int64_t nvec,
                               const int32_t* klist, int8_t* strip, hipStream_t st);

// ---- 2:4-structured execution (sparse24.hip, gemm_sparse24.hip)
// A reduced operand in 2:4 form: P1 (first two codes of a group of four k) and P2 (third and
// fourth), each as code bytes + position nibbles in the K-tile-major layout of sparse24.hip, and
// one flag word per (block of 256 vectors, K-tile) telling where P2 holds anything; plus the
// dense operand it is multiplied with, and (second product of a paired launch only) the scales
// paired with the rows and columns of C.
struct Sparse24Operand {
  const int8_t *vals1, *vals2;
  const uint8_t *nib1, *nib2;
  const uint32_t* flags;
  const int8_t* Qb;           // dense operand, K-contiguous
  int64_t ldb;
  const float *s_row, *s_col;
};
constexpr int kSparse24MaxKTiles = 256;      // K / 128 may not exceed this (one flag row = one wave-wide load)
// flag words per block of 256 vectors (a multiple of 4: rows start 16-byte aligned), and of a whole
// operand including the padding that lets the product kernel read 256 words from any row start
__host__ __device__ inline int64_t sparse24_flag_stride(int64_t kc) { return ((kc >> 7) + 3) & ~(int64_t)3; }
inline int64_t sparse24_flag_words(int64_t nvec, int64_t kc) {
  return ((nvec + 255) / 256) * sparse24_flag_stride(kc) + kSparse24MaxKTiles;
}
// compaction pass that also writes the 2:4 form (flags must be zero on entry)
bool scatter24_ok(int64_t nvec, int64_t kc, const int8_t* Q, int64_t ldq);
hipError_t launch_scatter24(const uint64_t* mask, int64_t nvec, int64_t veclen, int64_t kc, const int8_t* Q,
                            int64_t ldq, const int32_t* ptr, int32_t* idx, int8_t* val, int64_t capacity,
                            int8_t* vals1, uint8_t* nib1, int8_t* vals2, uint8_t* nib2, uint32_t* flags,
                            hipStream_t st);
// C (M x N) += dequant(product).  One product (second == null): `op` with its sparse vectors along
// the rows of C (trans false) or along its columns (trans true; scales from the epilogue either
// way).  Two products: op = term 1 (rows), *second = term 2 (columns, with its own scales).
bool gemm_sparse24_ok(int64_t M, int64_t N, int64_t K, const Sparse24Operand& op, bool trans, const GemmEpilogue& ep);
hipError_t launch_gemm_i8_sparse24(int64_t M, int64_t N, int64_t K, const Sparse24Operand& op, bool trans,
                                   const Sparse24Operand* second, const GemmEpilogue& ep, hipStream_t st);

// (paths_dev != null: the executions are read from the device, path_a / path_b ignored)
hipError_t launch_stats(const int64_t* nnz_a, const int64_t* nnz_b, int path_a, int path_b, int64_t cap_a,
                        int64_t cap_b, srq_stats_t* out, hipStream_t st, const int32_t* paths_dev = nullptr);
// SRQ_STRATEGY_AUTO's choice on the device: paths[t] = 0 if term t does not exist, else the matrix
// cores (2) if the operand keeps at least min_mfma[t] entries, else the vector ALUs (1)
hipError_t launch_decide_paths(const int64_t* nnz, int term_a, int term_b, int64_t min_mfma_a, int64_t min_mfma_b,
                               int32_t* paths, int32_t* seen, hipStream_t st);
hipError_t launch_scale_only(int64_t M, int64_t N, const GemmEpilogue& ep, hipStream_t st);

}  // namespace srq
#endif
