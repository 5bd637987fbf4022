// Host side of the C ABI: argument validation, workspace planning and the kernel pipeline of
// Algorithm 1.  No device memory is allocated here; everything lives in the caller's
// workspace.
#include <math.h>
#include <mutex>
#include <new>
#include <string.h>

#include "srq_internal.h"

using namespace srq;

// Scratch memory of the one entry point that may not use a caller's workspace
// (srq_gemm_i8_static_scratch): a fixed array in the code object, one copy per GPU the library is
// loaded on, holding the partial sums of |D_F| between the product and the kernel that turns them
// into means.  Every call on a GPU shares that GPU's copy; every slot a call reads it has written
// before, so nothing has to be cleared between calls.
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

// The array's name is only a host-side handle; its device address differs per GPU and is looked up
// once per device (srq_create, with that device current) with hipGetSymbolAddress.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
char* g_scratch_ptr[kMaxDevices] = {nullptr};
hipError_t g_scratch_error = hipSuccess;

hipError_t prime_static_scratch(int device) {      // the device is current
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (g_scratch_ptr[device]) return hipSuccess;
  void* ptr = nullptr;
  hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
  if (e != hipSuccess) { g_scratch_error = e; return e; }
  g_scratch_ptr[device] = static_cast<char*>(ptr);
  return hipSuccess;
}

char* static_scratch_of(int device) {
  if (device < 0 || device >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  return g_scratch_ptr[device];
}

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// Densities at and above which SRQ_STRATEGY_AUTO runs a sparse product on the matrix cores
// (the paper's switch between SPMM and GEMM, Algorithm 1 lines 11-15, with the ratio of the
// two kernels' throughputs on MI355X in place of the paper's eta).  Measured at 8192^3: the
// vector-ALU kernel takes 0.19 ms + 0.37 ms per percent of density for A' (rows of C written
// straight), 0.15 ms + 0.54 ms per percent for B' (columns of C, through LDS); the expanded
// operand on the matrix cores takes 0.48 ms at any density when both terms share a launch, 0.51
// alone.  Whole calls with both terms on one or the other kernel break even at 0.65 % (8192^3),
// 0.6 % (4096^3), 0.95 % (6144^3, whose 576 tiles load the 256 compute units unevenly) and
// 0.62 % (16384^3).
// execution of a correction term as reported in srq_stats_t (0: term skipped)
constexpr int kPathValu = 1, kPathMfma = 2, kPathDense = 3, kPath24 = 4, kPathColblock = 5;
constexpr int kPathOnDevice = 6;          // host-side marker: vector ALUs or matrix cores, decided on the device
inline int strategy_path(srq_strategy_t s) {
  return s == SRQ_STRATEGY_CSR_VALU ? kPathValu : s == SRQ_STRATEGY_CSR_SMFMAC ? kPath24
       : s == SRQ_STRATEGY_COLBLOCK ? kPathColblock : kPathMfma;
}
// which layouts of the OTHER operand's residual codes an execution reads: k-major for the vector
// ALUs (also the remainder of the column-block split),
// K-contiguous for the matrix cores
inline bool path_reads_em(int path) { return path == kPathValu || path == kPathColblock; }
inline bool path_reads_vm(int path) { return path >= kPathMfma; }

// share of an operand's vectors that must keep an index k for k to join the dense strip
constexpr double kColblockKeepRatio = 0.9;

constexpr int64_t kNoCap = INT64_MAX;     // capacity of an operand that is not compacted

constexpr double kAutoMfmaDensityA = 0.008;
constexpr double kAutoMfmaDensityALongK = 0.0062;
constexpr double kAutoMfmaDensityB = 0.007;
constexpr double kAutoMfmaDensityBLongK = 0.0062;

struct Carver {
  char* base;
  size_t off;
  template <class T>
  T* take(size_t n) {
    T* p = reinterpret_cast<T*>(base + off);
    off += align_up(n * sizeof(T));
    return p;
  }
};

struct Plan {
  int8_t *A_int, *B_int, *RA_int, *RB_int, *RA_em, *RB_em, *Ad, *Bd;
  float *s_a, *lam_a, *s_ra, *lam_ra, *drow, *t_a;
  float *s_b, *lam_b, *s_rb, *lam_rb, *dcol, *t_b;
  uint32_t *amax_b, *ramax_b;   // column maxima of B and of its residual as bit patterns
  double *row_part, *col_part;
  int32_t *cnt_a, *tot_a, *a_ptr, *cnt_b, *tot_b, *b_ptr;
  int64_t* nnz;   // [2]
  int32_t* paths; // [2] executions SRQ_STRATEGY_AUTO decided on the device
  uint64_t *mask_a, *mask_b;   // keep-bits, one row of words per vector
  int32_t *a_idx, *b_idx;
  int8_t *a_val, *b_val;
  int64_t cap_a, cap_b;
  // 2:4 form of the reduced operands: codes and position nibbles of P1 and P2, overflow flags
  int8_t *a24v1, *a24v2, *b24v1, *b24v2;
  uint8_t *a24n1, *a24n2, *b24n1, *b24n2;
  uint32_t *a24f, *b24f;
  // column-block split: per-k counts, the strip's k list and flag bitmap, strips of both operands
  int32_t *kcnt, *klist_a, *klist_b, *nstrip;   // kcnt is shared by the two operands (used one after the other)
  uint32_t *kflag_a, *kflag_b;
  int8_t *strip_a, *strip_rb, *strip_b, *strip_ra;
  size_t fixed_bytes;
};

int64_t tiles(int64_t n, int t) { return (n + t - 1) / t; }

// workspace per kept entry: index + value
constexpr double kBytesPerEntry = 5.0;

// Leading dimension of the K-contiguous code matrices in the workspace: K rounded up to a
// multiple of 128 with zeros in the padding, so that every row is 128-byte aligned and the
// matrix-core kernels take their aligned, full-K-tile paths whatever K is (zero codes add nothing).
int64_t code_ld(int64_t K) { return (K + 127) / 128 * 128; }

// Lays the fixed-size regions out; returns the bytes they take.  base may be null (sizing).
size_t plan_fixed(char* base, int64_t M, int64_t N, int64_t K, Plan* p) {
  Carver c{base, 0};
  const int64_t Kc = code_ld(K);
  size_t mk = (size_t)M * Kc, nk = (size_t)N * Kc;
  p->A_int = c.take<int8_t>(mk);
  p->B_int = c.take<int8_t>(nk);
  p->RA_int = c.take<int8_t>(mk);
  p->RB_int = c.take<int8_t>(nk);
  p->RA_em = c.take<int8_t>((size_t)M * K);
  p->RB_em = c.take<int8_t>((size_t)N * K);
  p->Ad = c.take<int8_t>(mk);
  p->Bd = c.take<int8_t>(nk);
  p->s_a = c.take<float>(M); p->lam_a = c.take<float>(M); p->s_ra = c.take<float>(M);
  p->lam_ra = c.take<float>(M); p->drow = c.take<float>(M); p->t_a = c.take<float>(M);
  p->s_b = c.take<float>(N); p->lam_b = c.take<float>(N); p->s_rb = c.take<float>(N);
  p->lam_rb = c.take<float>(N); p->dcol = c.take<float>(N); p->t_b = c.take<float>(N);
  p->amax_b = c.take<uint32_t>(N); p->ramax_b = c.take<uint32_t>(N);
  p->row_part = c.take<double>((size_t)tiles(N, gemm_tile_n()) * M);
  p->col_part = c.take<double>((size_t)tiles(M, gemm_tile_m()) * N);
  int64_t chk = select_chunks(K);
  p->cnt_a = c.take<int32_t>((size_t)chk * M); p->tot_a = c.take<int32_t>(M);
  p->a_ptr = c.take<int32_t>(M + 1);
  p->cnt_b = c.take<int32_t>((size_t)chk * N); p->tot_b = c.take<int32_t>(N);
  p->b_ptr = c.take<int32_t>(N + 1);
  p->nnz = c.take<int64_t>(2);
  p->paths = c.take<int32_t>(2);
  p->mask_a = c.take<uint64_t>((size_t)M * mask_words(K));
  p->mask_b = c.take<uint64_t>((size_t)N * mask_words(K));
  const size_t mk256 = (size_t)((M + 255) / 256 * 256) * Kc, nk256 = (size_t)((N + 255) / 256 * 256) * Kc;
  p->a24v1 = c.take<int8_t>(mk256 / 2); p->a24n1 = c.take<uint8_t>(mk256 / 8);
  p->a24v2 = c.take<int8_t>(mk256 / 2); p->a24n2 = c.take<uint8_t>(mk256 / 8);
  p->b24v1 = c.take<int8_t>(nk256 / 2); p->b24n1 = c.take<uint8_t>(nk256 / 8);
  p->b24v2 = c.take<int8_t>(nk256 / 2); p->b24n2 = c.take<uint8_t>(nk256 / 8);
  p->a24f = c.take<uint32_t>((size_t)sparse24_flag_words(M, Kc));
  p->b24f = c.take<uint32_t>((size_t)sparse24_flag_words(N, Kc));
  p->kcnt = c.take<int32_t>((size_t)mask_words(K) * 64);
  p->klist_a = c.take<int32_t>(kStripK); p->klist_b = c.take<int32_t>(kStripK);
  p->nstrip = c.take<int32_t>(2);
  p->kflag_a = c.take<uint32_t>((size_t)mask_words(K) * 2); p->kflag_b = c.take<uint32_t>((size_t)mask_words(K) * 2);
  p->strip_a = c.take<int8_t>((size_t)M * kStripK); p->strip_rb = c.take<int8_t>((size_t)N * kStripK);
  p->strip_b = c.take<int8_t>((size_t)N * kStripK); p->strip_ra = c.take<int8_t>((size_t)M * kStripK);
  p->fixed_bytes = c.off;
  return c.off;
}

// Splits what is left of the workspace into the two compressed operands.
bool plan_compressed(char* base, size_t bytes, int64_t M, int64_t N, int64_t K, Plan* p) {
  if (bytes < p->fixed_bytes + 8 * kAlign) { p->cap_a = p->cap_b = 0; return false; }
  size_t rest = bytes - p->fixed_bytes - 8 * kAlign;
  // 5 bytes per kept entry
  double total = (double)rest / kBytesPerEntry;
  double fa = (M + N) > 0 ? (double)M / (double)(M + N) : 0.5;
  int64_t cap_a = (int64_t)(total * fa), cap_b = (int64_t)(total * (1.0 - fa));
  int64_t max_a = M * K, max_b = N * K;
  if (cap_a > max_a) cap_a = max_a;
  if (cap_b > max_b) cap_b = max_b;
  const int64_t lim = 2147483647;
  if (cap_a > lim) cap_a = lim;
  if (cap_b > lim) cap_b = lim;
  p->cap_a = cap_a;
  p->cap_b = cap_b;
  if (base) {
    Carver c{base, p->fixed_bytes};
    p->a_idx = c.take<int32_t>(cap_a);
    p->a_val = c.take<int8_t>(cap_a);
    p->b_idx = c.take<int32_t>(cap_b);
    p->b_val = c.take<int8_t>(cap_b);
  }
  return true;
}

size_t stage_bytes(int64_t M, int64_t N, int64_t K) {
  size_t big = (size_t)(M > N ? M : N);
  size_t mx = big > (size_t)K ? big : (size_t)K;
  size_t b = 0;
  b += align_up(mx * 4) * 4;                                            // lambdas, totals, ptr
  b += align_up(((size_t)select_chunks(K) * big + (size_t)select_chunks(big) * K) * 4);  // counts
  b += align_up(((size_t)tiles(N, gemm_tile_n()) * M + (size_t)tiles(M, gemm_tile_m()) * N) * 8);
  b += align_up(big * K);                                               // expanded operand
  // srq_build_sparse_residual's streaming path on an operand of up to max(M,N) x K or K x max(M,N):
  // three vectors of per-vector values, the keep-mask and the codes (rows padded to 16)
  const size_t fast = align_up(mx * 4) * 3 + align_up((big * ((size_t)K + 63) / 64 + (size_t)K * ((big + 63) / 64)) * 8) +
                      align_up(big * (((size_t)K + 15) / 16 * 16) + (size_t)K * ((big + 15) / 16 * 16));
  if (b < fast) b = fast;
  return b + 8 * kAlign;
}

inline srq_status_t hip_fail(srq_handle_t h, hipError_t e) {
  if (h) h->last_hip_error = (int)e;
  return SRQ_STATUS_HIP_ERROR;
}

#define SRQ_HIP(h, expr)                                   \
  do {                                                     \
    hipError_t e__ = (expr);                               \
    if (e__ != hipSuccess) return hip_fail((h), e__);      \
  } while (0)

srq_status_t check_common(srq_handle_t h, int bits) {
  if (!h) return SRQ_STATUS_INVALID_ARG;
  if (bits < 2 || bits > 8) return SRQ_STATUS_UNSUPPORTED;
  return SRQ_STATUS_OK;
}

bool k_overflows(int64_t K, int qmax) { return K * (int64_t)qmax * qmax >= (1LL << 31); }

constexpr int kProfRing = 64;   // (the size of the arrays in the handle)

struct StageTimer {
  srq_handle_t h;
  hipStream_t st;
  int id;
  StageTimer(srq_handle_t h_, hipStream_t st_, int id_) : h(h_), st(st_), id(id_) {
    if (on()) {
      (void)hipEventRecord(h->prof_ev[h->prof_slot][2 * id], st);
      h->prof_used[h->prof_slot] |= 1u << id;
    }
  }
  ~StageTimer() {
    if (on()) (void)hipEventRecord(h->prof_ev[h->prof_slot][2 * id + 1], st);
  }
  bool on() const { return h->prof_enabled && ((h->prof_mask >> id) & 1u); }
};

srq_status_t bind_device(srq_handle_t h) {
  if (h->device < 0) return SRQ_STATUS_NO_DEVICE;
  SRQ_HIP(h, hipSetDevice(h->device));
  return SRQ_STATUS_OK;
}

}  // namespace

extern "C" {

const char* srq_status_string(srq_status_t s) {
  switch (s) {
    case SRQ_STATUS_OK: return "ok";
    case SRQ_STATUS_INVALID_ARG: return "invalid argument";
    case SRQ_STATUS_UNSUPPORTED: return "unsupported bit width";
    case SRQ_STATUS_K_OVERFLOW: return "K*qmax^2 overflows the INT32 accumulator";
    case SRQ_STATUS_CAPACITY: return "compressed-storage capacity too small";
    case SRQ_STATUS_WORKSPACE: return "workspace missing or too small";
    case SRQ_STATUS_HIP_ERROR: return "HIP runtime error";
    case SRQ_STATUS_NO_DEVICE: return "handle has no device";
  }
  return "unknown status";
}

srq_status_t srq_create(srq_handle_t* handle, int device) {
  if (!handle) return SRQ_STATUS_INVALID_ARG;
  *handle = nullptr;
  srq_context* c = new (std::nothrow) srq_context();
  if (!c) return SRQ_STATUS_INVALID_ARG;
  memset(c, 0, sizeof(*c));
  c->device = device;
  if (device >= 0) {
    int n = 0;
    hipError_t e = hipGetDeviceCount(&n);
    if (e != hipSuccess || device >= n) { delete c; return SRQ_STATUS_HIP_ERROR; }
    e = hipSetDevice(device);
    if (e == hipSuccess) e = hipHostMalloc(reinterpret_cast<void**>(&c->host_nnz), 4 * sizeof(int64_t), 0);
    if (e == hipSuccess) c->host_nnz[2] = 0;   // (the two executions the device reported last, see seen_paths)
    int cus = 0;
    if (e == hipSuccess) e = srq::gemm_device_cus(&cus);
    if (e != hipSuccess) { delete c; return SRQ_STATUS_HIP_ERROR; }
    // (a failure here only disables srq_gemm_i8_static_scratch, which then reports it)
    c->last_hip_error = (int)prime_static_scratch(device);
  }
  *handle = c;
  return SRQ_STATUS_OK;
}

// Two words of the handle's pinned host buffer into which the deciding kernel of SRQ_STRATEGY_AUTO
// stores, straight from the device, the execution it chose for each term: the next call on the
// handle reads them as its expectation without any synchronisation (whatever is there is only a
// hint: a stale or half-updated value costs time, never a result).
static volatile int32_t* seen_paths(srq_handle_t h) {
  return h->host_nnz ? reinterpret_cast<volatile int32_t*>(h->host_nnz + 2) : nullptr;
}

srq_status_t srq_set_scale_mode(srq_handle_t h, srq_scale_t mode) {
  if (!h || (mode != SRQ_SCALE_VECTOR && mode != SRQ_SCALE_GLOBAL)) return SRQ_STATUS_INVALID_ARG;
  h->scale_mode = (int)mode;
  return SRQ_STATUS_OK;
}

srq_status_t srq_set_auto_hint(srq_handle_t h, int path_a, int path_b) {
  if (!h || path_a < 0 || path_a > 2 || path_b < 0 || path_b > 2) return SRQ_STATUS_INVALID_ARG;
  h->last_path_a = path_a;
  h->last_path_b = path_b;
  if (volatile int32_t* seen = seen_paths(h)) { seen[0] = path_a; seen[1] = path_b; }
  return SRQ_STATUS_OK;
}

srq_status_t srq_profile_enable(srq_handle_t h, int enable) {
  if (!h) return SRQ_STATUS_INVALID_ARG;
  if (enable && !h->prof_created) {
    srq_status_t s = bind_device(h);
    if (s) return s;
    for (int r = 0; r < kProfRing; ++r)
      for (int i = 0; i < 2 * SRQ_NUM_STAGES; ++i) SRQ_HIP(h, hipEventCreate(&h->prof_ev[r][i]));
    h->prof_created = 1;
  }
  h->prof_enabled = enable ? 1 : 0;
  // (an event record keeps the kernel after it from starting under the tail of the one before:
  // about 3 us each, 0.044 ms over the sixteen of a call at 8192^3)
  h->prof_mask = enable == SRQ_PROFILE_PRODUCTS
                     ? (1u << SRQ_STAGE_GEMM) | (1u << SRQ_STAGE_TERM1) | (1u << SRQ_STAGE_TERM2)
                     : (1u << SRQ_NUM_STAGES) - 1u;
  h->prof_calls = 0;
  return SRQ_STATUS_OK;
}

srq_status_t srq_profile_read(srq_handle_t h, float* ms) {
  if (!h || !ms) return SRQ_STATUS_INVALID_ARG;
  for (int i = 0; i < SRQ_NUM_STAGES; ++i) ms[i] = 0.f;
  if (!h->prof_created) return SRQ_STATUS_OK;
  const int64_t n = h->prof_calls < kProfRing ? h->prof_calls : kProfRing;
  for (int64_t c = h->prof_calls - n; c < h->prof_calls; ++c) {
    const int r = (int)(c % kProfRing);
    for (int i = 0; i < SRQ_NUM_STAGES; ++i) {
      if (!(h->prof_used[r] & (1u << i))) continue;
      float t = 0.f;
      SRQ_HIP(h, hipEventSynchronize(h->prof_ev[r][2 * i + 1]));
      SRQ_HIP(h, hipEventElapsedTime(&t, h->prof_ev[r][2 * i], h->prof_ev[r][2 * i + 1]));
      ms[i] += t;
    }
  }
  h->prof_calls = 0;
  return SRQ_STATUS_OK;
}

srq_status_t srq_destroy(srq_handle_t h) {
  if (!h) return SRQ_STATUS_INVALID_ARG;
  if (h->prof_created)
    for (int r = 0; r < kProfRing; ++r)
      for (int i = 0; i < 2 * SRQ_NUM_STAGES; ++i) (void)hipEventDestroy(h->prof_ev[r][i]);
  if (h->host_nnz) (void)hipHostFree(h->host_nnz);
  delete h;
  return SRQ_STATUS_OK;
}

int srq_last_hip_error(srq_handle_t h) { return h ? h->last_hip_error : 0; }

srq_status_t srq_workspace_bytes(int64_t M, int64_t N, int64_t K, double max_density, size_t* bytes) {
  if (!bytes || M < 0 || N < 0 || K < 0 || !(max_density >= 0.0) || max_density > 1.0)
    return SRQ_STATUS_INVALID_ARG;
  Plan p;
  size_t fixed = plan_fixed(nullptr, M, N, K, &p);
  // the capacity is shared out in proportion to the operand sizes, so size for the larger
  double entries = max_density * (double)K * (double)(M + N) + 1024.0;
  size_t total = fixed + 8 * kAlign + (size_t)(entries * kBytesPerEntry) + 64;
  size_t st = stage_bytes(M, N, K);
  *bytes = align_up(total > st ? total : st);
  return SRQ_STATUS_OK;
}

srq_status_t srq_stage_workspace_bytes(int64_t M, int64_t N, int64_t K, size_t* bytes) {
  if (!bytes || M < 0 || N < 0 || K < 0) return SRQ_STATUS_INVALID_ARG;
  *bytes = stage_bytes(M, N, K);
  return SRQ_STATUS_OK;
}

srq_status_t srq_set_workspace(srq_handle_t h, void* ws, size_t bytes) {
  if (!h) return SRQ_STATUS_INVALID_ARG;
  if (ws && (reinterpret_cast<uintptr_t>(ws) % kAlign) != 0) return SRQ_STATUS_INVALID_ARG;
  h->ws = ws;
  h->ws_bytes = ws ? bytes : 0;
  memset(&h->last, 0, sizeof(h->last));
  return SRQ_STATUS_OK;
}

srq_status_t srq_get_intermediates(srq_handle_t h, srq_intermediates_t* out) {
  if (!h || !out) return SRQ_STATUS_INVALID_ARG;
  *out = h->last;
  return SRQ_STATUS_OK;
}

// ------------------------------------------------------------------------------------------
srq_status_t srq_quantize(srq_handle_t h, const float* X, int64_t rows, int64_t cols, int64_t ldx,
                          srq_axis_t axis, int bits, srq_round_t round, srq_layout_t layout,
                          int8_t* Q, int64_t ldq, float* scale, float* lambda, void* stream) {
  srq_status_t s = check_common(h, bits);
  if (s) return s;
  if (rows < 0 || cols < 0) return SRQ_STATUS_INVALID_ARG;
  if (axis != SRQ_AXIS_ROW && axis != SRQ_AXIS_COL) return SRQ_STATUS_INVALID_ARG;
  if (round != SRQ_ROUND_NEAREST_EVEN && round != SRQ_ROUND_TRUNC) return SRQ_STATUS_INVALID_ARG;
  if (layout != SRQ_LAYOUT_VECTOR_MAJOR && layout != SRQ_LAYOUT_ELEMENT_MAJOR) return SRQ_STATUS_INVALID_ARG;
  int64_t nvec = axis == SRQ_AXIS_ROW ? rows : cols, veclen = axis == SRQ_AXIS_ROW ? cols : rows;
  if (rows == 0 || cols == 0) {
    // no codes; scales of empty vectors are zero, nothing to validate beyond the handle
    if (nvec > 0 && !scale) return SRQ_STATUS_INVALID_ARG;
  } else {
    if (!X || !Q || !scale) return SRQ_STATUS_INVALID_ARG;
    if (ldx < cols) return SRQ_STATUS_INVALID_ARG;
    if (ldq < (layout == SRQ_LAYOUT_VECTOR_MAJOR ? veclen : nvec)) return SRQ_STATUS_INVALID_ARG;
  }
  float* lam = lambda;
  if (!lam && rows > 0 && cols > 0) {
    if (!h->ws || h->ws_bytes < align_up((size_t)nvec * 4)) return SRQ_STATUS_WORKSPACE;
    lam = reinterpret_cast<float*>(h->ws);
  }
  s = bind_device(h);
  if (s) return s;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  int qmax = qmax_of_bits(bits);
  if (nvec == 0) return SRQ_STATUS_OK;
  const int trunc = round == SRQ_ROUND_TRUNC;
  // streaming kernels for aligned operands: rows in one pass, columns in two
  if (rows > 0 && cols > 0 && axis == SRQ_AXIS_ROW && layout == SRQ_LAYOUT_VECTOR_MAJOR &&
      rows_fused_ok(X, cols, ldx, Q, ldq, nullptr, 0)) {
    SRQ_HIP(h, launch_rows_fused(X, rows, cols, ldx, qmax, trunc, Q, ldq, scale, lam, nullptr, 0, nullptr,
                                 nullptr, st));
    return SRQ_STATUS_OK;
  }
  SRQ_HIP(h, launch_fill_u32(reinterpret_cast<uint32_t*>(scale), nvec, 0, st));
  if (rows == 0 || cols == 0) {
    if (lambda) SRQ_HIP(h, launch_fill_u32(reinterpret_cast<uint32_t*>(lambda), nvec, 0, st));
    return SRQ_STATUS_OK;
  }
  // (the column kernels store 16 codes of a vector, resp. 4 codes of a row, at a time: the
  // caller's Q must be aligned for that, otherwise the generic kernels run)
  const uintptr_t qaddr = reinterpret_cast<uintptr_t>(Q);
  const bool q_ok = layout == SRQ_LAYOUT_VECTOR_MAJOR ? ((qaddr % 16) == 0 && (ldq % 16) == 0)
                                                      : ((qaddr % 4) == 0 && (ldq % 4) == 0);
  if (axis == SRQ_AXIS_COL && cols_pass_ok(X, cols, ldx) && q_ok) {
    const bool vm = layout == SRQ_LAYOUT_VECTOR_MAJOR;
    SRQ_HIP(h, launch_cols_amax(X, rows, cols, ldx, reinterpret_cast<uint32_t*>(scale), st));
    SRQ_HIP(h, launch_scales(reinterpret_cast<uint32_t*>(scale), lam, nvec, qmax, st));
    SRQ_HIP(h, launch_cols_codes(X, rows, cols, ldx, qmax, trunc, scale, lam, vm ? Q : nullptr, ldq,
                                 vm ? nullptr : Q, ldq, nullptr, st));
    return SRQ_STATUS_OK;
  }
  SRQ_HIP(h, launch_amax(X, rows, cols, ldx, axis, reinterpret_cast<uint32_t*>(scale), st));
  SRQ_HIP(h, launch_scales(reinterpret_cast<uint32_t*>(scale), lam, nvec, qmax, st));
  SRQ_HIP(h, launch_quantize_tiles(X, rows, cols, ldx, axis, scale, lam, qmax, trunc, layout, Q, ldq, nullptr,
                                   st));
  return SRQ_STATUS_OK;
}

// ------------------------------------------------------------------------------------------
srq_status_t srq_build_sparse_residual(srq_handle_t h, const float* X, int64_t rows, int64_t cols,
                                       int64_t ldx, srq_axis_t axis, const float* scale,
                                       const float* lambda, const float* thresh, int bits,
                                       srq_round_t round, int8_t* Rq, int64_t ldr, srq_layout_t r_layout,
                                       float* rscale, int32_t* ptr, int32_t* idx, int8_t* val,
                                       int64_t capacity, int64_t* nnz_dev, void* stream) {
  srq_status_t s = check_common(h, bits);
  if (s) return s;
  if (rows < 0 || cols < 0) return SRQ_STATUS_INVALID_ARG;
  if (axis != SRQ_AXIS_ROW && axis != SRQ_AXIS_COL) return SRQ_STATUS_INVALID_ARG;
  if (round != SRQ_ROUND_NEAREST_EVEN && round != SRQ_ROUND_TRUNC) return SRQ_STATUS_INVALID_ARG;
  if (r_layout != SRQ_LAYOUT_VECTOR_MAJOR && r_layout != SRQ_LAYOUT_ELEMENT_MAJOR) return SRQ_STATUS_INVALID_ARG;
  const bool do_res = Rq || rscale, do_sel = ptr || idx || val;
  if (do_res && (!Rq || !rscale)) return SRQ_STATUS_INVALID_ARG;
  if (do_sel && (!ptr || !thresh || capacity < 0 || (capacity > 0 && (!idx || !val)))) return SRQ_STATUS_INVALID_ARG;
  if (capacity > 2147483647LL) return SRQ_STATUS_INVALID_ARG;
  if (do_sel && rows > 0 && cols > 0 && rows > 2147483647LL / cols) return SRQ_STATUS_UNSUPPORTED;   // INT32 ptr
  int64_t nvec = axis == SRQ_AXIS_ROW ? rows : cols, veclen = axis == SRQ_AXIS_ROW ? cols : rows;
  if (rows > 0 && cols > 0) {
    if (!X || !scale || !lambda) return SRQ_STATUS_INVALID_ARG;
    if (ldx < cols) return SRQ_STATUS_INVALID_ARG;
    if (do_res && ldr < (r_layout == SRQ_LAYOUT_VECTOR_MAJOR ? veclen : nvec)) return SRQ_STATUS_INVALID_ARG;
  }
  int64_t nch = select_chunks(veclen);
  size_t need = align_up((size_t)nvec * 4) * 2 + align_up((size_t)nch * nvec * 4) + kAlign;
  if (nvec > 0 && (!h->ws || h->ws_bytes < need)) return SRQ_STATUS_WORKSPACE;
  s = bind_device(h);
  if (s) return s;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  int qmax = qmax_of_bits(bits), trunc = round == SRQ_ROUND_TRUNC;
  // ---- streaming kernels for aligned operands (the kernels of the whole-path call): codes of X go
  // to the workspace, the keep-mask is built in one more read of X and compacted from there
  if (rows > 0 && cols > 0) {
    const int64_t ldqw = (veclen + 15) / 16 * 16;
    Carver f{reinterpret_cast<char*>(h->ws), 0};
    float* rlam_w = f.take<float>(nvec);
    int32_t* tot_w = f.take<int32_t>(nvec);
    uint32_t* ramax_w = f.take<uint32_t>(nvec);
    uint64_t* mask_w = f.take<uint64_t>((size_t)nvec * mask_words(veclen));
    int8_t* q_w = f.take<int8_t>((size_t)nvec * ldqw);
    const bool fits = f.off <= h->ws_bytes;
    const bool vm = r_layout == SRQ_LAYOUT_VECTOR_MAJOR;
    auto al16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; };
    if (fits && axis == SRQ_AXIS_ROW && (!do_res || vm) &&
        rows_fused_ok(X, cols, ldx, q_w, ldqw, do_res ? Rq : nullptr, ldr)) {
      SRQ_HIP(h, launch_rows_fused(X, rows, cols, ldx, qmax, trunc, q_w, ldqw, nullptr, nullptr, do_res ? Rq : nullptr,
                                   ldr, do_res ? rscale : nullptr, do_res ? rlam_w : nullptr, st, scale, lambda));
      if (do_sel) {
        SRQ_HIP(h, launch_rows_mask(X, rows, cols, ldx, thresh, mask_w, tot_w, st));
        SRQ_HIP(h, launch_scan_pair(tot_w, nvec, ptr, nnz_dev, nullptr, 0, nullptr, nullptr, st));
        SRQ_HIP(h, launch_scatter_mask(mask_w, nvec, veclen, q_w, ldqw, ptr, idx, val, capacity, nullptr, 0, -1, st));
      }
      return SRQ_STATUS_OK;
    }
    const bool r_ok = !do_res || (al16(rscale) && (vm ? (al16(Rq) && (ldr % 16) == 0)
                                                    : ((reinterpret_cast<uintptr_t>(Rq) & 3) == 0 && (ldr % 4) == 0)));
    if (fits && axis == SRQ_AXIS_COL && cols_pass_ok(X, cols, ldx) && al16(scale) && al16(lambda) &&
        (!do_sel || al16(thresh)) && r_ok) {
      SRQ_HIP(h, launch_fill3_u32(ramax_w, nvec, reinterpret_cast<uint32_t*>(tot_w), nvec, nullptr, 0, st));
      SRQ_HIP(h, launch_cols_codes(X, rows, cols, ldx, qmax, trunc, scale, lambda, q_w, ldqw, nullptr, 0,
                                   do_res ? ramax_w : nullptr, st));
      if (do_res && do_sel)
        SRQ_HIP(h, launch_cols_mask_resid(X, rows, cols, ldx, qmax, trunc, scale, lambda, ramax_w, rscale, rlam_w,
                                          vm ? Rq : nullptr, ldr, vm ? nullptr : Rq, ldr, thresh, mask_w, tot_w, st));
      else if (do_res)
        SRQ_HIP(h, launch_cols_resid_from_amax(X, rows, cols, ldx, qmax, trunc, scale, lambda, ramax_w, rscale, rlam_w,
                                               vm ? Rq : nullptr, ldr, vm ? nullptr : Rq, ldr, st));
      else if (do_sel)
        SRQ_HIP(h, launch_cols_mask(X, rows, cols, ldx, thresh, mask_w, tot_w, st));
      if (do_sel) {
        SRQ_HIP(h, launch_scan_pair(tot_w, nvec, ptr, nnz_dev, nullptr, 0, nullptr, nullptr, st));
        SRQ_HIP(h, launch_scatter_mask(mask_w, nvec, veclen, q_w, ldqw, ptr, idx, val, capacity, nullptr, 0, -1, st));
      }
      return SRQ_STATUS_OK;
    }
  }
  Carver c{reinterpret_cast<char*>(h->ws), 0};
  float* rlam = c.take<float>(nvec);
  int32_t* totals = c.take<int32_t>(nvec);
  int32_t* cnt = c.take<int32_t>((size_t)nch * nvec);
  if (do_res && nvec > 0) {
    SRQ_HIP(h, launch_fill_u32(reinterpret_cast<uint32_t*>(rscale), nvec, 0, st));
    SRQ_HIP(h, launch_quantize_tiles(X, rows, cols, ldx, axis, scale, lambda, qmax, trunc,
                                     SRQ_LAYOUT_VECTOR_MAJOR, nullptr, 0,
                                     reinterpret_cast<uint32_t*>(rscale), st));
    SRQ_HIP(h, launch_scales(reinterpret_cast<uint32_t*>(rscale), rlam, nvec, qmax, st));
    bool vm = r_layout == SRQ_LAYOUT_VECTOR_MAJOR;
    SRQ_HIP(h, launch_residual_tiles(X, rows, cols, ldx, axis, scale, lambda, rlam, qmax, trunc,
                                     vm ? Rq : nullptr, ldr, vm ? nullptr : Rq, ldr, st));
  }
  if (do_sel) {
    SRQ_HIP(h, launch_select_count(X, rows, cols, ldx, axis, thresh, cnt, st));
    SRQ_HIP(h, launch_select_scan(cnt, nvec, (rows > 0 && cols > 0) ? nch : 0, totals, ptr, nnz_dev, st));
    SRQ_HIP(h, launch_select_scatter(X, rows, cols, ldx, axis, thresh, lambda, qmax, trunc, ptr, cnt, idx,
                                     val, capacity, st));
  }
  return SRQ_STATUS_OK;
}

// ------------------------------------------------------------------------------------------
// The first product with its means; `scratch` = where the partial sums of |D_F| go: the handle's
// workspace (use_static false) or this device's copy of the library's static scratch array.
static srq_status_t gemm_i8_impl(srq_handle_t h, int64_t M, int64_t N, int64_t K, const int8_t* Qa, int64_t lda,
                                 const float* sa, const int8_t* Qb, int64_t ldb, const float* sb, float* D_F,
                                 int32_t* D_int, int64_t ldd, float* drow, float* dcol, void* stream,
                                 bool use_static) {
  if (!h) return SRQ_STATUS_INVALID_ARG;
  if (M < 0 || N < 0 || K < 0) return SRQ_STATUS_INVALID_ARG;
  if (k_overflows(K, 128)) return SRQ_STATUS_K_OVERFLOW;     // codes may use the full int8 range
  if (M > 0 && N > 0) {
    if (!sa || !sb || !D_F || ldd < N) return SRQ_STATUS_INVALID_ARG;
    if (K > 0 && (!Qa || !Qb || lda < K || ldb < K)) return SRQ_STATUS_INVALID_ARG;
  }
  if ((drow == nullptr) != (dcol == nullptr)) return SRQ_STATUS_INVALID_ARG;
  size_t need = align_up((size_t)tiles(N, gemm_tile_n()) * M * 8) + align_up((size_t)tiles(M, gemm_tile_m()) * N * 8);
  if (drow && M > 0 && N > 0) {
    // (a problem whose partial sums do not fit is refused before anything is launched)
    if (use_static ? need > kStaticScratchBytes : (!h->ws || h->ws_bytes < need)) return SRQ_STATUS_WORKSPACE;
  }
  srq_status_t s = bind_device(h);
  if (s) return s;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  if (M == 0 || N == 0) return SRQ_STATUS_OK;
  GemmEpilogue ep;
  memset(&ep, 0, sizeof(ep));
  ep.mode = kGemmFirst;
  ep.s_row = sa; ep.s_col = sb; ep.C = D_F; ep.ldc = ldd; ep.D_int = D_int; ep.ldd = ldd;
  ep.alpha = 1.f;
  if (drow) {
    char* base = reinterpret_cast<char*>(h->ws);
    if (use_static) {
      base = static_scratch_of(h->device);
      // (no address: the lookup at srq_create failed, or the device number is out of range)
      if (!base) return hip_fail(h, g_scratch_error != hipSuccess ? g_scratch_error : hipErrorInvalidDevice);
    }
    Carver c{base, 0};
    ep.row_part = c.take<double>((size_t)tiles(N, gemm_tile_n()) * M);
    ep.col_part = c.take<double>((size_t)tiles(M, gemm_tile_m()) * N);
  }
  SRQ_HIP(h, launch_gemm_i8(M, N, K, Qa, lda, Qb, ldb, ep, st));
  if (drow) {
    // (the persistent kernel leaves one partial per wave, two per 256-wide tile)
    int64_t parts_n, parts_m;
    gemm_sum_parts(M, N, K, Qa, lda, Qb, ldb, ep, &parts_n, &parts_m);
    SRQ_HIP(h, launch_reduce_means_pair(ep.row_part, parts_n, M, N, 0.f, drow, nullptr, ep.col_part, parts_m, N, M, 0.f,
                                        dcol, nullptr, st));
  }
  return SRQ_STATUS_OK;
}

srq_status_t srq_gemm_i8(srq_handle_t h, int64_t M, int64_t N, int64_t K, const int8_t* Qa, int64_t lda,
                         const float* sa, const int8_t* Qb, int64_t ldb, const float* sb, float* D_F,
                         int32_t* D_int, int64_t ldd, float* drow, float* dcol, void* stream) {
  return gemm_i8_impl(h, M, N, K, Qa, lda, sa, Qb, ldb, sb, D_F, D_int, ldd, drow, dcol, stream, false);
}

srq_status_t srq_gemm_i8_static_scratch(srq_handle_t h, int64_t M, int64_t N, int64_t K, const int8_t* Qa,
                                        int64_t lda, const float* sa, const int8_t* Qb, int64_t ldb,
                                        const float* sb, float* D_F, int32_t* D_int, int64_t ldd, float* drow,
                                        float* dcol, void* stream) {
  return gemm_i8_impl(h, M, N, K, Qa, lda, sa, Qb, ldb, sb, D_F, D_int, ldd, drow, dcol, stream, true);
}

size_t srq_static_scratch_bytes(void) { return kStaticScratchBytes; }

// ------------------------------------------------------------------------------------------
srq_status_t srq_spmm_accumulate(srq_handle_t h, srq_axis_t side, srq_strategy_t strategy, int64_t M,
                                 int64_t N, int64_t K, const int32_t* ptr, const int32_t* idx,
                                 const int8_t* val, const int8_t* Rq, int64_t ldr, const float* s_row,
                                 const float* s_col, float* C, int32_t* DR_int, int64_t ldc, void* stream) {
  if (!h) return SRQ_STATUS_INVALID_ARG;
  if (M < 0 || N < 0 || K < 0) return SRQ_STATUS_INVALID_ARG;
  if (side != SRQ_AXIS_ROW && side != SRQ_AXIS_COL) return SRQ_STATUS_INVALID_ARG;
  if (strategy != SRQ_STRATEGY_CSR_VALU && strategy != SRQ_STRATEGY_CSR_MFMA) return SRQ_STATUS_INVALID_ARG;
  if (k_overflows(K, 128)) return SRQ_STATUS_K_OVERFLOW;
  int64_t nvec = side == SRQ_AXIS_ROW ? M : N, nelem = side == SRQ_AXIS_ROW ? N : M;
  if (M > 0 && N > 0) {
    if (!ptr || !s_row || !s_col || !C || ldc < N) return SRQ_STATUS_INVALID_ARG;
    if (K > 0) {
      if (!Rq) return SRQ_STATUS_INVALID_ARG;
      if (ldr < (strategy == SRQ_STRATEGY_CSR_VALU ? nelem : K)) return SRQ_STATUS_INVALID_ARG;
    }
  }
  size_t need = align_up((size_t)nvec * K) + kAlign;
  if (strategy == SRQ_STRATEGY_CSR_MFMA && M > 0 && N > 0 && K > 0 && (!h->ws || h->ws_bytes < need))
    return SRQ_STATUS_WORKSPACE;
  srq_status_t s = bind_device(h);
  if (s) return s;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  if (M == 0 || N == 0) return SRQ_STATUS_OK;
  GemmEpilogue ep;
  memset(&ep, 0, sizeof(ep));
  ep.mode = kGemmAccum;
  ep.s_row = s_row; ep.s_col = s_col; ep.C = C; ep.ldc = ldc; ep.D_int = DR_int; ep.ldd = ldc;
  ep.alpha = 1.f;
  const int64_t cap = 2147483647LL;
  if (strategy == SRQ_STRATEGY_CSR_VALU) {
    SRQ_HIP(h, launch_spmm_valu(side == SRQ_AXIS_ROW ? 0 : 1, nvec, nelem, K, ptr, nullptr, idx, val, cap, Rq, ldr, ep, st));
  } else {
    int8_t* dense = reinterpret_cast<int8_t*>(h->ws);
    int64_t ldd = (K + 15) / 16 * 16;
    if ((size_t)nvec * ldd > h->ws_bytes) ldd = K;
    SRQ_HIP(h, launch_densify(ptr, idx, val, nvec, K, cap, dense, ldd, st));
    if (side == SRQ_AXIS_ROW)
      SRQ_HIP(h, launch_gemm_i8(M, N, K, dense, ldd, Rq, ldr, ep, st));
    else
      SRQ_HIP(h, launch_gemm_i8(M, N, K, Rq, ldr, dense, ldd, ep, st));
  }
  return SRQ_STATUS_OK;
}

// ------------------------------------------------------------------------------------------
srq_status_t srq_compensated_gemm(srq_handle_t h, int64_t M, int64_t N, int64_t K, const float* A,
                                  int64_t lda, const float* B, int64_t ldb, float theta_a, float theta_b,
                                  int bits, srq_round_t round, float dense_fallback_density,
                                  srq_strategy_t strategy, float alpha, float beta, const float* Cin,
                                  int64_t ldcin, float* C, int64_t ldc, srq_stats_t* stats_dev,
                                  const srq_debug_t* dbg, void* stream) {
  srq_status_t s = check_common(h, bits);
  if (s) return s;
  if (M < 0 || N < 0 || K < 0) return SRQ_STATUS_INVALID_ARG;
  if (round != SRQ_ROUND_NEAREST_EVEN && round != SRQ_ROUND_TRUNC) return SRQ_STATUS_INVALID_ARG;
  if (strategy != SRQ_STRATEGY_AUTO && strategy != SRQ_STRATEGY_CSR_VALU && strategy != SRQ_STRATEGY_CSR_MFMA &&
      strategy != SRQ_STRATEGY_CSR_SMFMAC && strategy != SRQ_STRATEGY_COLBLOCK)
    return SRQ_STATUS_INVALID_ARG;
  if (isnan(theta_a) || isnan(theta_b) || theta_a < 0.f || theta_b < 0.f) return SRQ_STATUS_INVALID_ARG;
  if (isnan(dense_fallback_density) || isnan(alpha) || isnan(beta)) return SRQ_STATUS_INVALID_ARG;
  const int qmax = qmax_of_bits(bits);
  if (k_overflows(K, qmax)) return SRQ_STATUS_K_OVERFLOW;
  if (M > 0 && N > 0) {
    if (!C || ldc < N) return SRQ_STATUS_INVALID_ARG;
    if (beta != 0.f && (!Cin || ldcin < N)) return SRQ_STATUS_INVALID_ARG;
    if (K > 0 && (!A || !B || lda < K || ldb < N)) return SRQ_STATUS_INVALID_ARG;
  }
  const bool term_a = !isinf(theta_a), term_b = !isinf(theta_b);
  const bool comp = (term_a || term_b) && K > 0;
  // row pointers of the compressed operands are INT32: an operand that could keep 2^31 entries
  // or more is refused rather than risking a wrapped pointer
  if (comp && ((term_a && M * K > 2147483647LL) || (term_b && N * K > 2147483647LL))) return SRQ_STATUS_UNSUPPORTED;
  Plan p;
  memset(&p, 0, sizeof(p));
  plan_fixed(nullptr, M, N, K, &p);
  if (M > 0 && N > 0) {
    if (!h->ws || h->ws_bytes < p.fixed_bytes) return SRQ_STATUS_WORKSPACE;
    if (comp && !plan_compressed(nullptr, h->ws_bytes, M, N, K, &p)) return SRQ_STATUS_WORKSPACE;
  }
  s = bind_device(h);
  if (s) return s;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  if (M == 0 || N == 0) return SRQ_STATUS_OK;

  char* base = reinterpret_cast<char*>(h->ws);
  plan_fixed(base, M, N, K, &p);
  if (comp) plan_compressed(base, h->ws_bytes, M, N, K, &p);
  const int trunc = round == SRQ_ROUND_TRUNC;
  const bool scale_needed = alpha != 1.f || beta != 0.f;
  const int64_t Kc = code_ld(K);                 // leading dimension of the K-contiguous code matrices
  if (strategy == SRQ_STRATEGY_AUTO) {
    // Problems that the small-tile matrix-core kernel takes: both correction products cost so little
    // there (one launch of 36 us at 2048^3) that the vector ALUs never win, whatever the density
    // (measured down to 0.1 %: 0.157 against 0.179 ms per call), so nothing is left to decide.
    GemmEpilogue probe;
    memset(&probe, 0, sizeof(probe));
    probe.mode = kGemmAccum;
    if (gemm_small_ok(M, N, Kc, p.A_int, Kc, p.B_int, Kc, probe)) strategy = SRQ_STRATEGY_CSR_MFMA;
  }

  srq_intermediates_t& im = h->last;
  memset(&im, 0, sizeof(im));
  im.ld_codes = Kc;
  im.A_int = p.A_int; im.B_int = p.B_int; im.s_a = p.s_a; im.lam_a = p.lam_a; im.s_b = p.s_b; im.lam_b = p.lam_b;

  if (h->prof_enabled) {
    h->prof_slot = (int)(h->prof_calls % kProfRing);
    h->prof_used[h->prof_slot] = 0;
    ++h->prof_calls;
  }
  // the one-pass kernels derive each vector's scale from the data they hold; a matrix-wide
  // scale needs all maxima first: one more pass, then the same kernels with the scales given
  const bool global_scale = h->scale_mode == SRQ_SCALE_GLOBAL;
  const bool fastA = K > 0 && rows_fused_ok(A, K, lda, p.A_int, Kc, p.RA_int, Kc);
  const bool fastB = K > 0 && cols_pass_ok(B, N, ldb);
  bool ra_vm_done = false, ra_em_done = false, rb_vm_done = false, rb_em_done = false;
  bool rb_in_select = false, rb_want_em = false, rb_want_vm = false;   // residual codes of B left to the selection pass
  // lines 1: Quant.  amax per vector -> scale, lambda -> codes (and max |residual| per vector)
  {
  StageTimer tm(h, st, SRQ_STAGE_QUANTIZE);
  if (Kc != K) {
    // the padding columns of every matrix a product may read (nothing else ever writes them)
    int8_t* mats[6] = {p.A_int, p.B_int, comp ? p.RA_int : nullptr, comp ? p.RB_int : nullptr,
                       comp ? p.Ad : nullptr, comp ? p.Bd : nullptr};
    const int64_t nrows[6] = {M, N, M, N, M, N};
    SRQ_HIP(h, launch_zero_pad(mats, nrows, 6, K, Kc, st));
  }
  if (strategy == SRQ_STRATEGY_AUTO && dense_fallback_density > 1.f) {
    // where the device-side decision of the previous calls went (or the caller's hint)
    if (volatile int32_t* seen = seen_paths(h)) {
      const int sa = seen[0], sb = seen[1];
      if (sa == kPathValu || sa == kPathMfma) h->last_path_a = sa;
      if (sb == kPathValu || sb == kPathMfma) h->last_path_b = sb;
    }
  }
  // the two vectors of column maxima and the per-column counts of the selection that B's passes
  // accumulate into start at zero
  const ClearList b_clear = {p.amax_b, N, comp ? p.ramax_b : nullptr, N,
                             (comp && term_b) ? reinterpret_cast<uint32_t*>(p.tot_b) : nullptr, N};
  bool b_cleared = false;
  // operand A: vectors are contiguous rows
  if (fastA) {
    // the K-contiguous residual codes of A feed the matrix-core executions of term 2; when that
    // term is expected on the vector ALUs (same prediction as for B's layouts below) only the
    // residual scales are produced here and A's selection pass writes the k-major codes
    const bool skip_ra_vm = comp && term_b && dense_fallback_density > 1.f &&
                            (strategy == SRQ_STRATEGY_CSR_VALU ||
                             (strategy == SRQ_STRATEGY_AUTO && h->last_path_b == kPathValu));
    // (SRQ_STRATEGY_AUTO goes by the caller's hint, srq_set_auto_hint; a wrong or missing hint only
    // costs the pass that writes the other layout once the decision is known)
    // (this launch also zeroes what B's passes accumulate into, see below)
    b_cleared = fastB && rows_fused_can_clear(M, b_clear);
    if (global_scale) {
      // one scale for the whole matrix: the maximum first (one more read of A), then the one-pass
      // kernel with the scales given; the residual codes keep a scale per row
      SRQ_HIP(h, launch_fill_u32(reinterpret_cast<uint32_t*>(p.s_a), M, 0, st));
      SRQ_HIP(h, launch_amax(A, M, K, lda, SRQ_AXIS_ROW, reinterpret_cast<uint32_t*>(p.s_a), st));
      SRQ_HIP(h, launch_broadcast_max(reinterpret_cast<uint32_t*>(p.s_a), M, st));
      SRQ_HIP(h, launch_scales(reinterpret_cast<uint32_t*>(p.s_a), p.lam_a, M, qmax, st));
    }
    SRQ_HIP(h, launch_rows_fused(A, M, K, lda, qmax, trunc, p.A_int, Kc, p.s_a, p.lam_a,
                                 (comp && !skip_ra_vm) ? p.RA_int : nullptr, Kc, comp ? p.s_ra : nullptr,
                                 comp ? p.lam_ra : nullptr, st, global_scale ? p.s_a : nullptr,
                                 global_scale ? p.lam_a : nullptr, b_cleared ? &b_clear : nullptr));
    ra_vm_done = comp && !skip_ra_vm;
  } else {
    SRQ_HIP(h, launch_fill_u32(reinterpret_cast<uint32_t*>(p.s_a), M, 0, st));
    if (comp) SRQ_HIP(h, launch_fill_u32(reinterpret_cast<uint32_t*>(p.s_ra), M, 0, st));
    SRQ_HIP(h, launch_amax(A, M, K, lda, SRQ_AXIS_ROW, reinterpret_cast<uint32_t*>(p.s_a), st));
    if (global_scale) SRQ_HIP(h, launch_broadcast_max(reinterpret_cast<uint32_t*>(p.s_a), M, st));
    SRQ_HIP(h, launch_scales(reinterpret_cast<uint32_t*>(p.s_a), p.lam_a, M, qmax, st));
    SRQ_HIP(h, launch_quantize_tiles(A, M, K, lda, SRQ_AXIS_ROW, p.s_a, p.lam_a, qmax, trunc,
                                     SRQ_LAYOUT_VECTOR_MAJOR, p.A_int, Kc,
                                     comp ? reinterpret_cast<uint32_t*>(p.s_ra) : nullptr, st));
    if (comp) SRQ_HIP(h, launch_scales(reinterpret_cast<uint32_t*>(p.s_ra), p.lam_ra, M, qmax, st));
  }
  // operand B: vectors are the columns of a row-major matrix; codes are stored transposed
  if (fastB) {
    // (cleared by A's pass where that ran, else by a launch of its own); the code and residual
    // passes derive the scales from the maxima themselves
    if (!b_cleared) SRQ_HIP(h, launch_fill3_u32(b_clear.a, b_clear.na, b_clear.b, b_clear.nb, b_clear.c, b_clear.nc, st));
    SRQ_HIP(h, launch_cols_amax(B, K, N, ldb, p.amax_b, st));
    // (one scale for the whole matrix: every column takes the largest of the maxima)
    if (global_scale) SRQ_HIP(h, launch_broadcast_max(p.amax_b, N, st));
    SRQ_HIP(h, launch_cols_codes_from_amax(B, K, N, ldb, qmax, trunc, p.amax_b, p.s_b, p.lam_b, p.B_int, Kc,
                                           comp ? p.ramax_b : nullptr, st));
    if (comp) {
      // the K-contiguous residual codes feed the matrix-core paths; the k-major copy is only
      // written now if the caller has fixed the vector-ALU path for term 1
      // (or, with SRQ_STRATEGY_AUTO, if the previous call on this handle ended up there: repeated
      // calls at a similar density then write the layout they need here and not in a second pass;
      // a wrong guess only costs that second pass)
      // (the 2:4 path reads both: K-contiguous codes on the matrix cores, k-major ones for its spill)
      const int expect_a = strategy == SRQ_STRATEGY_AUTO ? h->last_path_a : strategy_path(strategy);
      const bool want_em = term_a && dense_fallback_density > 1.f && path_reads_em(expect_a);
      const bool want_vm = !want_em || path_reads_vm(expect_a);
      // when B's selection pass will run it writes these codes too (one read of B less)
      rb_in_select = term_b;
      rb_want_em = want_em;
      rb_want_vm = want_vm;
      if (!rb_in_select)
        SRQ_HIP(h, launch_cols_resid_from_amax(B, K, N, ldb, qmax, trunc, p.s_b, p.lam_b, p.ramax_b, p.s_rb,
                                               p.lam_rb, want_vm ? p.RB_int : nullptr, Kc,
                                               want_em ? p.RB_em : nullptr, N, st));
      rb_vm_done = want_vm;
      rb_em_done = want_em;
    }
  } else {
    SRQ_HIP(h, launch_fill3_u32(reinterpret_cast<uint32_t*>(p.s_b), N,
                                comp ? reinterpret_cast<uint32_t*>(p.s_rb) : nullptr, N, nullptr, 0, st));
    SRQ_HIP(h, launch_amax(B, K, N, ldb, SRQ_AXIS_COL, reinterpret_cast<uint32_t*>(p.s_b), st));
    if (global_scale) SRQ_HIP(h, launch_broadcast_max(reinterpret_cast<uint32_t*>(p.s_b), N, st));
    SRQ_HIP(h, launch_scales(reinterpret_cast<uint32_t*>(p.s_b), p.lam_b, N, qmax, st));
    SRQ_HIP(h, launch_quantize_tiles(B, K, N, ldb, SRQ_AXIS_COL, p.s_b, p.lam_b, qmax, trunc,
                                     SRQ_LAYOUT_VECTOR_MAJOR, p.B_int, Kc,
                                     comp ? reinterpret_cast<uint32_t*>(p.s_rb) : nullptr, st));
    if (comp) SRQ_HIP(h, launch_scales(reinterpret_cast<uint32_t*>(p.s_rb), p.lam_rb, N, qmax, st));
  }
  if (comp) {
    im.s_ra = p.s_ra; im.s_rb = p.s_rb;
  }
  }

  // lines 2-3: D_int = A_int.B_int, D_F = dequant; line 7: partial sums of |D_F|
  GemmEpilogue ep;
  memset(&ep, 0, sizeof(ep));
  ep.mode = kGemmFirst;
  ep.s_row = p.s_a; ep.s_col = p.s_b; ep.C = C; ep.ldc = ldc;
  ep.alpha = alpha; ep.beta = beta; ep.Cin = Cin; ep.ldcin = ldcin;
  ep.ldd = N;
  if (dbg) { ep.D_int = dbg->D_int; ep.D_F_copy = dbg->D_F; }
  if (comp) { ep.row_part = p.row_part; ep.col_part = p.col_part; }
  ep.final_scale = !comp && scale_needed;
  {
    StageTimer tm(h, st, SRQ_STAGE_GEMM);
    SRQ_HIP(h, launch_gemm_i8(M, N, Kc, p.A_int, Kc, p.B_int, Kc, ep, st));
  }
  int path_a = 0, path_b = 0;
  bool decide_in_scan = false;                 // SRQ_STRATEGY_AUTO's decision and the statistics come from the scan kernel
  if (comp) {
    // line 9 and the branch of line 11 need the counts on the host in these modes
    // Only the density switch needs the counts on the host.  SRQ_STRATEGY_AUTO without it decides on
    // the device: a small kernel turns the counts into an execution per term, and every launch
    // that belongs to one outcome only checks that decision itself and does nothing otherwise.
    // (a limit <= 0 is reached by any density, including none kept: the dense branch needs no count)
    const bool always_dense = dense_fallback_density <= 0.f;
    const bool sync_mode = dense_fallback_density <= 1.f && !always_dense;
    const bool auto_dev = strategy == SRQ_STRATEGY_AUTO && !sync_mode && !always_dense;
    const RunIf a_on_mfma = {p.paths + 0, 1u << kPathMfma}, a_on_valu = {p.paths + 0, 1u << kPathValu};
    const RunIf b_on_mfma = {p.paths + 1, 1u << kPathMfma}, b_on_valu = {p.paths + 1, 1u << kPathValu};
    // the reduced operands in 2:4 form with the dense residual codes they are multiplied with
    // (term 2 is formed transposed: its sparse vectors are columns of C)
    const Sparse24Operand op24a = {p.a24v1, p.a24v2, p.a24n1, p.a24n2, p.a24f, p.RB_int, Kc, p.s_a, p.s_rb};
    const Sparse24Operand op24b = {p.b24v1, p.b24v2, p.b24n1, p.b24n2, p.b24f, p.RA_int, Kc, p.s_ra, p.s_b};
    {
    StageTimer tm(h, st, SRQ_STAGE_SELECT);
    // line 7: GetAvgVec, and the thresholds of Eq. avgQuan
    // (the persistent kernel leaves one partial per wave, two per 256-wide tile)
    int64_t parts_n, parts_m;
    gemm_sum_parts(M, N, Kc, p.A_int, Kc, p.B_int, Kc, ep, &parts_n, &parts_m);
    SRQ_HIP(h, launch_reduce_means_pair(p.row_part, parts_n, M, N, theta_a, p.drow, p.t_a, p.col_part, parts_m, N, M,
                                        theta_b, p.dcol, p.t_b, st));
    im.drow = p.drow; im.dcol = p.dcol; im.t_a = p.t_a; im.t_b = p.t_b;
    // lines 8-10: Reduce.  Keep-bits and per-vector counts, then the prefix scans
    int64_t chk = select_chunks(K);
    if (term_a) {
      // if term 2 is expected on the vector ALUs (fixed by the caller, or where SRQ_STRATEGY_AUTO
      // ended up in the previous call), A's selection pass also writes the k-major residual
      // codes that execution reads: one read of A less
      const int expect_b = strategy == SRQ_STRATEGY_AUTO ? h->last_path_b : strategy_path(strategy);
      const bool want_ra_em = term_b && dense_fallback_density > 1.f &&
                              path_reads_em(expect_b) &&
                              rows_mask_resid_em_ok(A, M, K, lda, p.s_a, p.lam_a, p.lam_ra, p.RA_em, M, p.t_a);
      if (want_ra_em) {
        SRQ_HIP(h, launch_rows_mask_resid_em(A, M, K, lda, qmax, trunc, p.s_a, p.lam_a, p.lam_ra, p.RA_em, M,
                                             p.t_a, p.mask_a, p.tot_a, st));
        ra_em_done = true;
      } else {
        SRQ_HIP(h, launch_rows_mask(A, M, K, lda, p.t_a, p.mask_a, p.tot_a, st));
      }
    }
    if (term_b) {
      if (fastB) {
        // (tot_b was cleared in the quantize stage)
        if (rb_in_select)
          SRQ_HIP(h, launch_cols_mask_resid(B, K, N, ldb, qmax, trunc, p.s_b, p.lam_b, p.ramax_b, p.s_rb, p.lam_rb,
                                            rb_want_vm ? p.RB_int : nullptr, Kc, rb_want_em ? p.RB_em : nullptr,
                                            N, p.t_b, p.mask_b, p.tot_b, st));
        else
          SRQ_HIP(h, launch_cols_mask(B, K, N, ldb, p.t_b, p.mask_b, p.tot_b, st));
      } else {
        SRQ_HIP(h, launch_select_count(B, K, N, ldb, SRQ_AXIS_COL, p.t_b, p.cnt_b, st));
        SRQ_HIP(h, launch_select_scan(p.cnt_b, N, chk, p.tot_b, p.b_ptr, p.nnz + 1, st));
      }
    }
    // line 9 and the branch of line 11: which execution each term takes.  SRQ_STRATEGY_AUTO: decided
    // on the device, by the scan kernel itself where it scans both operands (it then also writes
    // the statistics), else by a kernel of its own.
    // (for K > 8192 the K x 512-byte slab of codes an XCD gathers from outgrows its L2 and the
    // vector-ALU kernel loses earlier: measured crossover 0.62 % at 16384^3)
    const int64_t min_mfma_a =
        (int64_t)ceil((K > 8192 ? kAutoMfmaDensityALongK : kAutoMfmaDensityA) * (double)M * (double)K);
    const int64_t min_mfma_b =
        (int64_t)ceil((K > 8192 ? kAutoMfmaDensityBLongK : kAutoMfmaDensityB) * (double)N * (double)K);
    decide_in_scan = auto_dev && (!term_b || fastB);
    const ScanDecision dec = {p.paths, const_cast<int32_t*>(seen_paths(h)), min_mfma_a, min_mfma_b, stats_dev,
                              term_a ? p.cap_a : kNoCap, term_b ? p.cap_b : kNoCap};
    SRQ_HIP(h, launch_scan_pair(term_a ? p.tot_a : nullptr, M, p.a_ptr, p.nnz + 0,
                                (term_b && fastB) ? p.tot_b : nullptr, N, p.b_ptr, p.nnz + 1, st,
                                decide_in_scan ? &dec : nullptr));
    int64_t known_a = -1, known_b = -1;        // kept entries, once the host has read them
    if (auto_dev) {
      if (!decide_in_scan)
        SRQ_HIP(h, launch_decide_paths(p.nnz, term_a, term_b, min_mfma_a, min_mfma_b, p.paths,
                                       const_cast<int32_t*>(seen_paths(h)), st));
      if (term_a) path_a = kPathOnDevice;
      if (term_b) path_b = kPathOnDevice;
    } else if (sync_mode) {
      h->host_nnz[0] = h->host_nnz[1] = 0;
      SRQ_HIP(h, hipMemcpyAsync(h->host_nnz, p.nnz, 2 * sizeof(int64_t), hipMemcpyDeviceToHost, st));
      SRQ_HIP(h, hipStreamSynchronize(st));
      int64_t na = term_a ? h->host_nnz[0] : 0, nb = term_b ? h->host_nnz[1] : 0;
      double da = (double)na / ((double)M * (double)K), db = (double)nb / ((double)N * (double)K);
      known_a = na; known_b = nb;
      auto pick = [&](double d, double crossover) {
        if (d >= (double)dense_fallback_density) return 3;
        if (strategy == SRQ_STRATEGY_AUTO) return d >= crossover ? 2 : 1;
        return strategy_path(strategy);
      };
      // (for K > 8192 the K x 512-byte slab of codes an XCD gathers from outgrows its L2 and the
      // vector-ALU kernel loses earlier: measured crossover 0.62 % at 16384^3)
      if (term_a) path_a = pick(da, K > 8192 ? kAutoMfmaDensityALongK : kAutoMfmaDensityA);
      if (term_b) path_b = pick(db, K > 8192 ? kAutoMfmaDensityBLongK : kAutoMfmaDensityB);
      if (term_a && strategy == SRQ_STRATEGY_AUTO) h->last_path_a = path_a;
      if (term_b && strategy == SRQ_STRATEGY_AUTO) h->last_path_b = path_b;
      // an operand on the dense branch is not compacted, so only the others need room
      if ((path_a != 3 && na > p.cap_a) || (path_b != 3 && nb > p.cap_b)) {
        if (stats_dev)
          SRQ_HIP(h, launch_stats(term_a ? p.nnz : nullptr, term_b ? p.nnz + 1 : nullptr, 0, 0,
                                  path_a != 3 ? p.cap_a : kNoCap, path_b != 3 ? p.cap_b : kNoCap, stats_dev, st));
        return SRQ_STATUS_CAPACITY;
      }
    } else {
      if (term_a) path_a = always_dense ? kPathDense : strategy_path(strategy);
      if (term_b) path_b = always_dense ? kPathDense : strategy_path(strategy);
    }
    // the 2:4 kernel needs whole 256 x 256 tiles of C and cannot write the raw sums the debug
    // block asks for: such a term takes the plain matrix-core path
    // (B's 2:4 form is written from the keep-mask, which its generic, unaligned selection does not produce)
    if (path_a == kPath24 && (dbg || !scatter24_ok(M, Kc, p.A_int, Kc) || !gemm_sparse24_ok(M, N, Kc, op24a, false, ep)))
      path_a = kPathMfma;
    if (path_b == kPath24 &&
        (dbg || !fastB || !scatter24_ok(N, Kc, p.B_int, Kc) || !gemm_sparse24_ok(M, N, Kc, op24b, true, ep)))
      path_b = kPathMfma;
    // overflow flags of the 2:4 forms start at zero (one launch clears both)
    if (path_a == kPath24 || path_b == kPath24)
      SRQ_HIP(h, launch_fill3_u32(path_a == kPath24 ? p.a24f : nullptr, sparse24_flag_words(M, Kc),
                                  path_b == kPath24 ? p.b24f : nullptr, sparse24_flag_words(N, Kc), nullptr, 0, st));
    // the column-block split reads the keep-mask, which B's generic (unaligned) selection does not
    // produce: such a term runs as plain CSR on the vector ALUs
    if (path_b == kPathColblock && !fastB) path_b = kPathValu;
    if (path_a == kPathColblock)
      SRQ_HIP(h, launch_colblock_pick(p.mask_a, M, K, kColblockKeepRatio, p.kcnt, p.klist_a, p.kflag_a, p.nstrip, st));
    if (path_b == kPathColblock)
      SRQ_HIP(h, launch_colblock_pick(p.mask_b, N, K, kColblockKeepRatio, p.kcnt, p.klist_b, p.kflag_b, p.nstrip + 1,
                                      st));
    // compaction to CSR of A' / CSC of B'; a term that will run on the matrix cores also gets
    // its operand expanded to zero-filled dense codes in the same pass
    // (the dense branch multiplies the unreduced codes: its operand is counted, not compacted)
    if (term_a) {
      im.a_ptr = p.a_ptr; im.capacity_a = p.cap_a;
      if (path_a == kPath24) {
        // the compaction pass writes the 2:4 form of A' (P1, P2, flags) next to the CSR arrays
        SRQ_HIP(h, launch_scatter24(p.mask_a, M, K, Kc, p.A_int, Kc, p.a_ptr, p.a_idx, p.a_val, p.cap_a, p.a24v1,
                                    p.a24n1, p.a24v2, p.a24n2, p.a24f, st));
        im.a_idx = p.a_idx; im.a_val = p.a_val;
      } else if (path_a != 3) {
        SRQ_HIP(h, launch_scatter_mask(p.mask_a, M, K, p.A_int, Kc, p.a_ptr, p.a_idx, p.a_val, p.cap_a,
                                       (path_a == kPathMfma || auto_dev) ? p.Ad : nullptr, Kc, known_a, st,
                                       auto_dev ? a_on_mfma : kAlways));
        im.a_idx = p.a_idx; im.a_val = p.a_val;
      }
    }
    if (term_b && path_b == 3) {
      im.b_ptr = p.b_ptr; im.capacity_b = p.cap_b;
    } else if (term_b) {
      if (path_b == kPath24) {                          // (implies fastB)
        SRQ_HIP(h, launch_scatter24(p.mask_b, N, K, Kc, p.B_int, Kc, p.b_ptr, p.b_idx, p.b_val, p.cap_b, p.b24v1,
                                    p.b24n1, p.b24v2, p.b24n2, p.b24f, st));
      } else if (fastB) {
        SRQ_HIP(h, launch_scatter_mask(p.mask_b, N, K, p.B_int, Kc, p.b_ptr, p.b_idx, p.b_val, p.cap_b,
                                       (path_b == kPathMfma || auto_dev) ? p.Bd : nullptr, Kc, known_b, st,
                                       auto_dev ? b_on_mfma : kAlways));
      } else {
        SRQ_HIP(h, launch_select_scatter(B, K, N, ldb, SRQ_AXIS_COL, p.t_b, p.lam_b, qmax, trunc, p.b_ptr,
                                         p.cnt_b, p.b_idx, p.b_val, p.cap_b, st));
        if (path_b == kPathMfma || auto_dev)
          SRQ_HIP(h, launch_densify(p.b_ptr, p.b_idx, p.b_val, N, K, p.cap_b, p.Bd, Kc, st,
                                    auto_dev ? b_on_mfma : kAlways));
      }
      im.b_ptr = p.b_ptr; im.b_idx = p.b_idx; im.b_val = p.b_val; im.capacity_b = p.cap_b;
    }
    }
    // lines 4-6: residual matrices and their codes, in the layouts the chosen paths read
    // (RA feeds term 2, RB feeds term 1)
    bool ra_vm = path_reads_vm(path_b), ra_em = path_reads_em(path_b);
    bool rb_vm = path_reads_vm(path_a), rb_em = path_reads_em(path_a);
    if (auto_dev) {
      // which layout a term reads is only known on the device: a layout the earlier stages have not
      // written (they went by the hint) is written now, by a launch that does nothing unless the
      // decision asks for it.  Only what is certain to exist is exported as an intermediate.
      StageTimer tm(h, st, SRQ_STAGE_RESIDUAL);
      auto resid_a = [&](bool vm, RunIf run) -> hipError_t {
        if (!vm && rows_resid_em_ok(A, M, K, lda, p.s_a, p.lam_a, p.lam_ra, p.RA_em, M))
          return launch_rows_resid_em(A, M, K, lda, qmax, trunc, p.s_a, p.lam_a, p.lam_ra, p.RA_em, M, st, run);
        return launch_residual_tiles(A, M, K, lda, SRQ_AXIS_ROW, p.s_a, p.lam_a, p.lam_ra, qmax, trunc,
                                     vm ? p.RA_int : nullptr, Kc, vm ? nullptr : p.RA_em, M, st, run);
      };
      auto resid_b = [&](bool vm, RunIf run) -> hipError_t {
        if (fastB)
          return launch_cols_resid(B, K, N, ldb, qmax, trunc, p.s_b, p.lam_b, p.lam_rb, vm ? p.RB_int : nullptr, Kc,
                                   vm ? nullptr : p.RB_em, N, st, run);
        return launch_residual_tiles(B, K, N, ldb, SRQ_AXIS_COL, p.s_b, p.lam_b, p.lam_rb, qmax, trunc,
                                     vm ? p.RB_int : nullptr, Kc, vm ? nullptr : p.RB_em, N, st, run);
      };
      if (term_b && !ra_vm_done) SRQ_HIP(h, resid_a(true, b_on_mfma));
      if (term_b && !ra_em_done) SRQ_HIP(h, resid_a(false, b_on_valu));
      if (term_a && !rb_vm_done) SRQ_HIP(h, resid_b(true, a_on_mfma));
      if (term_a && !rb_em_done) SRQ_HIP(h, resid_b(false, a_on_valu));
      ra_vm = ra_vm_done; ra_em = ra_em_done; rb_vm = rb_vm_done; rb_em = rb_em_done;
    } else {
    StageTimer tm(h, st, SRQ_STAGE_RESIDUAL);
    // whatever the quantize stage has not already produced
    const bool need_ra_vm = ra_vm && !ra_vm_done, need_rb_vm = rb_vm && !rb_vm_done;
    const bool need_rb_em = rb_em && !rb_em_done, need_ra_em = ra_em && !ra_em_done;
    if (need_ra_em && !need_ra_vm && rows_resid_em_ok(A, M, K, lda, p.s_a, p.lam_a, p.lam_ra, p.RA_em, M))
      SRQ_HIP(h, launch_rows_resid_em(A, M, K, lda, qmax, trunc, p.s_a, p.lam_a, p.lam_ra, p.RA_em, M, st));
    else if (need_ra_vm || need_ra_em)
      SRQ_HIP(h, launch_residual_tiles(A, M, K, lda, SRQ_AXIS_ROW, p.s_a, p.lam_a, p.lam_ra, qmax, trunc,
                                       need_ra_vm ? p.RA_int : nullptr, Kc, need_ra_em ? p.RA_em : nullptr, M,
                                       st));
    if (need_rb_vm || need_rb_em) {
      if (fastB)
        SRQ_HIP(h, launch_cols_resid(B, K, N, ldb, qmax, trunc, p.s_b, p.lam_b, p.lam_rb,
                                     need_rb_vm ? p.RB_int : nullptr, Kc, need_rb_em ? p.RB_em : nullptr, N, st));
      else
        SRQ_HIP(h, launch_residual_tiles(B, K, N, ldb, SRQ_AXIS_COL, p.s_b, p.lam_b, p.lam_rb, qmax, trunc,
                                         need_rb_vm ? p.RB_int : nullptr, Kc, need_rb_em ? p.RB_em : nullptr, N,
                                         st));
    }
    }
    if (ra_vm) im.RA_int = p.RA_int;
    if (ra_em) im.RA_em = p.RA_em;
    if (rb_vm) im.RB_int = p.RB_int;
    if (rb_em) im.RB_em = p.RB_em;

    // lines 11-17: correction terms, accumulated into C in the order DR1 then DR2
    GemmEpilogue e1 = ep;
    e1.mode = kGemmAccum; e1.row_part = e1.col_part = nullptr; e1.D_F_copy = nullptr;
    e1.s_row = p.s_a; e1.s_col = p.s_rb;
    e1.D_int = dbg ? dbg->DR1_int : nullptr;
    e1.final_scale = scale_needed && path_b == 0;
    if (!sync_mode) {
      // the host has not seen the counts: every correction kernel checks them itself and leaves C
      // alone if an operand kept more entries than its compressed arrays hold
      e1.guard_nnz = p.nnz;
      e1.guard_cap_a = (path_a && path_a != kPathDense) ? p.cap_a : kNoCap;
      e1.guard_cap_b = (path_b && path_b != kPathDense) ? p.cap_b : kNoCap;
    }
    if (auto_dev) {
      // Every launch one of the four outcomes (vector ALUs / matrix cores per term) needs is
      // enqueued; each reads the decision and returns at once unless it is its turn:
      //   term t on the vector ALUs -> its sparse kernel
      //   term t on the matrix cores -> its product inside the paired launch, which runs one, the
      //   other or both of its products (where the shape allows no paired launch: a launch each)
      // The kernel of term 2 (or the pair) applies alpha / beta.
      const uint32_t kV = 1u << kPathValu, kM = 1u << kPathMfma, kAny = ~0u;
      GemmEpilogue e2 = e1;
      e2.s_row = p.s_ra; e2.s_col = p.s_b;
      e2.D_int = dbg ? dbg->DR2_int : nullptr;
      e2.final_scale = scale_needed;
      e1.final_scale = scale_needed && !term_b;
      e1.paths = e2.paths = p.paths;
      const GemmSecond sec = {p.RA_int, p.Bd, Kc, Kc, p.s_ra, p.s_b};
      const bool pair_ok = term_a && term_b && !dbg && gemm_pair_ok(M, N, Kc, p.Ad, Kc, p.RB_int, Kc, sec, e1);
      {
        StageTimer tm(h, st, SRQ_STAGE_TERM1);
        // (order of the additions to C: term 1, then term 2, whoever runs them)
        if (term_a) {
          GemmEpilogue ev = e1, em = e1;
          ev.ok_a = kV; ev.ok_b = kAny;
          SRQ_HIP(h, launch_spmm_valu(0, M, N, K, p.a_ptr, nullptr, p.a_idx, p.a_val, p.cap_a, p.RB_em, N, ev, st));
          em.ok_a = kM; em.ok_b = kAny;
          if (!pair_ok) SRQ_HIP(h, launch_gemm_i8(M, N, Kc, p.Ad, Kc, p.RB_int, Kc, em, st));
        }
        if (pair_ok) {
          GemmEpilogue e12 = e1;
          e12.final_scale = scale_needed;
          e12.ok_a = kM; e12.ok_b = kM; e12.each_product = 1;
          SRQ_HIP(h, launch_gemm_i8_pair(M, N, Kc, p.Ad, Kc, p.RB_int, Kc, sec, e12, st));
        }
      }
      if (term_b) {
        StageTimer tm(h, st, SRQ_STAGE_TERM2);
        GemmEpilogue ev = e2, em = e2;
        ev.ok_b = kV; ev.ok_a = kAny;
        SRQ_HIP(h, launch_spmm_valu(1, N, M, K, p.b_ptr, nullptr, p.b_idx, p.b_val, p.cap_b, p.RA_em, M, ev, st));
        em.ok_b = kM; em.ok_a = kAny;
        if (!pair_ok) SRQ_HIP(h, launch_gemm_i8(M, N, Kc, p.RA_int, Kc, p.Bd, Kc, em, st));
      }
      if (stats_dev && !decide_in_scan)
        SRQ_HIP(h, launch_stats(term_a ? p.nnz : nullptr, term_b ? p.nnz + 1 : nullptr, 0, 0, term_a ? p.cap_a : kNoCap,
                                term_b ? p.cap_b : kNoCap, stats_dev, st, p.paths));
      return SRQ_STATUS_OK;
    }
    // both terms on the dense matrix-core kernel: one launch, the two products of a tile back to
    // back (the tile of C is still cached when the second product adds to it)
    const int8_t* t1a = path_a == kPathMfma ? p.Ad : p.A_int;
    const int8_t* t2b = path_b == kPathMfma ? p.Bd : p.B_int;
    const GemmSecond sec12 = {p.RA_int, t2b, Kc, Kc, p.s_ra, p.s_b};
    const bool pair = (path_a == kPathMfma || path_a == kPathDense) && (path_b == kPathMfma || path_b == kPathDense) &&
                      !dbg && gemm_pair_ok(M, N, Kc, t1a, Kc, p.RB_int, Kc, sec12, e1);
    // both terms in 2:4 form: one launch as well, on the sparse matrix cores
    const bool pair24 = path_a == kPath24 && path_b == kPath24;
    if (pair) {
      StageTimer tm(h, st, SRQ_STAGE_TERM1);
      GemmEpilogue e12 = e1;
      e12.final_scale = scale_needed;
      SRQ_HIP(h, launch_gemm_i8_pair(M, N, Kc, t1a, Kc, p.RB_int, Kc, sec12, e12, st));
    } else if (pair24) {
      StageTimer tm(h, st, SRQ_STAGE_TERM1);
      GemmEpilogue e12 = e1;
      e12.final_scale = scale_needed;
      SRQ_HIP(h, launch_gemm_i8_sparse24(M, N, Kc, op24a, false, &op24b, e12, st));
    } else if (path_a == 1) {
      StageTimer tm(h, st, SRQ_STAGE_TERM1);
      SRQ_HIP(h, launch_spmm_valu(0, M, N, K, p.a_ptr, nullptr, p.a_idx, p.a_val, p.cap_a, p.RB_em, N, e1, st));
    } else if (path_a == 2) {
      StageTimer tm(h, st, SRQ_STAGE_TERM1);
      SRQ_HIP(h, launch_gemm_i8(M, N, Kc, p.Ad, Kc, p.RB_int, Kc, e1, st));
    } else if (path_a == 3) {
      StageTimer tm(h, st, SRQ_STAGE_TERM1);
      SRQ_HIP(h, launch_gemm_i8(M, N, Kc, p.A_int, Kc, p.RB_int, Kc, e1, st));
    } else if (path_a == kPathColblock) {
      // dense strip of the k kept almost everywhere on the matrix cores (one K-tile), then the
      // remainder of the CSR on the vector ALUs; with debug outputs the second adds its raw sums
      // to the first's
      {
        StageTimer tm(h, st, SRQ_STAGE_TERM1_PREP);
        SRQ_HIP(h, launch_strip_gather(p.A_int, Kc, p.mask_a, K, M, p.klist_a, p.strip_a, st));
        SRQ_HIP(h, launch_strip_gather(p.RB_int, Kc, nullptr, K, N, p.klist_a, p.strip_rb, st));
      }
      StageTimer tm(h, st, SRQ_STAGE_TERM1);
      GemmEpilogue es = e1;
      es.final_scale = 0;
      if (!dbg) es.run_if_nonzero = p.nstrip;
      SRQ_HIP(h, launch_gemm_i8(M, N, kStripK, p.strip_a, kStripK, p.strip_rb, kStripK, es, st));
      GemmEpilogue ev = e1;
      ev.dint_add = dbg ? 1 : 0;
      SRQ_HIP(h, launch_spmm_valu(0, M, N, K, p.a_ptr, nullptr, p.a_idx, p.a_val, p.cap_a, p.RB_em, N, ev, st,
                                  p.kflag_a));
    } else if (path_a == kPath24) {
      StageTimer tm(h, st, SRQ_STAGE_TERM1);
      SRQ_HIP(h, launch_gemm_i8_sparse24(M, N, Kc, op24a, false, nullptr, e1, st));
    }
    GemmEpilogue e2 = e1;
    e2.s_row = p.s_ra; e2.s_col = p.s_b;
    e2.D_int = dbg ? dbg->DR2_int : nullptr;
    e2.final_scale = scale_needed;
    if (pair || pair24) {
      // (term 2 went with term 1)
    } else if (path_b == 1) {
      StageTimer tm(h, st, SRQ_STAGE_TERM2);
      SRQ_HIP(h, launch_spmm_valu(1, N, M, K, p.b_ptr, nullptr, p.b_idx, p.b_val, p.cap_b, p.RA_em, M, e2, st));
    } else if (path_b == 2) {
      StageTimer tm(h, st, SRQ_STAGE_TERM2);
      SRQ_HIP(h, launch_gemm_i8(M, N, Kc, p.RA_int, Kc, p.Bd, Kc, e2, st));
    } else if (path_b == 3) {
      StageTimer tm(h, st, SRQ_STAGE_TERM2);
      SRQ_HIP(h, launch_gemm_i8(M, N, Kc, p.RA_int, Kc, p.B_int, Kc, e2, st));
    } else if (path_b == kPathColblock) {
      {
        StageTimer tm(h, st, SRQ_STAGE_TERM2_PREP);
        SRQ_HIP(h, launch_strip_gather(p.B_int, Kc, p.mask_b, K, N, p.klist_b, p.strip_b, st));
        SRQ_HIP(h, launch_strip_gather(p.RA_int, Kc, nullptr, K, M, p.klist_b, p.strip_ra, st));
      }
      StageTimer tm(h, st, SRQ_STAGE_TERM2);
      GemmEpilogue es = e2;
      es.final_scale = 0;
      if (!dbg) es.run_if_nonzero = p.nstrip + 1;
      SRQ_HIP(h, launch_gemm_i8(M, N, kStripK, p.strip_ra, kStripK, p.strip_b, kStripK, es, st));
      GemmEpilogue ev = e2;
      ev.dint_add = dbg ? 1 : 0;
      SRQ_HIP(h, launch_spmm_valu(1, N, M, K, p.b_ptr, nullptr, p.b_idx, p.b_val, p.cap_b, p.RA_em, M, ev, st,
                                  p.kflag_b));
    } else if (path_b == kPath24) {
      StageTimer tm(h, st, SRQ_STAGE_TERM2);
      SRQ_HIP(h, launch_gemm_i8_sparse24(M, N, Kc, op24b, true, nullptr, e2, st));
    }
    if (scale_needed && path_a == 0 && path_b == 0) {
      GemmEpilogue e3 = ep;
      SRQ_HIP(h, launch_scale_only(M, N, e3, st));
    }
  }
  if (stats_dev)
    SRQ_HIP(h, launch_stats(path_a ? p.nnz : nullptr, path_b ? p.nnz + 1 : nullptr, path_a, path_b,
                            (path_a && path_a != kPathDense) ? p.cap_a : kNoCap,
                            (path_b && path_b != kPathDense) ? p.cap_b : kNoCap, stats_dev, st));
  return SRQ_STATUS_OK;
}

}  // extern "C"
