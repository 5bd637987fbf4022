// Reduction of the operands to sparse matrices (Algorithm 1 lines 7-10; Eq. avgQuan):
// thresholds from the means of |D_F|, threshold-select, and stream compaction to CSR / CSC
// by count -> exclusive prefix scan -> scatter.  All integer work is deterministic.
#include "srq_internal.h"

namespace srq {
namespace {

__device__ __forceinline__ int quant_code(float x, float lam, float qmax, int trunc) {
  float y = x * lam;
  float r = trunc ? truncf(y) : rintf(y);
  r = fminf(fmaxf(r, -qmax), qmax);
  return (int)r;
}

// mean_v = (sum over partial sums, fixed order) / count, rounded once to float;
// thresh_v = fl(theta * mean_v)
// both mean vectors of one product in a single launch: vectors [0, n0) are rows, the rest columns
__global__ void reduce_means_pair_kernel(const double* __restrict__ part0, int64_t nparts0, int64_t n0,
                                         double count0, float theta0, float* __restrict__ mean0,
                                         float* __restrict__ thresh0, const double* __restrict__ part1,
                                         int64_t nparts1, int64_t n1, double count1, float theta1,
                                         float* __restrict__ mean1, float* __restrict__ thresh1) {
  int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (v >= n0 + n1) return;
  const bool second = v >= n0;
  if (second) v -= n0;
  const double* part = second ? part1 : part0;
  const int64_t nparts = second ? nparts1 : nparts0, nvec = second ? n1 : n0;
  double s = 0.0;
#pragma unroll 8
  for (int64_t p = 0; p < nparts; ++p) s += part[p * nvec + v];   // fixed order: reproducible means
  float m = (float)(s / (second ? count1 : count0));
  (second ? mean1 : mean0)[v] = m;
  float* thresh = second ? thresh1 : thresh0;       // (null: the means alone are wanted)
  if (thresh) thresh[v] = (second ? theta1 : theta0) * m;
}

// ---- vectors are rows: one wave per (row, chunk of kSelChunk consecutive elements) ----
template <bool SCATTER>
__global__ __launch_bounds__(256) void select_rows_kernel(
    const float* __restrict__ X, int64_t rows, int64_t cols, int64_t ldx, const float* __restrict__ thresh,
    const float* __restrict__ lambda, float qmax, int trunc, int64_t nchunks, int32_t* __restrict__ cnt,
    const int32_t* __restrict__ ptr, const int32_t* __restrict__ off, int32_t* __restrict__ idx,
    int8_t* __restrict__ val, int64_t capacity) {
  int lane = threadIdx.x & 63;
  int64_t g = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  int64_t v = g / nchunks, ch = g - v * nchunks;
  if (v >= rows) return;
  float t = thresh[v];
  float lam = SCATTER ? lambda[v] : 0.f;
  const float* row = X + v * ldx;
  int64_t base = 0;
  if (SCATTER) base = (int64_t)ptr[v] + off[ch * rows + v];
  int total = 0;
  int64_t e0 = ch * kSelChunk;
#pragma unroll
  for (int it = 0; it < kSelChunk / 64; ++it) {
    int64_t e = e0 + it * 64 + lane;
    float x = 0.f;
    bool keep = false;
    if (e < cols) {
      x = row[e];
      keep = fabsf(x) > t;
    }
    unsigned long long m = __ballot(keep);
    if (SCATTER) {
      if (keep) {
        int64_t pos = base + total + __popcll(m & ((1ull << lane) - 1ull));
        if (pos < capacity) {
          idx[pos] = (int32_t)e;
          val[pos] = (int8_t)quant_code(x, lam, qmax, trunc);
        }
      }
    }
    total += __popcll(m);
  }
  if (!SCATTER && lane == 0) cnt[ch * rows + v] = total;
}

// ---- vectors are columns: lane = column, one wave per (64 columns, chunk of rows) ----
template <bool SCATTER>
__global__ __launch_bounds__(256) void select_cols_kernel(
    const float* __restrict__ X, int64_t rows, int64_t cols, int64_t ldx, const float* __restrict__ thresh,
    const float* __restrict__ lambda, float qmax, int trunc, int64_t nchunks, int32_t* __restrict__ cnt,
    const int32_t* __restrict__ ptr, const int32_t* __restrict__ off, int32_t* __restrict__ idx,
    int8_t* __restrict__ val, int64_t capacity) {
  int lane = threadIdx.x & 63;
  int64_t ch = (int64_t)blockIdx.y * 4 + (threadIdx.x >> 6);
  int64_t v = (int64_t)blockIdx.x * 64 + lane;
  if (ch >= nchunks || v >= cols) return;
  float t = thresh[v];
  float lam = SCATTER ? lambda[v] : 0.f;
  int64_t pos = 0;
  if (SCATTER) pos = (int64_t)ptr[v] + off[ch * cols + v];
  int64_t r0 = ch * kSelChunk;
  int64_t r1 = r0 + kSelChunk < rows ? r0 + kSelChunk : rows;
  int total = 0;
#pragma unroll 8
  for (int64_t r = r0; r < r1; ++r) {
    float x = X[r * ldx + v];
    if (fabsf(x) > t) {
      if (SCATTER) {
        if (pos < capacity) {
          idx[pos] = (int32_t)r;
          val[pos] = (int8_t)quant_code(x, lam, qmax, trunc);
        }
        ++pos;
      }
      ++total;
    }
  }
  if (!SCATTER) cnt[ch * cols + v] = total;
}

// counts[chunk][vec] -> exclusive offsets within the vector (in place) and totals[vec]
__global__ void chunk_offsets_kernel(int32_t* __restrict__ cnt_then_off, int64_t nvec, int64_t nchunks,
                                     int32_t* __restrict__ totals) {
  int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (v >= nvec) return;
  int32_t run = 0;
  for (int64_t c = 0; c < nchunks; ++c) {
    int32_t n = cnt_then_off[c * nvec + v];
    cnt_then_off[c * nvec + v] = run;
    run += n;
  }
  totals[v] = run;
}

// exclusive prefix scan of totals[nvec] into ptr[nvec+1], one 1024-thread block
__global__ __launch_bounds__(1024) void scan_totals_kernel(const int32_t* __restrict__ totals, int64_t nvec,
                                                           int32_t* __restrict__ ptr,
                                                           int64_t* __restrict__ nnz_dev) {
  __shared__ int64_t wave_sum[16];
  __shared__ int64_t carry_s;
  int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  if (tid == 0) carry_s = 0;
  __syncthreads();
  for (int64_t base = 0; base < nvec; base += 1024) {
    int64_t v = base + tid;
    int64_t x = v < nvec ? totals[v] : 0;
    int64_t inc = x;                                   // inclusive scan within the wave
    for (int d = 1; d < 64; d <<= 1) {
      int64_t y = __shfl_up(inc, d, 64);
      if (lane >= d) inc += y;
    }
    if (lane == 63) wave_sum[w] = inc;
    __syncthreads();
    int64_t wave_off = 0;
    for (int i = 0; i < w; ++i) wave_off += wave_sum[i];
    int64_t carry = carry_s;
    if (v < nvec) ptr[v] = (int32_t)(carry + wave_off + inc - x);
    __syncthreads();
    if (tid == 1023) carry_s = carry + wave_off + inc;
    __syncthreads();
  }
  if (tid == 0) {
    ptr[nvec] = (int32_t)carry_s;
    if (nnz_dev) *nnz_dev = carry_s;
  }
}

// one block per vector: zero the dense vector, then drop the kept codes in
__global__ __launch_bounds__(256) void densify_kernel(const int32_t* __restrict__ ptr,
                                                      const int32_t* __restrict__ idx,
                                                      const int8_t* __restrict__ val, int64_t veclen,
                                                      int64_t capacity, int8_t* __restrict__ dense,
                                                      int64_t ld, RunIf run) {
  if (!run_if_ok(run)) return;
  int64_t v = blockIdx.x;
  int8_t* row = dense + v * ld;
  if ((reinterpret_cast<uintptr_t>(row) & 15) == 0) {
    int64_t n16 = veclen / 16;
    int4 z = make_int4(0, 0, 0, 0);
    for (int64_t i = threadIdx.x; i < n16; i += 256) reinterpret_cast<int4*>(row)[i] = z;
    for (int64_t i = n16 * 16 + threadIdx.x; i < veclen; i += 256) row[i] = 0;
  } else {
    for (int64_t i = threadIdx.x; i < veclen; i += 256) row[i] = 0;
  }
  __syncthreads();
  int64_t p0 = ptr[v], p1 = ptr[v + 1];
  if (p1 > capacity) p1 = capacity;
  for (int64_t p = p0 + threadIdx.x; p < p1; p += 256) row[idx[p]] = val[p];
}

// seen (optional): host-visible words that receive the decision of each term that exists, for
// the host to read whenever it next cares to
__global__ void decide_paths_kernel(const int64_t* nnz, int term_a, int term_b, int64_t min_a, int64_t min_b,
                                    int32_t* paths, int32_t* seen) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    const int pa = term_a ? (nnz[0] >= min_a ? 2 : 1) : 0;
    const int pb = term_b ? (nnz[1] >= min_b ? 2 : 1) : 0;
    paths[0] = pa;
    paths[1] = pb;
    if (seen && pa) seen[0] = pa;
    if (seen && pb) seen[1] = pb;
  }
}

__global__ void stats_kernel(const int64_t* nnz_a, const int64_t* nnz_b, int path_a, int path_b, int64_t cap_a,
                             int64_t cap_b, srq_stats_t* out, const int32_t* paths_dev) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    if (paths_dev) { path_a = paths_dev[0]; path_b = paths_dev[1]; }
    const int64_t na = nnz_a ? *nnz_a : 0, nb = nnz_b ? *nnz_b : 0;
    out->nnz_a = na;
    out->nnz_b = nb;
    out->path_a = path_a;
    out->path_b = path_b;
    out->overflow = (na > cap_a ? 1 : 0) | (nb > cap_b ? 2 : 0);
    out->reserved = 0;
  }
}

}  // namespace

hipError_t launch_reduce_means_pair(const double* part0, int64_t nparts0, int64_t n0, int64_t count0, float theta0,
                                    float* mean0, float* thresh0, const double* part1, int64_t nparts1,
                                    int64_t n1, int64_t count1, float theta1, float* mean1, float* thresh1,
                                    hipStream_t st) {
  if (n0 + n1 <= 0) return hipSuccess;
  hipLaunchKernelGGL(reduce_means_pair_kernel, dim3((unsigned)((n0 + n1 + 255) / 256)), dim3(256), 0, st, part0,
                     nparts0, n0, (double)count0, theta0, mean0, thresh0, part1, nparts1, n1, (double)count1,
                     theta1, mean1, thresh1);
  return hipGetLastError();
}

hipError_t launch_select_count(const float* X, int64_t rows, int64_t cols, int64_t ldx, int axis,
                               const float* thresh, int32_t* cnt, hipStream_t st) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  if (axis == SRQ_AXIS_ROW) {
    int64_t nch = select_chunks(cols);
    int64_t waves = rows * nch;
    hipLaunchKernelGGL(select_rows_kernel<false>, dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, st, X,
                       rows, cols, ldx, thresh, nullptr, 0.f, 0, nch, cnt, nullptr, nullptr, nullptr,
                       nullptr, 0);
  } else {
    int64_t nch = select_chunks(rows);
    dim3 grid((unsigned)((cols + 63) / 64), (unsigned)((nch + 3) / 4));
    hipLaunchKernelGGL(select_cols_kernel<false>, grid, dim3(256), 0, st, X, rows, cols, ldx, thresh,
                       nullptr, 0.f, 0, nch, cnt, nullptr, nullptr, nullptr, nullptr, 0);
  }
  return hipGetLastError();
}

hipError_t launch_select_scan(int32_t* cnt_then_off, int64_t nvec, int64_t nchunks, int32_t* totals,
                              int32_t* ptr, int64_t* nnz_dev, hipStream_t st) {
  if (nvec > 0 && nchunks > 0)
    hipLaunchKernelGGL(chunk_offsets_kernel, dim3((unsigned)((nvec + 255) / 256)), dim3(256), 0, st,
                       cnt_then_off, nvec, nchunks, totals);
  else if (nvec > 0) {
    hipError_t e = launch_fill_u32(reinterpret_cast<uint32_t*>(totals), nvec, 0, st);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(scan_totals_kernel, dim3(1), dim3(1024), 0, st, totals, nvec, ptr, nnz_dev);
  return hipGetLastError();
}

hipError_t launch_scan_totals(const int32_t* totals, int64_t nvec, int32_t* ptr, int64_t* nnz_dev,
                              hipStream_t st) {
  hipLaunchKernelGGL(scan_totals_kernel, dim3(1), dim3(1024), 0, st, totals, nvec, ptr, nnz_dev);
  return hipGetLastError();
}

hipError_t launch_select_scatter(const float* X, int64_t rows, int64_t cols, int64_t ldx, int axis,
                                 const float* thresh, const float* lambda, int qmax, int trunc,
                                 const int32_t* ptr, const int32_t* off, int32_t* idx, int8_t* val,
                                 int64_t capacity, hipStream_t st) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  if (axis == SRQ_AXIS_ROW) {
    int64_t nch = select_chunks(cols);
    int64_t waves = rows * nch;
    hipLaunchKernelGGL(select_rows_kernel<true>, dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, st, X,
                       rows, cols, ldx, thresh, lambda, (float)qmax, trunc, nch, nullptr, ptr, off, idx,
                       val, capacity);
  } else {
    int64_t nch = select_chunks(rows);
    dim3 grid((unsigned)((cols + 63) / 64), (unsigned)((nch + 3) / 4));
    hipLaunchKernelGGL(select_cols_kernel<true>, grid, dim3(256), 0, st, X, rows, cols, ldx, thresh,
                       lambda, (float)qmax, trunc, nch, nullptr, ptr, off, idx, val, capacity);
  }
  return hipGetLastError();
}

hipError_t launch_densify(const int32_t* ptr, const int32_t* idx, const int8_t* val, int64_t nvec,
                          int64_t veclen, int64_t capacity, int8_t* dense, int64_t ld, hipStream_t st, RunIf run) {
  if (nvec <= 0 || veclen <= 0) return hipSuccess;
  hipLaunchKernelGGL(densify_kernel, dim3((unsigned)nvec), dim3(256), 0, st, ptr, idx, val, veclen,
                     capacity, dense, ld, run);
  return hipGetLastError();
}

hipError_t launch_decide_paths(const int64_t* nnz, int term_a, int term_b, int64_t min_mfma_a, int64_t min_mfma_b,
                               int32_t* paths, int32_t* seen, hipStream_t st) {
  hipLaunchKernelGGL(decide_paths_kernel, dim3(1), dim3(64), 0, st, nnz, term_a, term_b, min_mfma_a, min_mfma_b,
                     paths, seen);
  return hipGetLastError();
}

hipError_t launch_stats(const int64_t* nnz_a, const int64_t* nnz_b, int path_a, int path_b, int64_t cap_a,
                        int64_t cap_b, srq_stats_t* out, hipStream_t st, const int32_t* paths_dev) {
  hipLaunchKernelGGL(stats_kernel, dim3(1), dim3(64), 0, st, nnz_a, nnz_b, path_a, path_b, cap_a, cap_b, out,
                     paths_dev);
  return hipGetLastError();
}

}  // namespace srq
