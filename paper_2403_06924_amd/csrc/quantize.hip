// Vector-wise symmetric quantization and residual quantization (Algorithm 1 lines 1, 4-6;
// Eq. Quantization, Eq. getlambda, Sec. 3.2).  Streaming kernels bound by HBM bandwidth.
#include "srq_internal.h"

namespace srq {

namespace {

constexpr int kTile = 64;          // X is processed in 64 x 64 tiles by 256 threads

__device__ __forceinline__ int quant_code(float x, float lam, float qmax, int trunc) {
  float y = x * lam;
  float r = trunc ? truncf(y) : rintf(y);
  r = fminf(fmaxf(r, -qmax), qmax);
  return (int)r;
}

__global__ void fill_u32_kernel(uint32_t* p, int64_t n, uint32_t v) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = v;
}

// one 256-thread block per row
__global__ __launch_bounds__(256) void amax_rows_kernel(const float* __restrict__ X, int64_t cols,
                                                        int64_t ldx, uint32_t* __restrict__ amax_bits) {
  const float* row = X + (int64_t)blockIdx.x * ldx;
  float m = 0.f;
  for (int64_t c = threadIdx.x; c < cols; c += 256) m = fmaxf(m, fabsf(row[c]));
  for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
  __shared__ float sm[4];
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    m = fmaxf(fmaxf(sm[0], sm[1]), fmaxf(sm[2], sm[3]));
    amax_bits[blockIdx.x] = __float_as_uint(m);
  }
}

// thread per column, blockIdx.y selects a band of rows; max is order independent, so the
// integer atomic on the bit pattern of a non-negative float is deterministic
constexpr int kColBand = 128;
__global__ __launch_bounds__(256) void amax_cols_kernel(const float* __restrict__ X, int64_t rows,
                                                        int64_t cols, int64_t ldx,
                                                        uint32_t* __restrict__ amax_bits) {
  int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (c >= cols) return;
  int64_t r0 = (int64_t)blockIdx.y * kColBand;
  int64_t r1 = r0 + kColBand < rows ? r0 + kColBand : rows;
  float m = 0.f;
  for (int64_t r = r0; r < r1; ++r) m = fmaxf(m, fabsf(X[r * ldx + c]));
  atomicMax(&amax_bits[c], __float_as_uint(m));
}

// Matrix-wide scale (Eq. getlambda's a_max over the whole matrix): one block replaces every
// per-vector maximum by the maximum over all vectors.  The patterns are those of
// non-negative floats, which order like unsigned integers.
__global__ __launch_bounds__(1024) void broadcast_max_kernel(uint32_t* bits, int64_t n) {
  __shared__ uint32_t sm[16];
  uint32_t m = 0;
  for (int64_t i = threadIdx.x; i < n; i += 1024) m = bits[i] > m ? bits[i] : m;
  for (int off = 32; off > 0; off >>= 1) {
    uint32_t y = __shfl_xor(m, off, 64);
    m = y > m ? y : m;
  }
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = m;
  __syncthreads();
  m = 0;
  for (int i = 0; i < 16; ++i) m = sm[i] > m ? sm[i] : m;
  for (int64_t i = threadIdx.x; i < n; i += 1024) bits[i] = m;
}

__global__ void scales_kernel(uint32_t* amax_bits_then_scale, float* lambda, int64_t nvec, float qmax) {
  int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (v >= nvec) return;
  float amax = __uint_as_float(amax_bits_then_scale[v]);
  float s = 0.f, lam = 0.f;
  if (amax > 0.f) {
    lam = qmax / amax;
    s = amax / qmax;
  }
  reinterpret_cast<float*>(amax_bits_then_scale)[v] = s;
  if (lambda) lambda[v] = lam;
}

// Writes one 64 x 64 tile of codes held in LDS as t[r][c] to Q, straight (Q[r*ld + c]) or
// transposed (Q[c*ld + r]).
__device__ __forceinline__ void store_tile(const int8_t (*t)[kTile + 4], bool transposed, int8_t* Q,
                                           int64_t ld, int64_t r0, int64_t c0, int64_t rows,
                                           int64_t cols) {
  int tid = threadIdx.x;
  if (!transposed) {
    // 64 rows x 64 bytes; thread -> (row = tid/4, 16-byte segment = tid%4)
    int r = tid >> 2, seg = (tid & 3) * 16;
    if (r0 + r < rows) {
      int8_t* dst = Q + (r0 + r) * ld + c0 + seg;
      bool vec = (c0 + seg + 16 <= cols) && ((reinterpret_cast<uintptr_t>(dst) & 15) == 0);
      if (vec) {
        int4 v;
        int8_t* b = reinterpret_cast<int8_t*>(&v);
#pragma unroll
        for (int i = 0; i < 16; ++i) b[i] = t[r][seg + i];
        *reinterpret_cast<int4*>(dst) = v;
      } else {
        for (int i = 0; i < 16; ++i)
          if (c0 + seg + i < cols) dst[i] = t[r][seg + i];
      }
    }
  } else {
    int c = tid >> 2, seg = (tid & 3) * 16;
    if (c0 + c < cols) {
      int8_t* dst = Q + (c0 + c) * ld + r0 + seg;
      bool vec = (r0 + seg + 16 <= rows) && ((reinterpret_cast<uintptr_t>(dst) & 15) == 0);
      if (vec) {
        int4 v;
        int8_t* b = reinterpret_cast<int8_t*>(&v);
#pragma unroll
        for (int i = 0; i < 16; ++i) b[i] = t[seg + i][c];
        *reinterpret_cast<int4*>(dst) = v;
      } else {
        for (int i = 0; i < 16; ++i)
          if (r0 + seg + i < rows) dst[i] = t[seg + i][c];
      }
    }
  }
}

// AXIS 0: vectors are rows; AXIS 1: vectors are columns.
template <int AXIS>
__global__ __launch_bounds__(256) void quantize_tile_kernel(
    const float* __restrict__ X, int64_t rows, int64_t cols, int64_t ldx, const float* __restrict__ scale,
    const float* __restrict__ lambda, float qmax, int trunc, int transposed, int8_t* __restrict__ Q,
    int64_t ldq, uint32_t* __restrict__ ramax_bits) {
  __shared__ int8_t t[kTile][kTile + 4];
  __shared__ uint32_t rmax[kTile];
  int64_t r0 = (int64_t)blockIdx.y * kTile, c0 = (int64_t)blockIdx.x * kTile;
  int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  if (threadIdx.x < kTile) rmax[threadIdx.x] = 0;
  __syncthreads();
  int64_t c = c0 + tx;
  float lam_c = 0.f, s_c = 0.f;
  if (AXIS == 1 && c < cols) { lam_c = lambda[c]; s_c = scale[c]; }
  float rm_col = 0.f;
#pragma unroll 4
  for (int it = 0; it < 16; ++it) {
    int rl = ty * 16 + it;
    int64_t r = r0 + rl;
    int code = 0;
    float res = 0.f;
    if (r < rows && c < cols) {
      float lam = lam_c, s = s_c;
      if (AXIS == 0) { lam = lambda[r]; s = scale[r]; }
      float x = X[r * ldx + c];
      code = quant_code(x, lam, qmax, trunc);
      float xh = (float)code * s;
      res = fabsf(x - xh);
    }
    if (ramax_bits) {          // uniform over the block, so every lane takes part below
      if (AXIS == 1) {
        rm_col = fmaxf(rm_col, res);
      } else {
        // the 64 lanes of this wave share row r
        for (int off = 32; off > 0; off >>= 1) res = fmaxf(res, __shfl_xor(res, off, 64));
        if (tx == 0) rmax[rl] = __float_as_uint(res);
      }
    }
    t[rl][tx] = (int8_t)code;
  }
  if (ramax_bits && AXIS == 1) atomicMax(&rmax[tx], __float_as_uint(rm_col));
  __syncthreads();
  if (ramax_bits && threadIdx.x < kTile) {
    int64_t v = (AXIS == 0 ? r0 : c0) + threadIdx.x;
    int64_t nvec = AXIS == 0 ? rows : cols;
    if (v < nvec) atomicMax(&ramax_bits[v], rmax[threadIdx.x]);
  }
  if (Q) store_tile(t, transposed != 0, Q, ldq, r0, c0, rows, cols);
}

template <int AXIS>
__global__ __launch_bounds__(256) void residual_tile_kernel(
    const float* __restrict__ X, int64_t rows, int64_t cols, int64_t ldx, const float* __restrict__ scale,
    const float* __restrict__ lambda, const float* __restrict__ rlambda, float qmax, int trunc,
    int8_t* __restrict__ R_straight, int64_t ld_straight, int8_t* __restrict__ R_transposed,
    int64_t ld_transposed, RunIf run) {
  __shared__ int8_t t[kTile][kTile + 4];
  if (!run_if_ok(run)) return;
  int64_t r0 = (int64_t)blockIdx.y * kTile, c0 = (int64_t)blockIdx.x * kTile;
  int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  int64_t c = c0 + tx;
  float lam_c = 0.f, s_c = 0.f, rl_c = 0.f;
  if (AXIS == 1 && c < cols) { lam_c = lambda[c]; s_c = scale[c]; rl_c = rlambda[c]; }
#pragma unroll 4
  for (int it = 0; it < 16; ++it) {
    int rl = ty * 16 + it;
    int64_t r = r0 + rl;
    int rcode = 0;
    if (r < rows && c < cols) {
      float lam = lam_c, s = s_c, rlam = rl_c;
      if (AXIS == 0) { lam = lambda[r]; s = scale[r]; rlam = rlambda[r]; }
      float x = X[r * ldx + c];
      int code = quant_code(x, lam, qmax, trunc);
      float xh = (float)code * s;
      float res = x - xh;
      rcode = quant_code(res, rlam, qmax, trunc);
    }
    t[rl][tx] = (int8_t)rcode;
  }
  __syncthreads();
  if (R_straight) store_tile(t, false, R_straight, ld_straight, r0, c0, rows, cols);
  if (R_transposed) store_tile(t, true, R_transposed, ld_transposed, r0, c0, rows, cols);
}

inline dim3 tile_grid(int64_t rows, int64_t cols) {
  return dim3((unsigned)((cols + kTile - 1) / kTile), (unsigned)((rows + kTile - 1) / kTile));
}

}  // namespace

hipError_t launch_fill_u32(uint32_t* p, int64_t n, uint32_t v, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  int64_t blocks = (n + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)blocks), dim3(256), 0, st, p, n, v);
  return hipGetLastError();
}

hipError_t launch_amax(const float* X, int64_t rows, int64_t cols, int64_t ldx, int axis,
                       uint32_t* amax_bits, hipStream_t st) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  if (axis == SRQ_AXIS_ROW) {
    hipLaunchKernelGGL(amax_rows_kernel, dim3((unsigned)rows), dim3(256), 0, st, X, cols, ldx, amax_bits);
  } else {
    dim3 grid((unsigned)((cols + 255) / 256), (unsigned)((rows + kColBand - 1) / kColBand));
    hipLaunchKernelGGL(amax_cols_kernel, grid, dim3(256), 0, st, X, rows, cols, ldx, amax_bits);
  }
  return hipGetLastError();
}

hipError_t launch_scales(uint32_t* amax_bits_then_scale, float* lambda, int64_t nvec, int qmax,
                         hipStream_t st) {
  if (nvec <= 0) return hipSuccess;
  hipLaunchKernelGGL(scales_kernel, dim3((unsigned)((nvec + 255) / 256)), dim3(256), 0, st,
                     amax_bits_then_scale, lambda, nvec, (float)qmax);
  return hipGetLastError();
}

__global__ void fill3_u32_kernel(uint32_t* a, int64_t na, uint32_t* b, int64_t nb, uint32_t* c, int64_t nc) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < na) a[i] = 0;
  if (i < nb) b[i] = 0;
  if (i < nc) c[i] = 0;
}

struct PadArgs { int8_t* m[6]; int64_t rows[6]; };

// one thread per (matrix, row, padding byte)
__global__ void zero_pad_kernel(PadArgs a, int n, int64_t cols, int64_t ld) {
  const int64_t pad = ld - cols;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int which = blockIdx.y;
  if (which >= n || !a.m[which]) return;
  const int64_t r = i / pad, c = i - r * pad;
  if (r < a.rows[which]) a.m[which][r * ld + cols + c] = 0;
}

hipError_t launch_zero_pad(int8_t* const* mats, const int64_t* rows, int n, int64_t cols, int64_t ld,
                           hipStream_t st) {
  if (ld <= cols || n <= 0) return hipSuccess;
  PadArgs a;
  int64_t most = 0;
  for (int i = 0; i < 6; ++i) {
    a.m[i] = i < n ? mats[i] : nullptr;
    a.rows[i] = i < n ? rows[i] : 0;
    if (a.m[i] && a.rows[i] > most) most = a.rows[i];
  }
  if (most <= 0) return hipSuccess;
  const int64_t work = most * (ld - cols);
  hipLaunchKernelGGL(zero_pad_kernel, dim3((unsigned)((work + 255) / 256), (unsigned)n), dim3(256), 0, st, a, n,
                     cols, ld);
  return hipGetLastError();
}

hipError_t launch_fill3_u32(uint32_t* a, int64_t na, uint32_t* b, int64_t nb, uint32_t* c, int64_t nc,
                            hipStream_t st) {
  if (!a) na = 0;
  if (!b) nb = 0;
  if (!c) nc = 0;
  int64_t n = na > nb ? na : nb;
  n = n > nc ? n : nc;
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(fill3_u32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, a, na, b, nb, c, nc);
  return hipGetLastError();
}

hipError_t launch_broadcast_max(uint32_t* bits, int64_t n, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(broadcast_max_kernel, dim3(1), dim3(1024), 0, st, bits, n);
  return hipGetLastError();
}

hipError_t launch_quantize_tiles(const float* X, int64_t rows, int64_t cols, int64_t ldx, int axis,
                                 const float* scale, const float* lambda, int qmax, int trunc,
                                 int layout, int8_t* Q, int64_t ldq, uint32_t* ramax_bits,
                                 hipStream_t st) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  // the output is "straight" (same orientation as X) when vectors are rows and the layout
  // is vector-major, or vectors are columns and the layout is element-major
  int transposed = (axis == SRQ_AXIS_ROW) != (layout == SRQ_LAYOUT_VECTOR_MAJOR);
  dim3 grid = tile_grid(rows, cols);
  if (axis == SRQ_AXIS_ROW)
    hipLaunchKernelGGL(quantize_tile_kernel<0>, grid, dim3(256), 0, st, X, rows, cols, ldx, scale, lambda,
                       (float)qmax, trunc, transposed, Q, ldq, ramax_bits);
  else
    hipLaunchKernelGGL(quantize_tile_kernel<1>, grid, dim3(256), 0, st, X, rows, cols, ldx, scale, lambda,
                       (float)qmax, trunc, transposed, Q, ldq, ramax_bits);
  return hipGetLastError();
}

hipError_t launch_residual_tiles(const float* X, int64_t rows, int64_t cols, int64_t ldx, int axis,
                                 const float* scale, const float* lambda, const float* rlambda,
                                 int qmax, int trunc, int8_t* R_vm, int64_t ld_vm, int8_t* R_em,
                                 int64_t ld_em, hipStream_t st, RunIf run) {
  if (rows <= 0 || cols <= 0 || (!R_vm && !R_em)) return hipSuccess;
  dim3 grid = tile_grid(rows, cols);
  if (axis == SRQ_AXIS_ROW)   // vector-major is straight, element-major is transposed
    hipLaunchKernelGGL(residual_tile_kernel<0>, grid, dim3(256), 0, st, X, rows, cols, ldx, scale, lambda,
                       rlambda, (float)qmax, trunc, R_vm, ld_vm, R_em, ld_em, run);
  else                        // element-major is straight, vector-major is transposed
    hipLaunchKernelGGL(residual_tile_kernel<1>, grid, dim3(256), 0, st, X, rows, cols, ldx, scale, lambda,
                       rlambda, (float)qmax, trunc, R_em, ld_em, R_vm, ld_vm, run);
  return hipGetLastError();
}

}  // namespace srq
