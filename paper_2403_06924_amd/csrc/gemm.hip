// INT8 x INT8 -> INT32 GEMM on the gfx950 matrix cores with the FP32 dequantization epilogue
// (Algorithm 1 lines 2-3 and, in accumulate mode, lines 12/14 with 16-17).
//
//   D_int[i,j] = sum_k Qa[i*lda + k] * Qb[j*ldb + k]       both operands K-contiguous
//   first mode : C = fl(float(D_int) * fl(s_row[i]*s_col[j])), plus per-tile partial sums
//                of |C| over rows and columns for the averages of Sec. 3.1.1
//   accum mode : C += the same dequantized product
#include "srq_internal.h"

namespace srq {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int LDS_STRIDE = BK + 16;   // bytes per tile row in LDS (16-byte aligned, skewed)

// 16 bytes of row `row` starting at byte k, zero where outside [0,K) or row >= nrows
template <bool ALIGNED>
__device__ __forceinline__ v4i load16(const int8_t* __restrict__ base, int64_t ld, int64_t row,
                                      int64_t nrows, int64_t k, int64_t K) {
  v4i out = {0, 0, 0, 0};
  if (row >= nrows || k >= K) return out;
  const int8_t* p = base + row * ld + k;
  if (ALIGNED && k + 16 <= K) return *reinterpret_cast<const v4i*>(p);
  int8_t* b = reinterpret_cast<int8_t*>(&out);
  for (int i = 0; i < 16; ++i)
    if (k + i < K) b[i] = p[i];
  return out;
}

template <bool ALIGNED>
__global__ __launch_bounds__(256) void gemm_i8_kernel(int64_t M, int64_t N, int64_t K,
                                                      const int8_t* __restrict__ Qa, int64_t lda,
                                                      const int8_t* __restrict__ Qb, int64_t ldb,
                                                      GemmEpilogue ep) {
  __shared__ __attribute__((aligned(16))) int8_t As[BM * LDS_STRIDE];
  __shared__ __attribute__((aligned(16))) int8_t Bs[BN * LDS_STRIDE];
  __shared__ double red[2][128];

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int wm = w >> 1, wn = w & 1;
  const int64_t tile_m = blockIdx.y, tile_n = blockIdx.x;
  const int64_t m0 = tile_m * BM, n0 = tile_n * BN;

  v16i acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0;

  // global -> register staging: two 16-byte pieces of each operand tile per thread
  const int lrow0 = tid >> 2, lseg = (tid & 3) * 16;
  v4i ra[2], rb[2];
  auto gload = [&](int64_t k0) {
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      int r = lrow0 + s * 64;
      ra[s] = load16<ALIGNED>(Qa, lda, m0 + r, M, k0 + lseg, K);
      rb[s] = load16<ALIGNED>(Qb, ldb, n0 + r, N, k0 + lseg, K);
    }
  };
  const int64_t nk = (K + BK - 1) / BK;
  if (nk > 0) gload(0);
  const int frow = lane & 31, fk = (lane >> 5) * 16;
  for (int64_t kt = 0; kt < nk; ++kt) {
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      int r = lrow0 + s * 64;
      *reinterpret_cast<v4i*>(&As[r * LDS_STRIDE + lseg]) = ra[s];
      *reinterpret_cast<v4i*>(&Bs[r * LDS_STRIDE + lseg]) = rb[s];
    }
    __syncthreads();
    if (kt + 1 < nk) gload((kt + 1) * BK);
#pragma unroll
    for (int kk = 0; kk < BK / 32; ++kk) {
      v4i fa[2], fb[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        fa[t] = *reinterpret_cast<const v4i*>(&As[(wm * 64 + t * 32 + frow) * LDS_STRIDE + kk * 32 + fk]);
        fb[t] = *reinterpret_cast<const v4i*>(&Bs[(wn * 64 + t * 32 + frow) * LDS_STRIDE + kk * 32 + fk]);
      }
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[a], fb[b], acc[a][b], 0, 0, 0);
    }
    __syncthreads();
  }

  // ---- epilogue.  acc[a][b][v] is element (row, col) of the wave's 64 x 64 block with
  //      row = a*32 + 8*(v/4) + 4*(lane/32) + v%4,  col = b*32 + lane%32
  const bool first = ep.mode == kGemmFirst;
  const bool sums = first && ep.row_part != nullptr;
  const int half = lane >> 5, cl = lane & 31;
  double colsum[2] = {0.0, 0.0};
  float scol[2];
  int64_t gcol[2];
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    gcol[b] = n0 + wn * 64 + b * 32 + cl;
    scol[b] = gcol[b] < N ? ep.s_col[gcol[b]] : 0.f;
  }
#pragma unroll
  for (int a = 0; a < 2; ++a) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      int rl = wm * 64 + a * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
      int64_t gi = m0 + rl;
      float srow = gi < M ? ep.s_row[gi] : 0.f;
      double rsum = 0.0;
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        if (gi < M && gcol[b] < N) {
          int iv = acc[a][b][v];
          float d = (float)iv * (srow * scol[b]);
          if (ep.D_int) ep.D_int[gi * ep.ldd + gcol[b]] = iv;
          float out;
          if (first) {
            out = d;
            if (ep.D_F_copy) ep.D_F_copy[gi * ep.ldd + gcol[b]] = d;
            double ad = (double)fabsf(d);
            rsum += ad;
            colsum[b] += ad;
          } else {
            out = ep.C[gi * ep.ldc + gcol[b]] + d;
          }
          if (ep.final_scale) {
            out = ep.alpha * out;
            if (ep.beta != 0.f) out = out + ep.beta * ep.Cin[gi * ep.ldcin + gcol[b]];
          }
          ep.C[gi * ep.ldc + gcol[b]] = out;
        }
      }
      if (sums) {
        // sum over the 32 lanes holding this row (fixed tree), then over the two waves
        for (int off = 16; off > 0; off >>= 1) rsum += __shfl_xor(rsum, off, 64);
        if (cl == 0) red[wn][rl] = rsum;
      }
    }
  }
  if (sums) {
    __syncthreads();
    if (tid < BM && m0 + tid < M)
      ep.row_part[tile_n * M + m0 + tid] = red[0][tid] + red[1][tid];
    __syncthreads();
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      double c = colsum[b];
      c += __shfl_xor(c, 32, 64);                 // the two half-waves hold different rows
      if (half == 0) red[wm][wn * 64 + b * 32 + cl] = c;
    }
    __syncthreads();
    if (tid < BN && n0 + tid < N)
      ep.col_part[tile_m * N + n0 + tid] = red[0][tid] + red[1][tid];
  }
}

// C = alpha*C + beta*Cin when no product term carries the final scaling
__global__ void scale_only_kernel(int64_t M, int64_t N, GemmEpilogue ep) {
  int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= N) return;
  for (int64_t i = blockIdx.y; i < M; i += gridDim.y) {
    float out = ep.alpha * ep.C[i * ep.ldc + j];
    if (ep.beta != 0.f) out = out + ep.beta * ep.Cin[i * ep.ldcin + j];
    ep.C[i * ep.ldc + j] = out;
  }
}

}  // namespace

int gemm_tile_m() { return BM; }
int gemm_tile_n() { return BN; }

hipError_t launch_gemm_i8(int64_t M, int64_t N, int64_t K, const int8_t* Qa, int64_t lda,
                          const int8_t* Qb, int64_t ldb, const GemmEpilogue& ep, hipStream_t st) {
  if (M <= 0 || N <= 0) return hipSuccess;
  dim3 grid((unsigned)((N + BN - 1) / BN), (unsigned)((M + BM - 1) / BM));
  bool aligned = ((reinterpret_cast<uintptr_t>(Qa) | reinterpret_cast<uintptr_t>(Qb)) & 15) == 0 &&
                 (lda % 16) == 0 && (ldb % 16) == 0;
  if (aligned)
    hipLaunchKernelGGL(gemm_i8_kernel<true>, grid, dim3(256), 0, st, M, N, K, Qa, lda, Qb, ldb, ep);
  else
    hipLaunchKernelGGL(gemm_i8_kernel<false>, grid, dim3(256), 0, st, M, N, K, Qa, lda, Qb, ldb, ep);
  return hipGetLastError();
}

hipError_t launch_scale_only(int64_t M, int64_t N, const GemmEpilogue& ep, hipStream_t st) {
  if (M <= 0 || N <= 0) return hipSuccess;
  dim3 grid((unsigned)((N + 255) / 256), (unsigned)(M < 32768 ? M : 32768));
  hipLaunchKernelGGL(scale_only_kernel, grid, dim3(256), 0, st, M, N, ep);
  return hipGetLastError();
}

}  // namespace srq
