// Sparse x dense correction products on the vector ALUs (Algorithm 1 line 12, SPMM), with
// the dequantize-and-accumulate epilogue of lines 16-17 fused in.
//
//   out[v, e] = sum_{p in [ptr[v], ptr[v+1])} val[p] * R[idx[p]*ldr + e]
//
// v runs over the vectors of the compressed operand (rows of A' / columns of B'), e over the
// free dimension of the dense residual codes, which are stored k-major so that consecutive
// lanes read consecutive bytes.  side 0 accumulates into C[v, e], side 1 into C[e, v].
#include "srq_internal.h"

namespace srq {
namespace {

constexpr int kLaneElems = 4;                 // consecutive e handled by one lane
constexpr int kBlockElems = 64 * kLaneElems;  // one wave per block

template <int SIDE>
__global__ __launch_bounds__(64) void spmm_valu_kernel(int64_t nvec, int64_t nelem,
                                                       const int32_t* __restrict__ ptr,
                                                       const int32_t* __restrict__ idx,
                                                       const int8_t* __restrict__ val, int64_t capacity,
                                                       const int8_t* __restrict__ R, int64_t ldr,
                                                       GemmEpilogue ep) {
  const int64_t v = blockIdx.y;
  const int64_t e0 = (int64_t)blockIdx.x * kBlockElems + threadIdx.x * kLaneElems;
  int64_t p0 = ptr[v], p1 = ptr[v + 1];
  if (p1 > capacity) p1 = capacity;
  int acc[kLaneElems] = {0, 0, 0, 0};
  const bool full = e0 + kLaneElems <= nelem;
  const bool vec = full && (((reinterpret_cast<uintptr_t>(R) | (uintptr_t)ldr) & 3) == 0);
  if (e0 < nelem) {
    for (int64_t p = p0; p < p1; ++p) {
      const int a = val[p];
      const int8_t* src = R + (int64_t)idx[p] * ldr + e0;
      if (vec) {
        int w = *reinterpret_cast<const int*>(src);
        acc[0] += a * (int)(int8_t)(w & 0xff);
        acc[1] += a * (int)(int8_t)((w >> 8) & 0xff);
        acc[2] += a * (int)(int8_t)((w >> 16) & 0xff);
        acc[3] += a * (w >> 24);
      } else {
#pragma unroll
        for (int t = 0; t < kLaneElems; ++t)
          if (e0 + t < nelem) acc[t] += a * (int)src[t];
      }
    }
#pragma unroll
    for (int t = 0; t < kLaneElems; ++t) {
      int64_t e = e0 + t;
      if (e >= nelem) break;
      int64_t i = SIDE == 0 ? v : e;
      int64_t j = SIDE == 0 ? e : v;
      float d = (float)acc[t] * (ep.s_row[i] * ep.s_col[j]);
      if (ep.D_int) ep.D_int[i * ep.ldd + j] = acc[t];
      float out = ep.C[i * ep.ldc + j] + d;
      if (ep.final_scale) {
        out = ep.alpha * out;
        if (ep.beta != 0.f) out = out + ep.beta * ep.Cin[i * ep.ldcin + j];
      }
      ep.C[i * ep.ldc + j] = out;
    }
  }
}

}  // namespace

hipError_t launch_spmm_valu(int side, int64_t nvec, int64_t nelem, const int32_t* ptr,
                            const int32_t* idx, const int8_t* val, int64_t capacity, const int8_t* R,
                            int64_t ldr, const GemmEpilogue& ep, hipStream_t st) {
  if (nvec <= 0 || nelem <= 0) return hipSuccess;
  const int64_t kMaxY = 65535;
  for (int64_t v0 = 0; v0 < nvec; v0 += kMaxY) {   // gridDim.y is limited to 65535
    int64_t nv = nvec - v0 < kMaxY ? nvec - v0 : kMaxY;
    GemmEpilogue e2 = ep;
    const int32_t* p2 = ptr + v0;
    // shift the output window so that blockIdx.y = 0 is vector v0
    if (side == 0) {
      e2.C = ep.C + v0 * ep.ldc;
      e2.s_row = ep.s_row + v0;
      if (ep.D_int) e2.D_int = ep.D_int + v0 * ep.ldd;
      if (ep.Cin) e2.Cin = ep.Cin + v0 * ep.ldcin;
    } else {
      e2.C = ep.C + v0;
      e2.s_col = ep.s_col + v0;
      if (ep.D_int) e2.D_int = ep.D_int + v0;
      if (ep.Cin) e2.Cin = ep.Cin + v0;
    }
    dim3 grid((unsigned)((nelem + kBlockElems - 1) / kBlockElems), (unsigned)nv);
    if (side == 0)
      hipLaunchKernelGGL(spmm_valu_kernel<0>, grid, dim3(64), 0, st, nv, nelem, p2, idx, val, capacity, R,
                         ldr, e2);
    else
      hipLaunchKernelGGL(spmm_valu_kernel<1>, grid, dim3(64), 0, st, nv, nelem, p2, idx, val, capacity, R,
                         ldr, e2);
  }
  return hipGetLastError();
}

}  // namespace srq
