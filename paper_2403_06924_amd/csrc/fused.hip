// Streaming kernels of the timed path, laid out for HBM bandwidth (Algorithm 1 lines 1, 4-6,
// 8-10).  They compute exactly what the generic kernels in quantize.hip / select.hip compute,
// with fewer passes over the FP32 operands:
//
//   rows_fused_kernel   operand A (one scale per row): the row is read ONCE into registers;
//                       amax, lambda, codes, residual, residual amax and residual codes all
//                       come out of that one read.
//   cols_pass_kernel    operand B (one scale per column, row-major K x N): three streaming
//                       passes (amax | codes + max|residual| | residual codes), each thread
//                       holding a 16-row x 4-column patch so that the transposed (K-contiguous)
//                       INT8 output is written 16 bytes at a time without going through LDS.
//   *_mask_kernel       threshold compare of Eq. avgQuan -> one keep-bit per element (the only
//                       pass that has to re-read FP32 after the first product) + per-vector
//                       counts.  Inside the whole-path call the residual codes whose layout is
//                       only needed after the selection come out of this read as well: B's
//                       third pass is the selection pass (cols_pass_kernel<kColsMaskResid>),
//                       and the k-major residual codes of A are written by A's selection pass
//                       when the vector ALUs will run the second term
//                       (rows_resid_em_kernel<true>).
//   scatter_mask_kernel compaction to CSR / CSC from the bit mask and the INT8 codes.
#include <cstring>
#include "srq_internal.h"

namespace srq {
namespace {

__device__ __forceinline__ int quant_code(float x, float lam, float qmax, int trunc) {
  float y = x * lam;
  float r = trunc ? truncf(y) : rintf(y);
  r = fminf(fmaxf(r, -qmax), qmax);
  return (int)r;
}

__device__ __forceinline__ float block_max_256(float m, float* sm) {
  for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
  __syncthreads();                                   // sm may still be read from a previous use
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = m;
  __syncthreads();
  return fmaxf(fmaxf(sm[0], sm[1]), fmaxf(sm[2], sm[3]));
}

// 16-byte load that does not displace cached data (used for the last read of an operand before
// a product runs in between)
__device__ __forceinline__ float4 load_streaming(const float4* p) {
  typedef float f4v __attribute__((ext_vector_type(4)));
  f4v t = __builtin_nontemporal_load(reinterpret_cast<const f4v*>(p));
  return make_float4(t.x, t.y, t.z, t.w);
}

__device__ __forceinline__ unsigned pack4(int a, int b, int c, int d) {
  return (unsigned)(a & 0xff) | ((unsigned)(b & 0xff) << 8) | ((unsigned)(c & 0xff) << 16) |
         ((unsigned)(d & 0xff) << 24);
}

// ---- operand with contiguous vectors (A): one 256-thread block per row --------------------
template <int NV4>   // float4 pieces per thread; the row has at most 1024*NV4 elements
__global__ __launch_bounds__(256) void rows_fused_kernel(const float* __restrict__ X, int64_t cols,
                                                         int64_t ldx, float qmax, int trunc,
                                                         int8_t* __restrict__ Q, int64_t ldq,
                                                         float* __restrict__ scale, float* __restrict__ lambda,
                                                         int8_t* __restrict__ Rq, int64_t ldr,
                                                         float* __restrict__ rscale,
                                                         float* __restrict__ rlambda,
                                                         // when given, the row's scale and lambda are taken
                                                         // from here instead of from its maximum (and not
                                                         // written back)
                                                         const float* __restrict__ given_scale,
                                                         const float* __restrict__ given_lambda,
                                                         // words this launch zeroes on the side (one per
                                                         // thread and array), so that the kernels after it
                                                         // need no launch to clear their accumulators
                                                         ClearList clr) {
  __shared__ float sm[4];
  {
    const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (clr.a && g < clr.na) clr.a[g] = 0u;
    if (clr.b && g < clr.nb) clr.b[g] = 0u;
    if (clr.c && g < clr.nc) clr.c[g] = 0u;
  }
  const int64_t row = blockIdx.x;
  const float4* src = reinterpret_cast<const float4*>(X + row * ldx);
  const int64_t n4 = cols >> 2;
  float4 x[NV4];
  float m = 0.f;
#pragma unroll
  for (int i = 0; i < NV4; ++i) {
    int64_t c4 = threadIdx.x + i * 256;
    x[i] = c4 < n4 ? load_streaming(src + c4) : make_float4(0.f, 0.f, 0.f, 0.f);
    m = fmaxf(m, fmaxf(fmaxf(fabsf(x[i].x), fabsf(x[i].y)), fmaxf(fabsf(x[i].z), fabsf(x[i].w))));
  }
  float lam = 0.f, s = 0.f;
  if (given_scale) {
    lam = given_lambda[row];
    s = given_scale[row];
  } else {
    const float amax = block_max_256(m, sm);
    if (amax > 0.f) { lam = qmax / amax; s = amax / qmax; }
  }
  unsigned* qdst = reinterpret_cast<unsigned*>(Q + row * ldq);
  float rm = 0.f;
#pragma unroll
  for (int i = 0; i < NV4; ++i) {
    int64_t c4 = threadIdx.x + i * 256;
    int q0 = quant_code(x[i].x, lam, qmax, trunc), q1 = quant_code(x[i].y, lam, qmax, trunc);
    int q2 = quant_code(x[i].z, lam, qmax, trunc), q3 = quant_code(x[i].w, lam, qmax, trunc);
    if (c4 < n4) __builtin_nontemporal_store(pack4(q0, q1, q2, q3), &qdst[c4]);
    if (rscale) {
      // residual r = fl(x - fl(float(q) * s)); kept in place of x
      x[i].x = x[i].x - (float)q0 * s; x[i].y = x[i].y - (float)q1 * s;
      x[i].z = x[i].z - (float)q2 * s; x[i].w = x[i].w - (float)q3 * s;
      rm = fmaxf(rm, fmaxf(fmaxf(fabsf(x[i].x), fabsf(x[i].y)), fmaxf(fabsf(x[i].z), fabsf(x[i].w))));
    }
  }
  if (threadIdx.x == 0 && !given_scale) { scale[row] = s; lambda[row] = lam; }
  if (!rscale) return;
  const float ramax = block_max_256(rm, sm);
  float rlam = 0.f, rs = 0.f;
  if (ramax > 0.f) { rlam = qmax / ramax; rs = ramax / qmax; }
  if (threadIdx.x == 0) {
    rscale[row] = rs;
    if (rlambda) rlambda[row] = rlam;
  }
  if (!Rq) return;                                   // residual scales only: the codes are written elsewhere
  unsigned* rdst = reinterpret_cast<unsigned*>(Rq + row * ldr);
#pragma unroll
  for (int i = 0; i < NV4; ++i) {
    int64_t c4 = threadIdx.x + i * 256;
    if (c4 < n4)
      // (residual codes are first read two products later: kept out of the caches)
      __builtin_nontemporal_store(pack4(quant_code(x[i].x, rlam, qmax, trunc), quant_code(x[i].y, rlam, qmax, trunc),
                                        quant_code(x[i].z, rlam, qmax, trunc), quant_code(x[i].w, rlam, qmax, trunc)),
                                  &rdst[c4]);
  }
}

// ---- operand with strided vectors (B, columns of a row-major matrix) ------------------------
// A block of 256 threads covers (256 / CG * 16) rows x (4 * CG) columns; thread (cg, rb) holds rows
// rb*16..rb*16+15 of the four columns cg*4..cg*4+3.  CG sets the shape: the wider the block, the
// longer the contiguous piece of a row that one load instruction of a wave fetches (16 * CG bytes,
// up to 1 KiB), the shorter the contiguous piece of a column of transposed codes a block writes.
// (kColsMaskResid: the selection pass also writes the residual codes, so that B is read three
// times per call and not four)
constexpr int kCgAmax = 16, kCgMask = 8, kCgCodes = 8;   // (measured at 8192^2: 8 beats 16 by 3 % in the passes that write codes, 4 and 32 lose 15 %)
enum ColsMode { kColsAmax = 0, kColsCodes = 1, kColsResid = 2, kColsMask = 3, kColsMaskResid = 4 };
constexpr bool cols_resid(int mode) { return mode == kColsResid || mode == kColsMaskResid; }
constexpr bool cols_mask(int mode) { return mode == kColsMask || mode == kColsMaskResid; }
// column groups per block of each pass (powers of two, 16..64)
constexpr int cols_cg(int mode) { return mode == kColsAmax ? kCgAmax : mode == kColsMask ? kCgMask : kCgCodes; }

template <int MODE>
__global__ __launch_bounds__(256) void cols_pass_kernel(
    const float* __restrict__ X, int64_t rows, int64_t cols, int64_t ldx, float qmax, int trunc,
    const float* __restrict__ scale, const float* __restrict__ lambda, const float* __restrict__ rlambda,
    // when given, the scales are derived here from the maxima of an earlier pass (their bit
    // patterns) and the first row of blocks writes them out: no separate kernel in between
    const uint32_t* __restrict__ amax_in, float* __restrict__ scale_out, float* __restrict__ lambda_out,
    const float* __restrict__ thresh, uint32_t* __restrict__ amax_bits,   // amax or residual amax (bits)
    int8_t* __restrict__ Qvm, int64_t ldvm,      // transposed output [col][row], may be null
    int8_t* __restrict__ Qem, int64_t ldem,      // straight output [row][col], may be null
    uint8_t* __restrict__ mask, int64_t mask_stride,   // bytes per column of the transposed bit mask
    int32_t* __restrict__ counts, RunIf run) {
  constexpr int CG = cols_cg(MODE), BC = 4 * CG, BR = 256 / CG * 16;   // block: BR rows x BC columns
  __shared__ uint32_t red[BC];
  if (!run_if_ok(run)) return;
  const int cg = threadIdx.x & (CG - 1), rb = threadIdx.x / CG;
  const int64_t col0 = (int64_t)blockIdx.x * BC + cg * 4;
  const int64_t row0 = (int64_t)blockIdx.y * BR + rb * 16;
  const bool colok = col0 < cols;                 // cols is a multiple of 4
  if (MODE != kColsResid) {
    if (threadIdx.x < BC) red[threadIdx.x] = 0;
    __syncthreads();
  }
  float4 v[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    int64_t r = row0 + i;
    const float4* src = reinterpret_cast<const float4*>(X + r * ldx + col0);
    const bool ok = colok && r < rows;
    if (cols_resid(MODE) || cols_mask(MODE)) v[i] = ok ? load_streaming(src) : make_float4(0.f, 0.f, 0.f, 0.f);
    else v[i] = ok ? *src : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  if (MODE == kColsAmax) {
    float m[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      m[0] = fmaxf(m[0], fabsf(v[i].x)); m[1] = fmaxf(m[1], fabsf(v[i].y));
      m[2] = fmaxf(m[2], fabsf(v[i].z)); m[3] = fmaxf(m[3], fabsf(v[i].w));
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) atomicMax(&red[cg * 4 + c], __float_as_uint(m[c]));
    __syncthreads();
    if (threadIdx.x < BC) {
      int64_t col = (int64_t)blockIdx.x * BC + threadIdx.x;
      if (col < cols) atomicMax(&amax_bits[col], red[threadIdx.x]);
    }
    return;
  }
  if (cols_mask(MODE)) {
    float4 t = colok ? *reinterpret_cast<const float4*>(thresh + col0) : make_float4(0.f, 0.f, 0.f, 0.f);
    const float tt[4] = {t.x, t.y, t.z, t.w};
    unsigned bits[4] = {0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      bool ok = colok && row0 + i < rows;
      const float xv[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
      for (int c = 0; c < 4; ++c) bits[c] |= (ok && fabsf(xv[c]) > tt[c]) ? (1u << i) : 0u;
    }
    if (colok && row0 < mask_stride * 8) {
#pragma unroll
      for (int c = 0; c < 4; ++c)
        *reinterpret_cast<uint16_t*>(mask + (col0 + c) * mask_stride + (row0 >> 3)) = (uint16_t)bits[c];
    }
#pragma unroll
    for (int c = 0; c < 4; ++c)
      if (bits[c]) atomicAdd(&red[cg * 4 + c], (uint32_t)__popc(bits[c]));
    __syncthreads();
    if (threadIdx.x < BC) {
      int64_t col = (int64_t)blockIdx.x * BC + threadIdx.x;
      if (col < cols && red[threadIdx.x]) atomicAdd(&counts[col], (int32_t)red[threadIdx.x]);
    }
    if (MODE == kColsMask) return;
  }
  // codes / residual codes
  float lam[4] = {0.f, 0.f, 0.f, 0.f}, sc[4] = {0.f, 0.f, 0.f, 0.f}, rlam[4] = {0.f, 0.f, 0.f, 0.f};
  const bool writer = blockIdx.y == 0 && rb == 0 && colok;
  if (MODE == kColsCodes && amax_in) {
    if (colok) {
      const uint4 a4 = *reinterpret_cast<const uint4*>(amax_in + col0);
      const float am[4] = {__uint_as_float(a4.x), __uint_as_float(a4.y), __uint_as_float(a4.z), __uint_as_float(a4.w)};
#pragma unroll
      for (int c = 0; c < 4; ++c)
        if (am[c] > 0.f) { lam[c] = qmax / am[c]; sc[c] = am[c] / qmax; }
    }
    if (writer) {
      *reinterpret_cast<float4*>(scale_out + col0) = make_float4(sc[0], sc[1], sc[2], sc[3]);
      *reinterpret_cast<float4*>(lambda_out + col0) = make_float4(lam[0], lam[1], lam[2], lam[3]);
    }
  } else if (colok) {
    float4 l4 = *reinterpret_cast<const float4*>(lambda + col0);
    float4 s4 = *reinterpret_cast<const float4*>(scale + col0);
    lam[0] = l4.x; lam[1] = l4.y; lam[2] = l4.z; lam[3] = l4.w;
    sc[0] = s4.x; sc[1] = s4.y; sc[2] = s4.z; sc[3] = s4.w;
  }
  if (cols_resid(MODE) && colok) {
    if (amax_in) {
      const uint4 a4 = *reinterpret_cast<const uint4*>(amax_in + col0);
      const float am[4] = {__uint_as_float(a4.x), __uint_as_float(a4.y), __uint_as_float(a4.z), __uint_as_float(a4.w)};
      float rs[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int c = 0; c < 4; ++c)
        if (am[c] > 0.f) { rlam[c] = qmax / am[c]; rs[c] = am[c] / qmax; }
      if (writer) {
        *reinterpret_cast<float4*>(scale_out + col0) = make_float4(rs[0], rs[1], rs[2], rs[3]);
        *reinterpret_cast<float4*>(lambda_out + col0) = make_float4(rlam[0], rlam[1], rlam[2], rlam[3]);
      }
    } else {
      float4 r4 = *reinterpret_cast<const float4*>(rlambda + col0);
      rlam[0] = r4.x; rlam[1] = r4.y; rlam[2] = r4.z; rlam[3] = r4.w;
    }
  }
  float rm[4] = {0.f, 0.f, 0.f, 0.f};
  unsigned packed[4][4];                            // [column][word]: 16 codes of one column
#pragma unroll
  for (int c = 0; c < 4; ++c)
#pragma unroll
    for (int wd = 0; wd < 4; ++wd) packed[c][wd] = 0;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const float xv[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
    int code[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      int q = quant_code(xv[c], lam[c], qmax, trunc);
      float res = xv[c] - (float)q * sc[c];
      if (MODE == kColsCodes) {
        code[c] = q;
        rm[c] = fmaxf(rm[c], fabsf(res));
      } else {
        code[c] = quant_code(res, rlam[c], qmax, trunc);
      }
      packed[c][i >> 2] |= (unsigned)(code[c] & 0xff) << (8 * (i & 3));
    }
    if (Qem && colok && row0 + i < rows)
      *reinterpret_cast<unsigned*>(Qem + (row0 + i) * ldem + col0) = pack4(code[0], code[1], code[2], code[3]);
  }
  if (Qvm && colok && row0 < rows) {
    const bool full = row0 + 16 <= rows;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      int8_t* dst = Qvm + (col0 + c) * ldvm + row0;
      if (full) {
        typedef unsigned u4v __attribute__((ext_vector_type(4)));
        u4v pk = {packed[c][0], packed[c][1], packed[c][2], packed[c][3]};
        __builtin_nontemporal_store(pk, reinterpret_cast<u4v*>(dst));
      } else {
        for (int i = 0; i < 16; ++i)
          if (row0 + i < rows) dst[i] = (int8_t)((packed[c][i >> 2] >> (8 * (i & 3))) & 0xff);
      }
    }
  }
  if (MODE == kColsCodes && amax_bits) {
#pragma unroll
    for (int c = 0; c < 4; ++c) atomicMax(&red[cg * 4 + c], __float_as_uint(rm[c]));
    __syncthreads();
    if (threadIdx.x < BC) {
      int64_t col = (int64_t)blockIdx.x * BC + threadIdx.x;
      if (col < cols) atomicMax(&amax_bits[col], red[threadIdx.x]);
    }
  }
}

// ---- k-major residual codes of the row-scaled operand (RA as K x M, read by the vector-ALU
// execution of the second correction term): the 16-row x 4-column patches of cols_pass_kernel
// with the scales taken per row, so that the sixteen codes of one k go out as one 16-byte store.
// MASK: the pass is also the selection pass of the operand (threshold compare per row; cols is
// then a multiple of 64): the sixteen lanes that share a row assemble its 64 keep-bits with
// shuffles.  The per-row counts are taken from the mask afterwards (mask_count_kernel).
template <bool MASK>
__global__ __launch_bounds__(256) void rows_resid_em_kernel(const float* __restrict__ X, int64_t rows,
                                                            int64_t cols, int64_t ldx, float qmax, int trunc,
                                                            const float* __restrict__ scale,
                                                            const float* __restrict__ lambda,
                                                            const float* __restrict__ rlambda,
                                                            int8_t* __restrict__ Rem, int64_t ldem,
                                                            const float* __restrict__ thresh,
                                                            uint8_t* __restrict__ mask, int64_t mask_stride,
                                                            RunIf run) {
  if (!run_if_ok(run)) return;
  const int cg = threadIdx.x & 15, rb = threadIdx.x >> 4;
  const int64_t col0 = (int64_t)blockIdx.x * 64 + cg * 4;
  const int64_t row0 = (int64_t)blockIdx.y * 256 + rb * 16;     // rows is a multiple of 16
  if (col0 >= cols || row0 >= rows) return;
  float sc[16], lam[16], rlam[16];
#pragma unroll
  for (int i = 0; i < 16; i += 4) {
    const float4 a = *reinterpret_cast<const float4*>(scale + row0 + i);
    const float4 b = *reinterpret_cast<const float4*>(lambda + row0 + i);
    const float4 c = *reinterpret_cast<const float4*>(rlambda + row0 + i);
    sc[i] = a.x; sc[i + 1] = a.y; sc[i + 2] = a.z; sc[i + 3] = a.w;
    lam[i] = b.x; lam[i + 1] = b.y; lam[i + 2] = b.z; lam[i + 3] = b.w;
    rlam[i] = c.x; rlam[i + 1] = c.y; rlam[i + 2] = c.z; rlam[i + 3] = c.w;
  }
  float4 v[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) v[i] = load_streaming(reinterpret_cast<const float4*>(X + (row0 + i) * ldx + col0));
  if (MASK) {
#pragma unroll
    for (int i = 0; i < 16; i += 4) {
      const float4 t4 = *reinterpret_cast<const float4*>(thresh + row0 + i);
      const float tt[4] = {t4.x, t4.y, t4.z, t4.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float4 x = v[i + j];
        const float t = tt[j];
        const unsigned nib = (fabsf(x.x) > t ? 1u : 0u) | (fabsf(x.y) > t ? 2u : 0u) |
                             (fabsf(x.z) > t ? 4u : 0u) | (fabsf(x.w) > t ? 8u : 0u);
        // (all sixteen lanes of a row are active together: cols is a multiple of 64)
        const unsigned b8 = nib | (__shfl_down(nib, 1, 64) << 4);
        const unsigned b16 = b8 | (__shfl_down(b8, 2, 64) << 8);
        const unsigned b32 = b16 | (__shfl_down(b16, 4, 64) << 16);
        if (!(cg & 7)) *reinterpret_cast<unsigned*>(mask + (row0 + i + j) * mask_stride + (col0 >> 3)) = b32;
      }
    }
  }
  unsigned packed[4][4];
#pragma unroll
  for (int c = 0; c < 4; ++c)
#pragma unroll
    for (int wd = 0; wd < 4; ++wd) packed[c][wd] = 0;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const float xv[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int q = quant_code(xv[c], lam[i], qmax, trunc);
      const float res = xv[c] - (float)q * sc[i];
      const int code = quant_code(res, rlam[i], qmax, trunc);
      packed[c][i >> 2] |= (unsigned)(code & 0xff) << (8 * (i & 3));
    }
  }
  typedef unsigned u4v __attribute__((ext_vector_type(4)));
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    u4v pk = {packed[c][0], packed[c][1], packed[c][2], packed[c][3]};
    __builtin_nontemporal_store(pk, reinterpret_cast<u4v*>(Rem + (col0 + c) * ldem + row0));
  }
}

// kept entries per vector from a finished mask: one wave per vector
__global__ __launch_bounds__(256) void mask_count_kernel(const uint64_t* __restrict__ mask, int64_t words,
                                                         int64_t nvec, int32_t* __restrict__ counts) {
  const int64_t v = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (v >= nvec) return;
  const int lane = threadIdx.x & 63;
  int total = 0;
  for (int64_t wd = lane; wd < words; wd += 64) total += __popcll(mask[v * words + wd]);
  for (int off = 32; off > 0; off >>= 1) total += __shfl_xor(total, off, 64);
  if (lane == 0) counts[v] = total;
}

// ---- keep-mask of an operand with contiguous vectors (A): one block per row ------------------
// Generic version: one 64-bit word per wave iteration via ballot.
__global__ __launch_bounds__(256) void rows_mask_kernel(const float* __restrict__ X, int64_t cols, int64_t ldx,
                                                        const float* __restrict__ thresh,
                                                        uint64_t* __restrict__ mask, int64_t words,
                                                        int32_t* __restrict__ counts) {
  __shared__ int sm[4];
  const int64_t row = blockIdx.x;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const float t = thresh[row];
  const float* src = X + row * ldx;
  int total = 0;
  for (int64_t wd = w; wd < words; wd += 4) {
    int64_t e = wd * 64 + lane;
    bool keep = e < cols && fabsf(src[e]) > t;
    unsigned long long m = __ballot(keep);
    if (lane == 0) mask[row * words + wd] = m;
    total += __popcll(m);
  }
  if (lane == 0) sm[w] = total;
  __syncthreads();
  if (threadIdx.x == 0) counts[row] = sm[0] + sm[1] + sm[2] + sm[3];
}

// Streaming version (16-byte aligned rows of at most 1024*NV4 elements): every thread has all
// of its float4 loads in flight at once; two neighbouring threads make one mask byte.
template <int NV4>
__global__ __launch_bounds__(256) void rows_mask_vec_kernel(const float* __restrict__ X, int64_t cols, int64_t ldx,
                                                            const float* __restrict__ thresh,
                                                            uint8_t* __restrict__ mask, int64_t mask_stride,
                                                            int32_t* __restrict__ counts) {
  __shared__ int sm[4];
  const int64_t row = blockIdx.x;
  const float t = thresh[row];
  const float4* src = reinterpret_cast<const float4*>(X + row * ldx);
  const int64_t n4 = cols >> 2;
  float4 x[NV4];
#pragma unroll
  for (int i = 0; i < NV4; ++i) {
    int64_t c4 = threadIdx.x + i * 256;
    x[i] = c4 < n4 ? load_streaming(src + c4) : make_float4(0.f, 0.f, 0.f, 0.f);   // |0| > t is false for every t >= 0
  }
  uint8_t* mrow = mask + row * mask_stride;
  int total = 0;
#pragma unroll
  for (int i = 0; i < NV4; ++i) {
    int64_t c4 = threadIdx.x + i * 256;
    unsigned nib = (fabsf(x[i].x) > t ? 1u : 0u) | (fabsf(x[i].y) > t ? 2u : 0u) |
                   (fabsf(x[i].z) > t ? 4u : 0u) | (fabsf(x[i].w) > t ? 8u : 0u);
    if (c4 >= n4) nib = 0;
    total += __popc(nib);
    // eight neighbouring lanes assemble one 32-bit piece of the mask
    unsigned b8 = nib | (__shfl_down(nib, 1, 64) << 4);
    unsigned b16 = b8 | (__shfl_down(b8, 2, 64) << 8);
    unsigned b32 = b16 | (__shfl_down(b16, 4, 64) << 16);
    if (!(threadIdx.x & 7) && (c4 >> 1) < mask_stride)
      *reinterpret_cast<unsigned*>(mrow + (c4 >> 1)) = b32;
  }
  for (int off = 32; off > 0; off >>= 1) total += __shfl_xor(total, off, 64);
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = total;
  __syncthreads();
  if (threadIdx.x == 0) counts[row] = sm[0] + sm[1] + sm[2] + sm[3];
}

// ---- compaction: one block per vector, a quarter of the vector per wave.  A wave first counts
// the kept entries of its quarter from the mask words (that fixes where it writes), then walks
// the quarter 256 elements at a time, four per lane: the position of a lane's first kept entry
// is the wave's running offset plus the number of kept entries in lower lanes, obtained from
// three ballots of the bits of the lane's own count (0..4).  Neighbouring lanes therefore write
// neighbouring slots of idx / val at any density.  Optionally the vector is also written
// expanded to zero-filled dense codes (operand of the matrix-core execution of the sparse
// product), from the same registers.
template <bool SKIP>   // SKIP: for operands that keep well under one entry per 256 elements and
                       // need no expansion; a wave looks at the mask first and leaves the codes
                       // of a chunk without kept entries unread
__global__ __launch_bounds__(256) void scatter_mask_kernel(const uint64_t* __restrict__ mask, int64_t words,
                                                           int64_t veclen, const int8_t* __restrict__ Q,
                                                           int64_t ldq, const int32_t* __restrict__ ptr,
                                                           int32_t* __restrict__ idx, int8_t* __restrict__ val,
                                                           int64_t capacity, int8_t* __restrict__ dense,
                                                           int64_t ldd, RunIf dense_if) {
  __shared__ int wsum[4];
  const int64_t v = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const uint64_t* mv = mask + v * words;
  const uint32_t* mv32 = reinterpret_cast<const uint32_t*>(mv);
  const int8_t* qv = Q + v * ldq;
  int8_t* dv = (dense && run_if_ok(dense_if)) ? dense + v * ldd : nullptr;
  const bool qvec = (reinterpret_cast<uintptr_t>(qv) & 3) == 0;
  const bool dvec = dv && (reinterpret_cast<uintptr_t>(dv) & 3) == 0;
  // chunks of 256 elements (four mask words); wave w owns chunks [c0, c1)
  const int64_t nchunks = (veclen + 255) >> 8;
  const int64_t cpw = (nchunks + 3) >> 2;
  const int64_t c0 = w * cpw < nchunks ? w * cpw : nchunks;
  const int64_t c1 = c0 + cpw < nchunks ? c0 + cpw : nchunks;
  int mine = 0;
  for (int64_t i = c0 * 4 + lane; i < c1 * 4 && i < words; i += 64) {
    uint64_t m = mv[i];
    const int64_t left = veclen - i * 64;                 // bits at and past veclen do not count
    if (left < 64) m &= (1ull << left) - 1ull;
    mine += __popcll(m);
  }
  for (int off = 32; off > 0; off >>= 1) mine += __shfl_xor(mine, off, 64);
  if (lane == 0) wsum[w] = mine;
  __syncthreads();
  int64_t pos = ptr[v];
  for (int i = 0; i < w; ++i) pos += wsum[i];
  const uint64_t lower = (1ull << lane) - 1ull;
  for (int64_t c = c0; c < c1; ++c) {
    const int64_t e = c * 256 + 4 * lane;
    unsigned nib = 0, code = 0;
    if (SKIP) {
      if (e < veclen) nib = (mv32[e >> 5] >> (e & 31)) & 0xfu;   // the tail is masked below
      if (!__ballot(nib != 0)) continue;
    }
    if (e < veclen) {
      nib = (mv32[e >> 5] >> (e & 31)) & 0xfu;
      const int64_t left = veclen - e;
      if (left < 4) nib &= (1u << left) - 1u;
      if (qvec && left >= 4) {
        code = *reinterpret_cast<const unsigned*>(qv + e);
      } else {
        for (int j = 0; j < 4 && j < left; ++j) code |= (unsigned)(uint8_t)qv[e + j] << (8 * j);
      }
      if (dv) {
        const unsigned keep = ((nib & 1u) ? 0xffu : 0u) | ((nib & 2u) ? 0xff00u : 0u) |
                              ((nib & 4u) ? 0xff0000u : 0u) | ((nib & 8u) ? 0xff000000u : 0u);
        const unsigned out = code & keep;
        if (dvec && left >= 4) {
          __builtin_nontemporal_store(out, reinterpret_cast<unsigned*>(dv + e));
        } else {
          for (int j = 0; j < 4 && j < left; ++j) dv[e + j] = (int8_t)(out >> (8 * j));
        }
      }
    }
    const int cnt = __popc(nib);
    const uint64_t b0 = __ballot(cnt & 1), b1 = __ballot(cnt & 2), b2 = __ballot(cnt & 4);
    int64_t p = pos + __popcll(b0 & lower) + 2 * __popcll(b1 & lower) + 4 * __popcll(b2 & lower);
    pos += __popcll(b0) + 2 * __popcll(b1) + 4 * __popcll(b2);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (nib >> j & 1u) {
        if (p < capacity) {
          idx[p] = (int32_t)(e + j);
          val[p] = (int8_t)(code >> (8 * j));
        }
        ++p;
      }
    }
  }
}

// The same compaction for long, 16-byte aligned vectors: sixteen elements per lane (one 16-byte
// code load, one 16-bit piece of the mask, one 16-byte store of the expansion) and one pair of
// idx / val stores per kept entry, i.e. a quarter of the memory instructions of the kernel above
// at low and medium densities.  Chunks are 1024 elements; wave w owns chunks [c0, c1).
template <bool SKIP>
__global__ __launch_bounds__(256) void scatter_mask16_kernel(const uint64_t* __restrict__ mask, int64_t words,
                                                             int64_t veclen, const int8_t* __restrict__ Q,
                                                             int64_t ldq, const int32_t* __restrict__ ptr,
                                                             int32_t* __restrict__ idx, int8_t* __restrict__ val,
                                                             int64_t capacity, int8_t* __restrict__ dense,
                                                             int64_t ldd, RunIf dense_if) {
  __shared__ int wsum[4];
  const int64_t v = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const uint64_t* mv = mask + v * words;
  const uint16_t* mv16 = reinterpret_cast<const uint16_t*>(mv);
  const int8_t* qv = Q + v * ldq;                        // 16-byte aligned (checked by the launcher)
  int8_t* dv = (dense && run_if_ok(dense_if)) ? dense + v * ldd : nullptr;   // likewise
  const int64_t nchunks = (veclen + 1023) >> 10;
  const int64_t cpw = (nchunks + 3) >> 2;
  const int64_t c0 = w * cpw < nchunks ? w * cpw : nchunks;
  const int64_t c1 = c0 + cpw < nchunks ? c0 + cpw : nchunks;
  int mine = 0;
  for (int64_t i = c0 * 16 + lane; i < c1 * 16 && i < words; i += 64) {
    uint64_t m = mv[i];
    const int64_t left = veclen - i * 64;                 // bits at and past veclen do not count
    if (left < 64) m &= (1ull << left) - 1ull;
    mine += __popcll(m);
  }
  for (int off = 32; off > 0; off >>= 1) mine += __shfl_xor(mine, off, 64);
  if (lane == 0) wsum[w] = mine;
  __syncthreads();
  int64_t pos = ptr[v];
  for (int i = 0; i < w; ++i) pos += wsum[i];
  const uint64_t lower = (1ull << lane) - 1ull;
  typedef unsigned u4v __attribute__((ext_vector_type(4)));
  for (int64_t c = c0; c < c1; ++c) {
    const int64_t e = c * 1024 + 16 * lane;
    const int64_t left = veclen - e;
    unsigned m = 0;
    if (left > 0) {
      m = mv16[e >> 4];
      if (left < 16) m &= (1u << left) - 1u;
    }
    if (SKIP && !__ballot(m != 0)) continue;
    unsigned cw[4] = {0u, 0u, 0u, 0u};
    if (left >= 16) {
      const u4v t = *reinterpret_cast<const u4v*>(qv + e);
      cw[0] = t.x; cw[1] = t.y; cw[2] = t.z; cw[3] = t.w;
    } else if (left > 0) {
      for (int j = 0; j < left; ++j) {
        const unsigned byte = (unsigned)(uint8_t)qv[e + j] << (8 * (j & 3));
        cw[0] |= (j >> 2) == 0 ? byte : 0u; cw[1] |= (j >> 2) == 1 ? byte : 0u;
        cw[2] |= (j >> 2) == 2 ? byte : 0u; cw[3] |= (j >> 2) == 3 ? byte : 0u;
      }
    }
    if (dv && left > 0) {
      unsigned ow[4];
#pragma unroll
      for (int wd = 0; wd < 4; ++wd) {
        const unsigned nib = (m >> (4 * wd)) & 0xfu;
        const unsigned keep = ((nib & 1u) ? 0xffu : 0u) | ((nib & 2u) ? 0xff00u : 0u) |
                              ((nib & 4u) ? 0xff0000u : 0u) | ((nib & 8u) ? 0xff000000u : 0u);
        ow[wd] = cw[wd] & keep;
      }
      if (left >= 16) {
        const u4v o = {ow[0], ow[1], ow[2], ow[3]};
        __builtin_nontemporal_store(o, reinterpret_cast<u4v*>(dv + e));
      } else {
        for (int j = 0; j < left; ++j) {
          const unsigned word = (j >> 2) == 0 ? ow[0] : (j >> 2) == 1 ? ow[1] : (j >> 2) == 2 ? ow[2] : ow[3];
          dv[e + j] = (int8_t)(word >> (8 * (j & 3)));
        }
      }
    }
    const int cnt = __popc(m);                                   // 0..16
    const uint64_t b0 = __ballot(cnt & 1), b1 = __ballot(cnt & 2), b2 = __ballot(cnt & 4),
                   b3 = __ballot(cnt & 8), b4 = __ballot(cnt & 16);
    int64_t p = pos + __popcll(b0 & lower) + 2 * __popcll(b1 & lower) + 4 * __popcll(b2 & lower) +
                8 * __popcll(b3 & lower) + 16 * __popcll(b4 & lower);
    pos += __popcll(b0) + 2 * __popcll(b1) + 4 * __popcll(b2) + 8 * __popcll(b3) + 16 * __popcll(b4);
    while (m) {
      const int j = __ffs((int)m) - 1;
      m &= m - 1u;
      if (p < capacity) {
        const unsigned word = (j & 8) ? ((j & 4) ? cw[3] : cw[2]) : ((j & 4) ? cw[1] : cw[0]);
        idx[p] = (int32_t)(e + j);
        val[p] = (int8_t)(word >> (8 * (j & 3)));
      }
      ++p;
    }
  }
}

// Exclusive scan of one count vector by a group of NT threads of a block (tid = index in the group,
// wave_sum = NT / 64 words of LDS of the group's own); the block-wide barrier between the two
// phases is the caller's, so that two groups can scan two vectors side by side.  totals == null:
// nothing to do in either phase.
template <int NT>
struct ScanGroup {
  static constexpr int kHeld = 32;                    // spans of up to 32 vectors are held in registers:
  int32_t held[kHeld];                                // their loads are independent and all in flight at once
  int64_t x, inc, per, v0, v1;
  __device__ __forceinline__ void sums(const int32_t* totals, int64_t nvec, int tid, int64_t* wave_sum) {
    if (!totals) return;
    // thread t owns the `per` consecutive vectors from t * per on
    per = (nvec + NT - 1) / NT;
    v0 = tid * per;
    v1 = v0 + per < nvec ? v0 + per : nvec;
    x = 0;
    if (per <= kHeld) {
#pragma unroll
      for (int i = 0; i < kHeld; ++i) held[i] = v0 + i < v1 ? totals[v0 + i] : 0;
#pragma unroll
      for (int i = 0; i < kHeld; ++i) x += held[i];
    } else {
      for (int64_t v = v0; v < v1; ++v) x += totals[v];
    }
    const int lane = tid & 63;
    inc = x;
    for (int d = 1; d < 64; d <<= 1) {
      int64_t y = __shfl_up(inc, d, 64);
      if (lane >= d) inc += y;
    }
    if (lane == 63) wave_sum[tid >> 6] = inc;
  }
  __device__ __forceinline__ void offsets(const int32_t* totals, int64_t nvec, int32_t* ptr, int64_t* nnz_dev,
                                          int tid, const int64_t* wave_sum) {
    if (!totals) return;
    int64_t run = inc - x;                            // exclusive prefix of this thread's span
    for (int i = 0; i < (tid >> 6); ++i) run += wave_sum[i];
    if (per <= kHeld) {
#pragma unroll
      for (int i = 0; i < kHeld; ++i) {
        if (v0 + i < v1) ptr[v0 + i] = (int32_t)run;
        run += held[i];
      }
    } else {
      for (int64_t v = v0; v < v1; ++v) {
        ptr[v] = (int32_t)run;
        run += totals[v];
      }
    }
    if (tid == NT - 1) {
      ptr[nvec] = (int32_t)run;
      if (nnz_dev) *nnz_dev = run;
    }
  }
};

// Exclusive scans of two count vectors in one launch.  Two blocks of 1024 threads, one scan each;
// or, when the execution of each term is decided on the device (dec.paths != null), ONE block
// whose halves scan one vector each, after which its first thread takes that decision from the
// two totals and writes the call's statistics, so that neither needs a launch of its own.
__global__ __launch_bounds__(1024) void scan_pair_kernel(const int32_t* t0, int64_t n0, int32_t* p0, int64_t* z0,
                                                         const int32_t* t1, int64_t n1, int32_t* p1, int64_t* z1,
                                                         ScanDecision dec) {
  __shared__ int64_t wave_sum[16];
  if (!dec.paths) {
    const bool first = blockIdx.x == 0;
    ScanGroup<1024> g;
    g.sums(first ? t0 : t1, first ? n0 : n1, threadIdx.x, wave_sum);
    __syncthreads();
    g.offsets(first ? t0 : t1, first ? n0 : n1, first ? p0 : p1, first ? z0 : z1, threadIdx.x, wave_sum);
    return;
  }
  const bool first = threadIdx.x < 512;
  const int tid = threadIdx.x & 511;
  int64_t* ws = wave_sum + (first ? 0 : 8);
  ScanGroup<512> g;
  g.sums(first ? t0 : t1, first ? n0 : n1, tid, ws);
  __syncthreads();
  g.offsets(first ? t0 : t1, first ? n0 : n1, first ? p0 : p1, first ? z0 : z1, tid, ws);
  __syncthreads();                                   // (the totals z0 / z1 are visible to the block)
  if (threadIdx.x == 0) {
    const int64_t na = t0 ? *z0 : 0, nb = t1 ? *z1 : 0;
    const int pa = t0 ? (na >= dec.min_mfma_a ? 2 : 1) : 0;
    const int pb = t1 ? (nb >= dec.min_mfma_b ? 2 : 1) : 0;
    dec.paths[0] = pa;
    dec.paths[1] = pb;
    if (dec.seen && pa) dec.seen[0] = pa;
    if (dec.seen && pb) dec.seen[1] = pb;
    if (dec.stats) {
      dec.stats->nnz_a = na;
      dec.stats->nnz_b = nb;
      dec.stats->path_a = pa;
      dec.stats->path_b = pb;
      dec.stats->overflow = (na > dec.cap_a ? 1 : 0) | (nb > dec.cap_b ? 2 : 0);
      dec.stats->reserved = 0;
    }
  }
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

}  // namespace

bool rows_fused_ok(const float* X, int64_t cols, int64_t ldx, const int8_t* Q, int64_t ldq, const int8_t* Rq,
                   int64_t ldr) {
  return cols > 0 && cols <= 16384 && (cols % 4) == 0 && (ldx % 4) == 0 && aligned16(X) && (ldq % 4) == 0 &&
         aligned16(Q) && (!Rq || ((ldr % 4) == 0 && aligned16(Rq)));
}

hipError_t launch_rows_fused(const float* X, int64_t rows, int64_t cols, int64_t ldx, int qmax, int trunc,
                             int8_t* Q, int64_t ldq, float* scale, float* lambda, int8_t* Rq, int64_t ldr,
                             float* rscale, float* rlambda, hipStream_t st, const float* given_scale,
                             const float* given_lambda, const ClearList* clear) {
  if (rows <= 0) return hipSuccess;
  ClearList clr = {nullptr, 0, nullptr, 0, nullptr, 0};
  if (clear) clr = *clear;                                   // (the caller has checked rows_fused_can_clear)
  dim3 grid((unsigned)rows), block(256);
  const float qm = (float)qmax;
#define SRQ_ROWS(NV4)                                                                                        \
  hipLaunchKernelGGL(rows_fused_kernel<NV4>, grid, block, 0, st, X, cols, ldx, qm, trunc, Q, ldq, scale,     \
                     lambda, Rq, ldr, rscale, rlambda, given_scale, given_lambda, clr)
  if (cols <= 1024) SRQ_ROWS(1);
  else if (cols <= 2048) SRQ_ROWS(2);
  else if (cols <= 4096) SRQ_ROWS(4);
  else if (cols <= 8192) SRQ_ROWS(8);
  else SRQ_ROWS(16);
#undef SRQ_ROWS
  return hipGetLastError();
}

bool rows_fused_can_clear(int64_t rows, const ClearList& c) {
  const int64_t threads = rows * 256;
  return rows > 0 && (!c.a || c.na <= threads) && (!c.b || c.nb <= threads) && (!c.c || c.nc <= threads);
}

bool rows_resid_em_ok(const float* X, int64_t rows, int64_t cols, int64_t ldx, const float* scale,
                      const float* lambda, const float* rlambda, const int8_t* Rem, int64_t ldem) {
  return rows > 0 && cols > 0 && (rows % 16) == 0 && (cols % 4) == 0 && (ldx % 4) == 0 && (ldem % 16) == 0 &&
         aligned16(X) && aligned16(scale) && aligned16(lambda) && aligned16(rlambda) && aligned16(Rem);
}

hipError_t launch_rows_resid_em(const float* X, int64_t rows, int64_t cols, int64_t ldx, int qmax, int trunc,
                                const float* scale, const float* lambda, const float* rlambda, int8_t* Rem,
                                int64_t ldem, hipStream_t st, RunIf run) {
  dim3 grid((unsigned)((cols + 63) / 64), (unsigned)((rows + 255) / 256));
  hipLaunchKernelGGL(rows_resid_em_kernel<false>, grid, dim3(256), 0, st, X, rows, cols, ldx, (float)qmax, trunc,
                     scale, lambda, rlambda, Rem, ldem, nullptr, nullptr, 0, run);
  return hipGetLastError();
}

// the same pass doubling as the selection pass of the operand: keep-mask (mask_words(cols) words
// per row) and per-row counts as launch_rows_mask leaves them
bool rows_mask_resid_em_ok(const float* X, int64_t rows, int64_t cols, int64_t ldx, const float* scale,
                           const float* lambda, const float* rlambda, const int8_t* Rem, int64_t ldem,
                           const float* thresh) {
  return rows_resid_em_ok(X, rows, cols, ldx, scale, lambda, rlambda, Rem, ldem) && (cols % 64) == 0 &&
         aligned16(thresh);
}

hipError_t launch_rows_mask_resid_em(const float* X, int64_t rows, int64_t cols, int64_t ldx, int qmax, int trunc,
                                     const float* scale, const float* lambda, const float* rlambda, int8_t* Rem,
                                     int64_t ldem, const float* thresh, uint64_t* mask, int32_t* counts,
                                     hipStream_t st) {
  dim3 grid((unsigned)((cols + 63) / 64), (unsigned)((rows + 255) / 256));
  hipLaunchKernelGGL(rows_resid_em_kernel<true>, grid, dim3(256), 0, st, X, rows, cols, ldx, (float)qmax, trunc,
                     scale, lambda, rlambda, Rem, ldem, thresh, reinterpret_cast<uint8_t*>(mask),
                     mask_words(cols) * 8, kAlways);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(mask_count_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st, mask, mask_words(cols),
                     rows, counts);
  return hipGetLastError();
}

bool cols_pass_ok(const float* X, int64_t cols, int64_t ldx) {
  return cols > 0 && (cols % 4) == 0 && (ldx % 4) == 0 && aligned16(X);
}

static dim3 cols_grid(int mode, int64_t rows, int64_t cols) {
  const int bc = 4 * cols_cg(mode), br = 256 / cols_cg(mode) * 16;
  return dim3((unsigned)((cols + bc - 1) / bc), (unsigned)((rows + br - 1) / br));
}

hipError_t launch_cols_amax(const float* X, int64_t rows, int64_t cols, int64_t ldx, uint32_t* amax_bits,
                            hipStream_t st) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  hipLaunchKernelGGL(cols_pass_kernel<kColsAmax>, cols_grid(kColsAmax, rows, cols), dim3(256), 0, st, X, rows, cols, ldx,
                     0.f, 0, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, amax_bits, nullptr, 0,
                     nullptr, 0, nullptr, 0, nullptr, kAlways);
  return hipGetLastError();
}

hipError_t launch_cols_codes(const float* X, int64_t rows, int64_t cols, int64_t ldx, int qmax, int trunc,
                             const float* scale, const float* lambda, int8_t* Qvm, int64_t ldvm, int8_t* Qem,
                             int64_t ldem, uint32_t* ramax_bits, hipStream_t st) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  hipLaunchKernelGGL(cols_pass_kernel<kColsCodes>, cols_grid(kColsCodes, rows, cols), dim3(256), 0, st, X, rows, cols, ldx,
                     (float)qmax, trunc, scale, lambda, nullptr, nullptr, nullptr, nullptr, nullptr, ramax_bits,
                     Qvm, ldvm, Qem, ldem, nullptr, 0, nullptr, kAlways);
  return hipGetLastError();
}

// the same pass with the scales derived in the kernel from the column maxima of launch_cols_amax
hipError_t launch_cols_codes_from_amax(const float* X, int64_t rows, int64_t cols, int64_t ldx, int qmax,
                                       int trunc, const uint32_t* amax_bits, float* scale, float* lambda,
                                       int8_t* Qvm, int64_t ldvm, uint32_t* ramax_bits, hipStream_t st) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  hipLaunchKernelGGL(cols_pass_kernel<kColsCodes>, cols_grid(kColsCodes, rows, cols), dim3(256), 0, st, X, rows, cols, ldx,
                     (float)qmax, trunc, nullptr, nullptr, nullptr, amax_bits, scale, lambda, nullptr,
                     ramax_bits, Qvm, ldvm, nullptr, 0, nullptr, 0, nullptr, kAlways);
  return hipGetLastError();
}

// residual codes with the residual scales derived in the kernel from the maxima the codes pass left
hipError_t launch_cols_resid_from_amax(const float* X, int64_t rows, int64_t cols, int64_t ldx, int qmax,
                                       int trunc, const float* scale, const float* lambda,
                                       const uint32_t* ramax_bits, float* rscale, float* rlambda, int8_t* Rvm,
                                       int64_t ldvm, int8_t* Rem, int64_t ldem, hipStream_t st) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  hipLaunchKernelGGL(cols_pass_kernel<kColsResid>, cols_grid(kColsResid, rows, cols), dim3(256), 0, st, X, rows, cols, ldx,
                     (float)qmax, trunc, scale, lambda, nullptr, ramax_bits, rscale, rlambda, nullptr, nullptr,
                     Rvm, ldvm, Rem, ldem, nullptr, 0, nullptr, kAlways);
  return hipGetLastError();
}

hipError_t launch_cols_resid(const float* X, int64_t rows, int64_t cols, int64_t ldx, int qmax, int trunc,
                             const float* scale, const float* lambda, const float* rlambda, int8_t* Rvm,
                             int64_t ldvm, int8_t* Rem, int64_t ldem, hipStream_t st, RunIf run) {
  if (rows <= 0 || cols <= 0 || (!Rvm && !Rem)) return hipSuccess;
  hipLaunchKernelGGL(cols_pass_kernel<kColsResid>, cols_grid(kColsResid, rows, cols), dim3(256), 0, st, X, rows, cols, ldx,
                     (float)qmax, trunc, scale, lambda, rlambda, nullptr, nullptr, nullptr, nullptr, nullptr, Rvm,
                     ldvm, Rem, ldem, nullptr, 0, nullptr, run);
  return hipGetLastError();
}

// counts[cols] must be zero on entry; mask holds mask_words(rows) 64-bit words per column
hipError_t launch_cols_mask(const float* X, int64_t rows, int64_t cols, int64_t ldx, const float* thresh,
                            uint64_t* mask, int32_t* counts, hipStream_t st) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  hipLaunchKernelGGL(cols_pass_kernel<kColsMask>, cols_grid(kColsMask, rows, cols), dim3(256), 0, st, X, rows, cols, ldx,
                     0.f, 0, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, thresh, nullptr, nullptr, 0,
                     nullptr, 0, reinterpret_cast<uint8_t*>(mask), mask_words(rows) * 8, counts, kAlways);
  return hipGetLastError();
}

// selection pass that also writes the residual codes (scales derived as in launch_cols_resid_from_amax)
hipError_t launch_cols_mask_resid(const float* X, int64_t rows, int64_t cols, int64_t ldx, int qmax, int trunc,
                                  const float* scale, const float* lambda, const uint32_t* ramax_bits,
                                  float* rscale, float* rlambda, int8_t* Rvm, int64_t ldvm, int8_t* Rem,
                                  int64_t ldem, const float* thresh, uint64_t* mask, int32_t* counts,
                                  hipStream_t st) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  hipLaunchKernelGGL(cols_pass_kernel<kColsMaskResid>, cols_grid(kColsMaskResid, rows, cols), dim3(256), 0, st, X, rows, cols,
                     ldx, (float)qmax, trunc, scale, lambda, nullptr, ramax_bits, rscale, rlambda, thresh, nullptr,
                     Rvm, ldvm, Rem, ldem, reinterpret_cast<uint8_t*>(mask), mask_words(rows) * 8, counts, kAlways);
  return hipGetLastError();
}

hipError_t launch_rows_mask(const float* X, int64_t rows, int64_t cols, int64_t ldx, const float* thresh,
                            uint64_t* mask, int32_t* counts, hipStream_t st) {
  if (rows <= 0) return hipSuccess;
  const int64_t words = mask_words(cols);
  dim3 grid((unsigned)rows), block(256);
  if (cols > 0 && cols <= 16384 && (cols % 4) == 0 && (ldx % 4) == 0 && aligned16(X)) {
    uint8_t* mb = reinterpret_cast<uint8_t*>(mask);
#define SRQ_MASK(NV4)                                                                                     \
  hipLaunchKernelGGL(rows_mask_vec_kernel<NV4>, grid, block, 0, st, X, cols, ldx, thresh, mb, words * 8, counts)
    // the last word of a row is written in full only when cols is a multiple of 64; otherwise
    // the generic kernel, which writes whole words, is used
    if ((cols % 64) == 0) {
      if (cols <= 1024) SRQ_MASK(1);
      else if (cols <= 2048) SRQ_MASK(2);
      else if (cols <= 4096) SRQ_MASK(4);
      else if (cols <= 8192) SRQ_MASK(8);
      else SRQ_MASK(16);
      return hipGetLastError();
    }
#undef SRQ_MASK
  }
  hipLaunchKernelGGL(rows_mask_kernel, grid, block, 0, st, X, cols, ldx, thresh, mask, words, counts);
  return hipGetLastError();
}

hipError_t launch_scatter_mask(const uint64_t* mask, int64_t nvec, int64_t veclen, const int8_t* Q, int64_t ldq,
                               const int32_t* ptr, int32_t* idx, int8_t* val, int64_t capacity, int8_t* dense,
                               int64_t ldd, int64_t nnz_hint, hipStream_t st, RunIf dense_if) {
  if (nvec <= 0 || veclen <= 0) return hipSuccess;
  // measured at 8192 x 8192: skipping empty chunks pays below about one kept entry per 512
  const bool sparse = !dense && nnz_hint >= 0 && (double)nnz_hint * 512.0 < (double)nvec * (double)veclen;
  // long aligned vectors: sixteen elements per lane (unless the operand is known to keep more
  // than a third of its entries: there the per-entry stores of neighbouring lanes lie far apart
  // and the four-per-lane kernel is faster, 0.36 against 0.45 ms of selection at 8192^2, 50 %)
  const bool crowded = nnz_hint >= 0 && (double)nnz_hint * 3.0 > (double)nvec * (double)veclen;
  if (!crowded && veclen >= 4096 && aligned16(Q) && (ldq % 16) == 0 && (!dense || (aligned16(dense) && (ldd % 16) == 0))) {
    if (sparse)
      hipLaunchKernelGGL(scatter_mask16_kernel<true>, dim3((unsigned)nvec), dim3(256), 0, st, mask,
                         mask_words(veclen), veclen, Q, ldq, ptr, idx, val, capacity, dense, ldd, dense_if);
    else
      hipLaunchKernelGGL(scatter_mask16_kernel<false>, dim3((unsigned)nvec), dim3(256), 0, st, mask,
                         mask_words(veclen), veclen, Q, ldq, ptr, idx, val, capacity, dense, ldd, dense_if);
    return hipGetLastError();
  }
  if (sparse) {
    hipLaunchKernelGGL(scatter_mask_kernel<true>, dim3((unsigned)nvec), dim3(256), 0, st, mask,
                       mask_words(veclen), veclen, Q, ldq, ptr, idx, val, capacity, dense, ldd, dense_if);
  } else {
    hipLaunchKernelGGL(scatter_mask_kernel<false>, dim3((unsigned)nvec), dim3(256), 0, st, mask,
                       mask_words(veclen), veclen, Q, ldq, ptr, idx, val, capacity, dense, ldd, dense_if);
  }
  return hipGetLastError();
}

hipError_t launch_scan_pair(const int32_t* t0, int64_t n0, int32_t* p0, int64_t* z0, const int32_t* t1,
                            int64_t n1, int32_t* p1, int64_t* z1, hipStream_t st, const ScanDecision* decide) {
  ScanDecision dec;
  memset(&dec, 0, sizeof(dec));
  if (decide) dec = *decide;
  hipLaunchKernelGGL(scan_pair_kernel, dim3(dec.paths ? 1 : 2), dim3(1024), 0, st, t0, n0, p0, z0, t1, n1, p1, z1,
                     dec);
  return hipGetLastError();
}

}  // namespace srq
