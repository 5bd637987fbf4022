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
                                                       const int32_t* __restrict__ ptr_end,
                                                       const int32_t* __restrict__ idx,
                                                       const int8_t* __restrict__ val, int64_t capacity,
                                                       const int8_t* __restrict__ R, int64_t ldr,
                                                       GemmEpilogue ep, const uint32_t* __restrict__ kflag) {
  if (guard_tripped(ep)) return;
  const int64_t v = blockIdx.y;
  const int64_t e0 = (int64_t)blockIdx.x * kBlockElems + threadIdx.x * kLaneElems;
  int64_t p0 = ptr[v], p1 = ptr_end[v];
  if (p1 > capacity) p1 = capacity;
  int acc[kLaneElems] = {0, 0, 0, 0};
  const bool full = e0 + kLaneElems <= nelem;
  const bool vec = full && (((reinterpret_cast<uintptr_t>(R) | (uintptr_t)ldr) & 3) == 0);
  if (e0 < nelem) {
    for (int64_t p = p0; p < p1; ++p) {
      const int a = val[p];
      const int32_t k = idx[p];
      if (kflag && ((kflag[k >> 5] >> (k & 31)) & 1u)) continue;   // this k belongs to the dense strip
      const int8_t* src = R + (int64_t)k * ldr + e0;
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
      if (ep.D_int) ep.D_int[i * ep.ldd + j] = acc[t] + (ep.dint_add ? ep.D_int[i * ep.ldd + j] : 0);
      float out = ep.C[i * ep.ldc + j] + d;
      if (ep.final_scale) {
        out = ep.alpha * out;
        if (ep.beta != 0.f) out = out + ep.beta * ep.Cin[i * ep.ldcin + j];
      }
      ep.C[i * ep.ldc + j] = out;
    }
  }
}


// ------------------------------------------------------------------------------------------
// Tiled kernel for aligned operands.  A workgroup of four waves owns 32 vectors x E = 64*LE
// elements; a wave walks its eight vectors one after the other, each lane holding LE
// consecutive elements.  The (index, value) pairs of a vector are fetched 64 at a time, one
// pair per lane, and broadcast through the scalar unit, so that the row of residual codes
// is addressed from scalar registers and the stored value is a scalar operand of the dot
// instruction: v_dot4c(word, value << 8t) adds value * byte t of the word, one multiply-add
// per lane and instruction with no unpacking.  Workgroup ids are dealt round-robin to the
// eight XCDs, so an XCD keeps to the element chunks {x, x+8, ...}: the K x E slab of codes it
// gathers from stays in its own L2 while it sweeps all vectors of the chunk.
// side 1 stages the 32 x E integers in LDS and adds them to C transposed, 32 consecutive
// columns (128 bytes) per row.
constexpr int kVecPerBlock = 32;
constexpr int kVecPerWave = 8;
constexpr int kPairUnroll = 8;

typedef int word1_t;
typedef int word2_t __attribute__((ext_vector_type(2)));
typedef int word4_t __attribute__((ext_vector_type(4)));
template <int LE> struct LaneWords;
template <> struct LaneWords<4> { typedef word1_t type; };
template <> struct LaneWords<8> { typedef word2_t type; };
template <> struct LaneWords<16> { typedef word4_t type; };

// Gather loads go through a buffer descriptor of the whole code matrix: the descriptor and
// the row's byte offset sit in scalar registers and the lane's own offset in one vector
// register, so no 64-bit vector address is built per pair.
typedef unsigned uword2_t __attribute__((ext_vector_type(2)));
typedef unsigned uword4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void gather(word1_t& x, __amdgpu_buffer_rsrc_t rs, uint32_t row, uint32_t off) {
  x = (int)__builtin_amdgcn_raw_buffer_load_b32(rs, off, row, 0);
}
__device__ __forceinline__ void gather(word2_t& x, __amdgpu_buffer_rsrc_t rs, uint32_t row, uint32_t off) {
  uword2_t t = __builtin_amdgcn_raw_buffer_load_b64(rs, off, row, 0);
  x.x = (int)t.x; x.y = (int)t.y;
}
__device__ __forceinline__ void gather(word4_t& x, __amdgpu_buffer_rsrc_t rs, uint32_t row, uint32_t off) {
  uword4_t t = __builtin_amdgcn_raw_buffer_load_b128(rs, off, row, 0);
  x.x = (int)t.x; x.y = (int)t.y; x.z = (int)t.z; x.w = (int)t.w;
}
__device__ __forceinline__ int word_of(word1_t x, int) { return x; }
__device__ __forceinline__ int word_of(word2_t x, int i) { return i == 0 ? x.x : x.y; }
__device__ __forceinline__ int word_of(word4_t x, int i) { return i == 0 ? x.x : i == 1 ? x.y : i == 2 ? x.z : x.w; }

// FILTER: entries whose index is flagged in `kflag` (a bitmap over k) are skipped; the 64 pairs a
// wave fetches at a time are then walked through the ballot of the kept ones instead of lane by lane.
template <int SIDE, int LE, bool FILTER>
__global__ __launch_bounds__(256) void spmm_tile_kernel(int64_t nvec, int64_t nelem,
                                                        const int32_t* __restrict__ ptr,
                                                        const int32_t* __restrict__ ptr_end,
                                                        const int32_t* __restrict__ idx,
                                                        const int8_t* __restrict__ val, int64_t capacity,
                                                        const int8_t* __restrict__ R, int64_t ldr,
                                                        GemmEpilogue ep, int nvb, int nch, bool cvec,
                                                        const uint32_t* __restrict__ kflag) {
  constexpr int E = 64 * LE;
  constexpr int LDT = E + 1;                       // LDS row stride in words (side 1)
  extern __shared__ int tile[];
  const int id = blockIdx.x;
  const int local = id >> 3;
  const int chunk = (local / nvb) * 8 + (id & 7);
  const int vb = local % nvb;
  if (chunk >= nch || guard_tripped(ep)) return;
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t e0 = (int64_t)chunk * E + lane * LE;
  const bool lane_in = e0 < nelem;                 // nelem is a multiple of LE
  const uint32_t eoff = lane_in ? (uint32_t)e0 : 0u;   // lanes past the end gather from column 0 and store nothing

  // first and one-past-last pair of the wave's eight vectors, one vector per lane (for plain
  // CSR the end of a vector is the start of the next: ptr_end = ptr + 1)
  const int64_t v0 = (int64_t)vb * kVecPerBlock + w * kVecPerWave;
  int pl = 0, pe = 0;
  if (lane < kVecPerWave && v0 + lane < nvec) {
    const int64_t pp = ptr[v0 + lane], qq = ptr_end[v0 + lane];
    pl = (int)(pp < capacity ? pp : capacity);
    pe = (int)(qq < capacity ? qq : capacity);
  }
  typedef typename LaneWords<LE>::type words_t;
  // raw buffer over the code matrix; the caller guarantees K * ldr < 2^32
  const __amdgpu_buffer_rsrc_t rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t*>(R), 0, 0xffffffff, 0x00020000);

  for (int q = 0; q < kVecPerWave; ++q) {
    const int64_t v = v0 + q;                        // wave-uniform
    int acc[LE];
#pragma unroll
    for (int t = 0; t < LE; ++t) acc[t] = 0;
    if (v < nvec) {
      const int p0 = __builtin_amdgcn_readlane(pl, q), p1 = __builtin_amdgcn_readlane(pe, q);
      for (int pb = p0; pb < p1; pb += 64) {
        const int cnt = p1 - pb < 64 ? p1 - pb : 64;
        uint32_t ro = 0;                             // padding pairs: value 0 times row 0
        int aa = 0;
        bool kept = false;
        if (lane < cnt) {
          const uint32_t k = (uint32_t)idx[pb + lane];
          ro = k * (uint32_t)ldr;
          aa = val[pb + lane];
          kept = !FILTER || !((kflag[k >> 5] >> (k & 31)) & 1u);
        }
        // FILTER: the lanes holding pairs that are not part of the dense strip, walked in order by
        // two cursors (one for the gathers being issued, one for those being consumed)
        unsigned long long m_issue = FILTER ? __ballot(kept) : 0ull, m_use = m_issue;
        const int npairs = FILTER ? __popcll(m_issue) : cnt;
        const int ng = (npairs + kPairUnroll - 1) / kPairUnroll;
        words_t xa[kPairUnroll], xb[kPairUnroll];
        auto issue = [&](words_t (&x)[kPairUnroll], int g) {
#pragma unroll
          for (int u = 0; u < kPairUnroll; ++u) {
            uint32_t r;
            if (FILTER) {
              const int l = m_issue ? __builtin_ctzll(m_issue) : 0;
              r = m_issue ? __builtin_amdgcn_readlane(ro, l) : 0u;
              m_issue &= m_issue - 1ull;
            } else {
              r = __builtin_amdgcn_readlane(ro, g * kPairUnroll + u);   // row offset in bytes, < 2^32
            }
            gather(x[u], rsrc, r, eoff);
          }
        };
        auto consume = [&](words_t (&x)[kPairUnroll], int g) {
#pragma unroll
          for (int u = 0; u < kPairUnroll; ++u) {
            int a;
            if (FILTER) {
              const int l = m_use ? __builtin_ctzll(m_use) : 0;
              a = m_use ? (__builtin_amdgcn_readlane(aa, l) & 0xff) : 0;
              m_use &= m_use - 1ull;
            } else {
              a = __builtin_amdgcn_readlane(aa, g * kPairUnroll + u) & 0xff;
            }
#pragma unroll
            for (int t = 0; t < LE; ++t)
              acc[t] = __builtin_amdgcn_sdot4(word_of(x[u], t >> 2), a << (8 * (t & 3)), acc[t], false);
          }
        };
        // two groups of eight gathers in flight: one being consumed, one on its way
        issue(xa, 0);
        for (int g = 0; g < ng; g += 2) {
          if (g + 1 < ng) issue(xb, g + 1);
          consume(xa, g);
          if (g + 1 < ng) {
            if (g + 2 < ng) issue(xa, g + 2);
            consume(xb, g + 1);
          }
        }
      }
    }
    if (SIDE == 1) {
      int* dst = tile + (w * kVecPerWave + q) * LDT + lane * LE;
#pragma unroll
      for (int t = 0; t < LE; ++t) dst[t] = acc[t];
    } else if (v < nvec && lane_in &&
               (ep.final_scale || ep.D_int ||
                __builtin_amdgcn_readlane(pl, q) < __builtin_amdgcn_readlane(pe, q))) {
      // (a row without kept entries leaves C as it is unless this pass also applies alpha / beta)
      const float sr = ep.s_row[v];
      float* c = ep.C + v * ep.ldc + e0;
      if (cvec) {                                    // 16-byte accesses: C, s_col (and Cin) are aligned
#pragma unroll
        for (int t = 0; t < LE; t += 4) {
          const float4 sc = *reinterpret_cast<const float4*>(ep.s_col + e0 + t);
          float4 o = *reinterpret_cast<const float4*>(c + t);
          o.x = o.x + (float)acc[t] * (sr * sc.x);
          o.y = o.y + (float)acc[t + 1] * (sr * sc.y);
          o.z = o.z + (float)acc[t + 2] * (sr * sc.z);
          o.w = o.w + (float)acc[t + 3] * (sr * sc.w);
          if (ep.final_scale) {
            o.x = ep.alpha * o.x; o.y = ep.alpha * o.y; o.z = ep.alpha * o.z; o.w = ep.alpha * o.w;
            if (ep.beta != 0.f) {
              const float4 ci = *reinterpret_cast<const float4*>(ep.Cin + v * ep.ldcin + e0 + t);
              o.x = o.x + ep.beta * ci.x; o.y = o.y + ep.beta * ci.y;
              o.z = o.z + ep.beta * ci.z; o.w = o.w + ep.beta * ci.w;
            }
          }
          *reinterpret_cast<float4*>(c + t) = o;
        }
      } else {
#pragma unroll
        for (int t = 0; t < LE; ++t) {
          const float d = (float)acc[t] * (sr * ep.s_col[e0 + t]);
          if (ep.D_int) ep.D_int[v * ep.ldd + e0 + t] = acc[t] + (ep.dint_add ? ep.D_int[v * ep.ldd + e0 + t] : 0);
          float out = c[t] + d;
          if (ep.final_scale) {
            out = ep.alpha * out;
            if (ep.beta != 0.f) out = out + ep.beta * ep.Cin[v * ep.ldcin + e0 + t];
          }
          c[t] = out;
        }
      }
    }
  }
  if (SIDE == 1) {
    __syncthreads();
    const int64_t j0 = (int64_t)vb * kVecPerBlock;
    // fast form: the 32 columns of the block exist and rows of C are 16-byte aligned, so a thread
    // adds to four consecutive columns of one row at a time (eight threads per 128-byte segment)
    if (cvec && j0 + kVecPerBlock <= nvec) {
      const int q = threadIdx.x & 7;                     // which four columns
      const float4 sc4 = *reinterpret_cast<const float4*>(ep.s_col + j0 + 4 * q);
      const int* t0 = tile + (4 * q) * LDT;
#pragma unroll 4
      for (int e = threadIdx.x >> 3; e < E; e += 32) {
        const int64_t i = (int64_t)chunk * E + e;
        if (i >= nelem) continue;
        const float sr = ep.s_row[i];
        float* c = ep.C + i * ep.ldc + j0 + 4 * q;
        float4 o = *reinterpret_cast<const float4*>(c);
        o.x = o.x + (float)t0[e] * (sr * sc4.x);
        o.y = o.y + (float)t0[LDT + e] * (sr * sc4.y);
        o.z = o.z + (float)t0[2 * LDT + e] * (sr * sc4.z);
        o.w = o.w + (float)t0[3 * LDT + e] * (sr * sc4.w);
        if (ep.final_scale) {
          o.x = ep.alpha * o.x; o.y = ep.alpha * o.y; o.z = ep.alpha * o.z; o.w = ep.alpha * o.w;
          if (ep.beta != 0.f) {
            const float4 ci = *reinterpret_cast<const float4*>(ep.Cin + i * ep.ldcin + j0 + 4 * q);
            o.x = o.x + ep.beta * ci.x; o.y = o.y + ep.beta * ci.y;
            o.z = o.z + ep.beta * ci.z; o.w = o.w + ep.beta * ci.w;
          }
        }
        *reinterpret_cast<float4*>(c) = o;
      }
      return;
    }
    const int j = threadIdx.x & 31;                      // column of C inside the block of 32
    const int64_t jj = j0 + j;
    const float sc = jj < nvec ? ep.s_col[jj] : 0.f;
#pragma unroll 8
    for (int e = threadIdx.x >> 5; e < E; e += 8) {
      const int64_t i = (int64_t)chunk * E + e;
      if (i >= nelem || jj >= nvec) continue;
      const int a = tile[j * LDT + e];
      const float d = (float)a * (ep.s_row[i] * sc);
      if (ep.D_int) ep.D_int[i * ep.ldd + jj] = a + (ep.dint_add ? ep.D_int[i * ep.ldd + jj] : 0);
      float out = ep.C[i * ep.ldc + jj] + d;
      if (ep.final_scale) {
        out = ep.alpha * out;
        if (ep.beta != 0.f) out = out + ep.beta * ep.Cin[i * ep.ldcin + jj];
      }
      ep.C[i * ep.ldc + jj] = out;
    }
  }
}

template <int SIDE, int LE>
hipError_t launch_tile(int64_t nvec, int64_t nelem, const int32_t* ptr, const int32_t* ptr_end, const int32_t* idx,
                       const int8_t* val, int64_t capacity, const int8_t* R, int64_t ldr,
                       const GemmEpilogue& ep, const uint32_t* kflag, hipStream_t st) {
  constexpr int E = 64 * LE;
  const int64_t nvb = (nvec + kVecPerBlock - 1) / kVecPerBlock;
  const int64_t nch = (nelem + E - 1) / E;
  const int64_t blocks = (nch + 7) / 8 * 8 * nvb;
  // side 0 adds to C with 16-byte accesses when every row segment of a lane is aligned
  const bool cvec = !ep.D_int && (reinterpret_cast<uintptr_t>(ep.C) & 15) == 0 && ep.ldc % 4 == 0 &&
                    (reinterpret_cast<uintptr_t>(ep.s_col) & 15) == 0 &&
                    (!ep.Cin || ((reinterpret_cast<uintptr_t>(ep.Cin) & 15) == 0 && ep.ldcin % 4 == 0));
  const size_t lds = SIDE == 1 ? (size_t)kVecPerBlock * (E + 1) * sizeof(int) : 0;
  if (kflag)
    hipLaunchKernelGGL((spmm_tile_kernel<SIDE, LE, true>), dim3((unsigned)blocks), dim3(256), lds, st, nvec, nelem,
                       ptr, ptr_end, idx, val, capacity, R, ldr, ep, (int)nvb, (int)nch, cvec, kflag);
  else
    hipLaunchKernelGGL((spmm_tile_kernel<SIDE, LE, false>), dim3((unsigned)blocks), dim3(256), lds, st, nvec, nelem,
                       ptr, ptr_end, idx, val, capacity, R, ldr, ep, (int)nvb, (int)nch, cvec, kflag);
  return hipGetLastError();
}

// the tiled kernel reads whole aligned lane words and never a partial one
bool tile_ok(int64_t nvec, int64_t nelem, int64_t K, const int8_t* R, int64_t ldr, int le) {
  const int64_t nvb = (nvec + kVecPerBlock - 1) / kVecPerBlock;
  const int64_t nch = (nelem + 64 * le - 1) / (64 * le);
  return nelem % le == 0 && ldr % le == 0 && (reinterpret_cast<uintptr_t>(R) % le) == 0 &&
         nelem < (1LL << 31) && K * ldr < (1LL << 32) && (nch + 7) / 8 * 8 * nvb < (1LL << 31) && nvb < (1LL << 31);
}

}  // namespace

hipError_t launch_spmm_valu(int side, int64_t nvec, int64_t nelem, int64_t K, const int32_t* ptr,
                            const int32_t* ptr_end, const int32_t* idx, const int8_t* val, int64_t capacity,
                            const int8_t* R, int64_t ldr, const GemmEpilogue& ep, hipStream_t st,
                            const uint32_t* kflag) {
  if (nvec <= 0 || nelem <= 0) return hipSuccess;
  if (!ptr_end) ptr_end = ptr + 1;                 // plain CSR / CSC
  if (side == 0 && tile_ok(nvec, nelem, K, R, ldr, 8))
    return launch_tile<0, 8>(nvec, nelem, ptr, ptr_end, idx, val, capacity, R, ldr, ep, kflag, st);
  if (side == 1 && tile_ok(nvec, nelem, K, R, ldr, 4))
    return launch_tile<1, 4>(nvec, nelem, ptr, ptr_end, idx, val, capacity, R, ldr, ep, kflag, st);
  const int64_t kMaxY = 65535;
  for (int64_t v0 = 0; v0 < nvec; v0 += kMaxY) {   // gridDim.y is limited to 65535
    int64_t nv = nvec - v0 < kMaxY ? nvec - v0 : kMaxY;
    GemmEpilogue e2 = ep;
    const int32_t* p2 = ptr + v0;
    const int32_t* q2 = ptr_end + v0;
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
      hipLaunchKernelGGL(spmm_valu_kernel<0>, grid, dim3(64), 0, st, nv, nelem, p2, q2, idx, val, capacity, R,
                         ldr, e2, kflag);
    else
      hipLaunchKernelGGL(spmm_valu_kernel<1>, grid, dim3(64), 0, st, nv, nelem, p2, q2, idx, val, capacity, R,
                         ldr, e2, kflag);
  }
  return hipGetLastError();
}

}  // namespace srq
