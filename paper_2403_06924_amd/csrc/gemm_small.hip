// INT8 GEMM for aligned problems too small to give every compute unit a 256 x 256 tile (M, N
// multiples of 128, K a multiple of 128, 16-byte aligned operands): the products of Algorithm 1
// lines 2, 12 and 14 at sizes like 1024^3 .. 3072^3, where the time of a product is a chain of
// memory latencies rather than matrix-core throughput.
//
// One 128 x 128 output tile per 4-wave workgroup (64 x 64 per wave, v_mfma_i32_32x32x32_i8), K
// staged 128 bytes at a time as in the persistent kernel - global memory straight into LDS,
// unpadded rows, XOR swizzle of the 16-byte pieces - but through a ring of FOUR 32 KiB stages:
// the loads of K-tile g+3 are issued while K-tile g is multiplied, so three K-tiles (48 MFMAs
// per wave) are in flight to cover the latency of a load that comes from HBM.  With one stage in
// flight, as in the generic kernel, every K-tile of a 2048^3 product waits a full round trip.
//
// Epilogues as in the persistent kernel (dequantisation, partial sums of |D_F| per 128 columns /
// rows, accumulate mode, alpha / beta, a second product of the same tile in one launch).
#include <type_traits>
#include "srq_internal.h"
#include "gemm_tiles.h"

namespace srq {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BN = 128, BK = 128, KS = BK / 32, NST = 4;
constexpr int kOperand = BM * BK;                   // 16 KiB per operand tile
constexpr int kStage = 2 * kOperand;                // A tile then B tile
constexpr int TM = 2, TN = 2;                       // 32x32 MFMA tiles per wave
constexpr int kLdsScales = NST * kStage;            // float[BM + BN]
constexpr int kLdsRowX = kLdsScales + (BM + BN) * 4;   // float[2][BM]: row partials of the two wave columns
constexpr int kLdsColX = kLdsRowX + 2 * BM * 4;        // double[2][BN]: column partials of the two wave rows
constexpr int kLdsBytes = kLdsColX + 2 * BN * 8;
constexpr int kLoadsPerTile = 8;                    // per wave and K-tile: 4 for A, 4 for B

template <int MODE, bool SUMS, bool SCALE>
__global__ __launch_bounds__(256) void gemm_i8_small_kernel(int64_t M, int64_t N, int64_t K,
                                                            const int8_t* __restrict__ Qa, int64_t lda,
                                                            const int8_t* __restrict__ Qb, int64_t ldb,
                                                            int64_t tiles_m, int64_t tiles_n, GemmEpilogue ep,
                                                            GemmSecond sec) {
  extern __shared__ __attribute__((aligned(1024))) int8_t lds[];
  if (MODE == kGemmAccum && guard_tripped(ep)) return;   // the whole grid leaves together
  float* sc_row = reinterpret_cast<float*>(lds + kLdsScales);
  float* sc_col = sc_row + BM;
  float* xrow = reinterpret_cast<float*>(lds + kLdsRowX);
  double* xcol = reinterpret_cast<double*>(lds + kLdsColX);
  const uint32_t lds0 = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) int8_t*)lds);

  const int tid = threadIdx.x;
  const int lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6), wm = w >> 1, wn = w & 1;
  const int64_t nk = K / BK;
  const int nprod = (MODE == kGemmAccum && sec.Qa) ? 2 : 1;
  int p_lo, p_hi;                                   // the products this launch runs (device-side decision)
  pair_range(ep, nprod, p_lo, p_hi);
  const bool two = p_lo != p_hi;
  int64_t tile_m, tile_n;
  tile_of(blockIdx.x, tiles_m, tiles_n, tile_m, tile_n);
  const int64_t m0 = tile_m * BM, n0 = tile_n * BN;

  // ---- loader: wave w fetches rows 32w .. 32w+31 of each operand tile, eight rows per load.
  // Lane l of load j covers row 32w + 8j + l/8 and LDS piece l%8, which holds the logical piece
  // (l%8) ^ ((row >> 1) & 7); (row >> 1) & 7 = ((l >> 4) + 4j) & 7 depends on j only through
  // its parity.
  const int lrow = lane >> 3;
  int64_t kta = 0;                                  // cursor of the K-tile being fetched
  int proda = p_lo;                                 // ... and the product it belongs to
  const int8_t *pa, *pb;                            // row 32w of that K-tile in A and in B
  int64_t cur_lda = lda, cur_ldb = ldb;
  int64_t goff_a0 = 0, goff_a1 = 0, goff_b0 = 0, goff_b1 = 0;
  auto point = [&]() {
    const int8_t* A0 = proda ? sec.Qa : Qa;
    const int8_t* B0 = proda ? sec.Qb : Qb;
    cur_lda = proda ? sec.lda : lda;
    cur_ldb = proda ? sec.ldb : ldb;
    goff_a0 = (int64_t)lrow * cur_lda + 16 * ((lane & 7) ^ ((lane >> 4) & 7));
    goff_a1 = (int64_t)lrow * cur_lda + 16 * ((lane & 7) ^ (((lane >> 4) + 4) & 7));
    goff_b0 = (int64_t)lrow * cur_ldb + 16 * ((lane & 7) ^ ((lane >> 4) & 7));
    goff_b1 = (int64_t)lrow * cur_ldb + 16 * ((lane & 7) ^ (((lane >> 4) + 4) & 7));
    pa = A0 + (m0 + 32 * w) * cur_lda + kta * BK;
    pb = B0 + (n0 + 32 * w) * cur_ldb + kta * BK;
  };
  auto advance = [&]() {
    if (kta + 1 < nk) {
      ++kta;
      pa += BK;
      pb += BK;
    } else if (proda < p_hi) {
      ++proda;
      kta = 0;
      point();
    }                                               // else stay on the last K-tile (harmless re-fetch)
  };
  // load i (0..7) of the K-tile at the cursor into LDS buffer `stage`: even i -> A, odd i -> B
  auto issue_load = [&](int stage, int i) {
    const uint32_t la = __builtin_amdgcn_readfirstlane(lds0 + stage * kStage + (32 * w) * BK);
    const int j = i >> 1;
    if (i & 1)
      load_to_lds(pb + (int64_t)(8 * j) * cur_ldb + ((j & 1) ? goff_b1 : goff_b0), la + kOperand + j * 8 * BK);
    else
      load_to_lds(pa + (int64_t)(8 * j) * cur_lda + ((j & 1) ? goff_a1 : goff_a0), la + j * 8 * BK);
  };
  auto issue_loads = [&](int stage) {
#pragma unroll
    for (int i = 0; i < kLoadsPerTile; ++i) issue_load(stage, i);
  };

  // ---- fragment reads: lane (frow, kh) reads logical piece 2*step + kh of its rows
  const int frow = lane & 31, kh = lane >> 5, key = (frow >> 1) & 7;
  const int a_row = (wm * (BM / 2) + frow) * BK;
  const int b_row = kOperand + (wn * (BN / 2) + frow) * BK;
  int xoff[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s) xoff[s] = 16 * ((2 * s + kh) ^ key);
  v4i fa[2][TM], fb[2][TN];
  auto fread = [&](int stage, int step, int slot) {
    const int8_t* As = lds + stage * kStage + a_row + xoff[step];
    const int8_t* Bs = lds + stage * kStage + b_row + xoff[step];
#pragma unroll
    for (int t = 0; t < TM; ++t) fa[slot][t] = *reinterpret_cast<const v4i*>(As + t * 32 * BK);
#pragma unroll
    for (int t = 0; t < TN; ++t) fb[slot][t] = *reinterpret_cast<const v4i*>(Bs + t * 32 * BK);
  };

  // read r of a step's four fragment reads: 0, 1 -> A tiles, 2, 3 -> B tiles
  auto fread1 = [&](int stage, int step, int slot, int r) {
    if (r < TM)
      fa[slot][r] = *reinterpret_cast<const v4i*>(lds + stage * kStage + a_row + xoff[step] + r * 32 * BK);
    else
      fb[slot][r - TM] = *reinterpret_cast<const v4i*>(lds + stage * kStage + b_row + xoff[step] + (r - TM) * 32 * BK);
  };

  // scales of the tile: threads 0..127 hold the row scales, 128..255 the column scales
  float sreg = tid < BM ? (p_lo ? sec.s_row : ep.s_row)[m0 + tid] : (p_lo ? sec.s_col : ep.s_col)[n0 + tid - BM];

  point();
  issue_loads(0);
  advance();
  issue_loads(1);
  advance();
  issue_loads(2);
  advance();
  wait_loads_but<2 * kLoadsPerTile>();              // K-tile 0 has landed
  __syncthreads();
  fread(0, 0, 0);

  v16i acc[TM][TN];
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0;

  int g = 0;                                        // position in the stream of K-tiles (stage = g mod 4)
  for (int prod = p_lo; prod <= p_hi; ++prod) {
    for (int64_t kt = 0; kt < nk; ++kt, ++g) {
      const int cur = g & (NST - 1);
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        if (s == KS - 1) {
          // K-tile g+1 must have landed: everything but the eight loads of K-tile g+2 and the
          // six of K-tile g+3 that this K-tile's earlier steps issued.
          wait_loads_but<2 * kLoadsPerTile - 2>();
          __syncthreads();
          fread((cur + 1) & (NST - 1), 0, (s + 1) & 1);
          __builtin_amdgcn_sched_barrier(0);
        }
        // The stage of K-tile g-1 was handed over by the barrier of that K-tile and takes K-tile
        // g+3: two of its eight loads go out in each step (the CU's vector-memory path takes a
        // 1 KiB load about every 20 clocks; a wave whose load is not accepted yet also holds back
        // the MFMAs behind it).  The fragments of the next step: one read after each MFMA.
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
          for (int b = 0; b < TN; ++b) {
            acc[a][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[s & 1][a], fb[s & 1][b], acc[a][b], 0, 0, 0);
            if (s != KS - 1) fread1(cur, s + 1, (s + 1) & 1, a * TN + b);
            if (b == TN - 1) issue_load((cur + 3) & (NST - 1), 2 * s + a);
            __builtin_amdgcn_sched_barrier(0);
          }
      }
      advance();
    }

    // ================= epilogue; no bounds checks: tiles are full
    __syncthreads();                                // (the exchange areas of a previous product are free)
    sc_row[tid] = sreg;                             // sc_col follows sc_row
    __syncthreads();
    const int half = lane >> 5, cl = lane & 31;
    const int cbase = wn * (BN / 2) + cl;
    double colsum[TN];
    float scol[TN];
#pragma unroll
    for (int b = 0; b < TN; ++b) {
      colsum[b] = 0.0;
      scol[b] = sc_col[cbase + b * 32];
    }
    const bool do_scale = SCALE && prod == nprod - 1;
    const float alpha = SCALE ? ep.alpha : 1.f, beta = SCALE ? ep.beta : 0.f;
    const bool has_beta = SCALE && do_scale && beta != 0.f;
    const int64_t ldcin = SCALE ? ep.ldcin : 0;
    // C goes around the caches, except between the two products of a pair
    auto bands = [&](auto cached_load_tag, auto cached_store_tag) {
      constexpr bool CLOAD = decltype(cached_load_tag)::value, CSTORE = decltype(cached_store_tag)::value;
#pragma unroll
      for (int a = 0; a < TM; ++a) {
        const int rbase = wm * (BM / 2) + a * 32 + 4 * half;
        float* cband = ep.C + (m0 + rbase) * ep.ldc + n0 + cbase;
        float x[TN][16];
        float cin[TN][16];                            // the band of Cin, all loads in flight at once
        if (SCALE && has_beta) {
          const float* cinband = ep.Cin + (m0 + rbase) * ldcin + n0 + cbase;
#pragma unroll
          for (int v = 0; v < 16; ++v)
#pragma unroll
            for (int b = 0; b < TN; ++b)
              cin[b][v] = __builtin_nontemporal_load(&cinband[(int64_t)(8 * (v >> 2) + (v & 3)) * ldcin + b * 32]);
        }
        if (MODE == kGemmAccum) {
#pragma unroll
          for (int v = 0; v < 16; ++v)
#pragma unroll
            for (int b = 0; b < TN; ++b) {
              const float* src = &cband[(int64_t)(8 * (v >> 2) + (v & 3)) * ep.ldc + b * 32];
              x[b][v] = CLOAD ? *src : __builtin_nontemporal_load(src);
            }
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int ro = 8 * (v >> 2) + (v & 3);
          const float srow = sc_row[rbase + ro];
#pragma unroll
          for (int b = 0; b < TN; ++b) {
            const float d = (float)acc[a][b][v] * (srow * scol[b]);
            float out = MODE == kGemmFirst ? d : x[b][v] + d;
            if (SCALE && do_scale) {
              out = alpha * out;
              if (has_beta) out = out + beta * cin[b][v];
            }
            if (CSTORE) cband[(int64_t)ro * ep.ldc + b * 32] = out;
            else __builtin_nontemporal_store(out, &cband[(int64_t)ro * ep.ldc + b * 32]);
            if (SUMS) x[b][v] = fabsf(d);
            acc[a][b][v] = 0;
          }
        }
        if (SUMS) {
          // row sums by a reduce-scatter butterfly over the 32 lanes that share a row
          float r[16];
#pragma unroll
          for (int v = 0; v < 16; ++v) r[v] = x[0][v] + x[1][v];
#pragma unroll
          for (int n = 8, o = 16; n >= 1; n >>= 1, o >>= 1) {
            const bool up = (cl & o) != 0;
#pragma unroll
            for (int i = 0; i < n; ++i) {
              float send = up ? r[i] : r[i + n];
              float keep = up ? r[i + n] : r[i];
              r[i] = keep + __shfl_xor(send, o, 64);
            }
          }
          r[0] += __shfl_xor(r[0], 1, 64);
          const int v = cl >> 1;
          if (!(cl & 1)) xrow[wn * BM + rbase + 8 * (v >> 2) + (v & 3)] = r[0];
#pragma unroll
          for (int b = 0; b < TN; ++b) {
            float t8[8], t4[4];
#pragma unroll
            for (int i = 0; i < 8; ++i) t8[i] = x[b][2 * i] + x[b][2 * i + 1];
#pragma unroll
            for (int i = 0; i < 4; ++i) t4[i] = t8[2 * i] + t8[2 * i + 1];
            colsum[b] += (double)((t4[0] + t4[1]) + (t4[2] + t4[3]));
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    if (two && prod == 0) bands(std::false_type(), std::true_type());
    else if (two) bands(std::true_type(), std::false_type());
    else bands(std::false_type(), std::false_type());
    if (SUMS) {
      // one partial per tile and row / column: the two waves that share it add up through LDS
#pragma unroll
      for (int b = 0; b < TN; ++b) {
        double c = colsum[b];
        c += __shfl_xor(c, 32, 64);
        if (half == 0) xcol[wm * BN + cbase + b * 32] = c;
      }
      __syncthreads();
      if (tid < BM)
        ep.row_part[tile_n * (ep.part_ld_m ? ep.part_ld_m : M) + m0 + tid] = (double)xrow[tid] + (double)xrow[BM + tid];
      else
        ep.col_part[tile_m * (ep.part_ld_n ? ep.part_ld_n : N) + n0 + tid - BM] = xcol[tid - BM] + xcol[BN + tid - BM];
    }
    if (prod < p_hi) sreg = tid < BM ? sec.s_row[m0 + tid] : sec.s_col[n0 + tid - BM];
  }
  wait_loads();                                     // nothing may still be writing LDS when the wave ends
}

}  // namespace

bool gemm_small_ok(int64_t M, int64_t N, int64_t K, const int8_t* Qa, int64_t lda, const int8_t* Qb, int64_t ldb,
                   const GemmEpilogue& ep) {
  if (ep.D_int || ep.D_F_copy) return false;                 // parity-check outputs use the plain kernel
  if (M <= 0 || N <= 0 || K <= 0 || (M % BM) || (N % BN) || (K % BK)) return false;
  if (((reinterpret_cast<uintptr_t>(Qa) | reinterpret_cast<uintptr_t>(Qb)) & 15) || (lda % 16) || (ldb % 16))
    return false;
  // the partial sums of |D_F| are laid out per 128 columns / rows: only where the plain kernel
  // would use tiles of that size as well (the buffers are sized for it)
  return gemm_tiles_m(M, N) == M / BM && gemm_tiles_n(M, N) == N / BN;
}

hipError_t launch_gemm_i8_small(int64_t M, int64_t N, int64_t K, const int8_t* Qa, int64_t lda, const int8_t* Qb,
                                int64_t ldb, const GemmEpilogue& ep, hipStream_t st, const GemmSecond* second) {
  const int64_t tm = M / BM, tn = N / BN;
  const bool sums = ep.mode == kGemmFirst && ep.row_part != nullptr;
  const bool scale = ep.final_scale != 0;
  void (*kern)(int64_t, int64_t, int64_t, const int8_t*, int64_t, const int8_t*, int64_t, int64_t, int64_t,
               GemmEpilogue, GemmSecond);
  GemmSecond sec = {nullptr, nullptr, 0, 0, nullptr, nullptr};
  if (second && ep.mode == kGemmAccum) sec = *second;
  if (ep.mode == kGemmFirst) {
    kern = sums ? (scale ? gemm_i8_small_kernel<kGemmFirst, true, true> : gemm_i8_small_kernel<kGemmFirst, true, false>)
                : (scale ? gemm_i8_small_kernel<kGemmFirst, false, true>
                         : gemm_i8_small_kernel<kGemmFirst, false, false>);
  } else {
    kern = scale ? gemm_i8_small_kernel<kGemmAccum, false, true> : gemm_i8_small_kernel<kGemmAccum, false, false>;
  }
  hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), kLdsBytes);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3((unsigned)(tm * tn)), dim3(256), kLdsBytes, st, M, N, K, Qa, lda, Qb, ldb, tm, tn,
                     ep, sec);
  return hipGetLastError();
}

}  // namespace srq
