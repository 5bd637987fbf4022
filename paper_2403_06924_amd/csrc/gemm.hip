// INT8 x INT8 -> INT32 GEMM on the gfx950 matrix cores with the FP32 dequantization epilogue
// (Algorithm 1 lines 2-3 and, in accumulate mode, lines 12/14 with 16-17).
//
//   D_int[i,j] = sum_k Qa[i*lda + k] * Qb[j*ldb + k]       both operands K-contiguous
//   first mode : C = fl(float(D_int) * fl(s_row[i]*s_col[j])), plus per-tile partial sums
//                of |C| over rows and columns for the averages of Sec. 3.1.1
//   accum mode : C += the same dequantized product
//
// A workgroup of 256 threads (4 waves, 2 x 2) owns a BM x BN tile of the output; each wave
// owns (BM/2) x (BN/2) of it as a grid of 32x32 MFMA tiles (v_mfma_i32_32x32x32_i8, INT32
// accumulators in registers).  Operand tiles of BK bytes along K are staged
// global -> registers -> LDS, double buffered so that the loads of step t+1 are in flight
// while step t is multiplied.  LDS rows are padded by 16 bytes so the 16-byte fragment reads
// of 16 consecutive rows fall on distinct banks.

#include "srq_internal.h"

namespace srq {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// 16 bytes of row `row` starting at byte k.  FAST: the caller guarantees 16-byte alignment
// and k + 16 <= K; rows past the end are clamped (their products are never stored).
// Otherwise bytes are fetched one by one and zero-filled outside [0,K).  No local is
// addressed through a pointer, so everything stays in registers.
template <bool FAST>
__device__ __forceinline__ v4i load16(const int8_t* __restrict__ base, int64_t ld, int64_t row,
                                      int64_t nrows, int64_t k, int64_t K) {
  if (row >= nrows) row = nrows - 1;
  const int8_t* p = base + row * ld + k;
  if (FAST) return *reinterpret_cast<const v4i*>(p);
  v4i out;
#pragma unroll
  for (int wd = 0; wd < 4; ++wd) {
    unsigned u = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int64_t kk = k + wd * 4 + i;
      unsigned byte = kk < K ? (unsigned)(uint8_t)p[wd * 4 + i] : 0u;
      u |= byte << (8 * i);
    }
    out[wd] = (int)u;
  }
  return out;
}

template <int BM, int BN, int BK>
struct Cfg {
  static constexpr int kStride = BK + 16;                 // bytes per LDS row
  static constexpr int kStage = (BM + BN) * kStride;      // bytes per pipeline stage
  static constexpr int kSegs = BK / 16;                   // 16-byte pieces per row
  static constexpr int kPiecesA = BM * kSegs / 256;       // pieces per thread
  static constexpr int kPiecesB = BN * kSegs / 256;
  static constexpr int TM = BM / 64, TN = BN / 64;        // 32x32 MFMA tiles per wave
  static constexpr int kLds = 2 * kStage;
};

template <int BM, int BN, int BK, bool FAST, bool DBG>
__global__ __launch_bounds__(256) void gemm_i8_kernel(int64_t M, int64_t N, int64_t K,
                                                      const int8_t* __restrict__ Qa, int64_t lda,
                                                      const int8_t* __restrict__ Qb, int64_t ldb,
                                                      int64_t tiles_m, int64_t tiles_n,
                                                      GemmEpilogue ep) {
  using C = Cfg<BM, BN, BK>;
  extern __shared__ __attribute__((aligned(16))) int8_t lds[];
  if (guard_tripped(ep)) return;                   // the whole grid leaves together

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int wm = w >> 1, wn = w & 1;

  // Workgroups are handed to the 8 XCDs round-robin; give each XCD a contiguous band of
  // tile rows so that the tiles sharing an L2 also share operand panels.
  int64_t bid = blockIdx.x;
  const int64_t total = tiles_m * tiles_n;
  {
    const int64_t per = total / 8;
    if (per > 0 && bid < per * 8) bid = (bid & 7) * per + (bid >> 3);
  }
  // within the band, walk the tiles in groups of 8 rows (column-major inside a group)
  int64_t tile_m, tile_n;
  {
    const int64_t g = 8;
    int64_t grp = bid / (g * tiles_n);
    int64_t first = grp * g;
    int64_t rows_in = tiles_m - first < g ? tiles_m - first : g;
    int64_t in = bid - grp * g * tiles_n;
    tile_m = first + in % rows_in;
    tile_n = in / rows_in;
  }
  const int64_t m0 = tile_m * BM, n0 = tile_n * BN;

  v16i acc[C::TM][C::TN];
#pragma unroll
  for (int a = 0; a < C::TM; ++a)
#pragma unroll
    for (int b = 0; b < C::TN; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0;

  v4i ra[C::kPiecesA], rb[C::kPiecesB];
  auto gload = [&](int64_t k0) {
#pragma unroll
    for (int s = 0; s < C::kPiecesA; ++s) {
      int p = tid + s * 256;
      int r = p / C::kSegs, seg = (p % C::kSegs) * 16;
      ra[s] = load16<FAST>(Qa, lda, m0 + r, M, k0 + seg, K);
    }
#pragma unroll
    for (int s = 0; s < C::kPiecesB; ++s) {
      int p = tid + s * 256;
      int r = p / C::kSegs, seg = (p % C::kSegs) * 16;
      rb[s] = load16<FAST>(Qb, ldb, n0 + r, N, k0 + seg, K);
    }
  };
  auto lstore = [&](int stage) {
    int8_t* As = lds + stage * C::kStage;
    int8_t* Bs = As + BM * C::kStride;
#pragma unroll
    for (int s = 0; s < C::kPiecesA; ++s) {
      int p = tid + s * 256;
      int r = p / C::kSegs, seg = (p % C::kSegs) * 16;
      *reinterpret_cast<v4i*>(&As[r * C::kStride + seg]) = ra[s];
    }
#pragma unroll
    for (int s = 0; s < C::kPiecesB; ++s) {
      int p = tid + s * 256;
      int r = p / C::kSegs, seg = (p % C::kSegs) * 16;
      *reinterpret_cast<v4i*>(&Bs[r * C::kStride + seg]) = rb[s];
    }
  };

  const int64_t nk = (K + BK - 1) / BK;
  constexpr int KS = BK / 32;                     // MFMA k-steps per staged tile
  const int frow = lane & 31, fk = (lane >> 5) * 16;
  const int a_off = (wm * (BM / 2) + frow) * C::kStride + fk;
  const int b_off = BM * C::kStride + (wn * (BN / 2) + frow) * C::kStride + fk;
  v4i fa[2][C::TM], fb[2][C::TN];                 // fragment double buffer
  auto fread = [&](int stage, int step, int slot) {
    const int8_t* As = lds + stage * C::kStage + a_off + step * 32;
    const int8_t* Bs = lds + stage * C::kStage + b_off + step * 32;
#pragma unroll
    for (int t = 0; t < C::TM; ++t) fa[slot][t] = *reinterpret_cast<const v4i*>(As + t * 32 * C::kStride);
#pragma unroll
    for (int t = 0; t < C::TN; ++t) fb[slot][t] = *reinterpret_cast<const v4i*>(Bs + t * 32 * C::kStride);
  };
  // scales of this tile's rows and columns, parked in LDS for the epilogue
  float* sc_row = reinterpret_cast<float*>(lds + C::kLds);
  float* sc_col = sc_row + BM;
  for (int t = tid; t < BM; t += 256) sc_row[t] = m0 + t < M ? ep.s_row[m0 + t] : 0.f;
  for (int t = tid; t < BN; t += 256) sc_col[t] = n0 + t < N ? ep.s_col[n0 + t] : 0.f;
  if (nk > 0) {
    gload(0);
    lstore(0);
    if (nk > 1) gload(BK);
    __syncthreads();
    fread(0, 0, 0);
  }
  // Software pipeline, branch-free so that each k-step is one scheduling region.  While the
  // MFMAs of step s run, the fragments of step s+1 are read from LDS; the tile of stage kt+1
  // goes from registers to the other LDS buffer during step 1 and the global loads of stage
  // kt+2 are issued during step 2, each interleaved one-for-one with the MFMAs; the single
  // barrier per stage sits before the last step, whose MFMAs cover the first fragment reads
  // of the next stage.  Past the end the loads repeat the last tile and the stores hit a
  // buffer nobody reads any more.
  constexpr int S_WRITE = KS >= 4 ? 1 : 0, S_LOAD = KS >= 4 ? 2 : 0;
  constexpr int NMFMA = C::TM * C::TN, NFRAG = C::TM + C::TN, NPIECE = C::kPiecesA + C::kPiecesB;
  constexpr int WPER = NMFMA > NFRAG ? (NPIECE + NMFMA - NFRAG - 1) / (NMFMA - NFRAG) : NPIECE;
  for (int64_t kt = 0; kt < nk; ++kt) {
    const int cur = (int)(kt & 1);
    const int64_t k_ahead = (kt + 2 < nk ? kt + 2 : nk - 1) * BK;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      if (s == KS - 1) {
        __syncthreads();
        fread(cur ^ 1, 0, (s + 1) & 1);
      } else {
        fread(cur, s + 1, (s + 1) & 1);
      }
      if (s == S_WRITE) lstore(cur ^ 1);
      if (s == S_LOAD) gload(k_ahead);
#pragma unroll
      for (int a = 0; a < C::TM; ++a)
#pragma unroll
        for (int b = 0; b < C::TN; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[s & 1][a], fb[s & 1][b], acc[a][b], 0, 0, 0);
      // issue order within the step (0x008 MFMA, 0x100 DS read, 0x200 DS write, 0x020 VMEM read)
      // (LDS reads precede LDS writes in program order and may not be swapped with them)
      if (KS >= 4 && s == S_WRITE) {
#pragma unroll
        for (int i = 0; i < NFRAG; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
#pragma unroll
        for (int i = NFRAG; i < NMFMA; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x200, WPER, 0);
        }
      } else if (KS >= 4 && s == S_LOAD) {
#pragma unroll
        for (int i = 0; i < NMFMA; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          if (i < NFRAG) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
          if (i < NPIECE) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
      } else {
        // fragment reads up front, one per MFMA, so the last one is back long before step s+1
#pragma unroll
        for (int i = 0; i < NFRAG; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, NMFMA > NFRAG ? NMFMA - NFRAG : 1, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  __syncthreads();

  // ---- epilogue.  acc[a][b][v] is element (row, col) of the wave's block with
  //      row = a*32 + 8*(v/4) + 4*(lane/32) + v%4,  col = b*32 + lane%32.
  // Partial sums of |D_F| are taken in float over at most 7 additions of non-negative terms
  // (pairwise over the lane's values, then a fixed shuffle tree over the 32 lanes of a row),
  // and in double from there on, in a fixed order: the result is reproducible run to run.
  double* red = reinterpret_cast<double*>(lds);            // [2][max(BM,BN)], operand tiles are dead
  constexpr int RED = BM > BN ? BM : BN;
  const bool first = ep.mode == kGemmFirst;
  const bool sums = first && ep.row_part != nullptr;
  const int half = lane >> 5, cl = lane & 31;
  const int cbase = wn * (BN / 2) + cl;                    // column of b = 0 inside the tile
  double colsum[C::TN];
  float scol[C::TN];
  bool colok[C::TN];
#pragma unroll
  for (int b = 0; b < C::TN; ++b) {
    colsum[b] = 0.0;
    scol[b] = sc_col[cbase + b * 32];
    colok[b] = n0 + cbase + b * 32 < N;
  }
#pragma unroll
  for (int a = 0; a < C::TM; ++a) {
    const int rbase = wm * (BM / 2) + a * 32 + 4 * half;   // row of v = 0 inside the tile
    float old[C::TN][16];
    if (!first) {
      // accumulate mode: fetch the 16 x TN previous values of this lane in one batch
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int64_t gi = m0 + rbase + 8 * (v >> 2) + (v & 3);
        const float* crow = ep.C + gi * ep.ldc + n0 + cbase;
#pragma unroll
        for (int b = 0; b < C::TN; ++b) old[b][v] = (gi < M && colok[b]) ? crow[b * 32] : 0.f;
      }
    }
    // (the band of Cin as well: one batch of loads, not one round trip per element)
    const bool has_beta = ep.final_scale && ep.beta != 0.f;
    float cin[C::TN][16];
    if (has_beta) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int64_t gi = m0 + rbase + 8 * (v >> 2) + (v & 3);
        const float* cirow = ep.Cin + gi * ep.ldcin + n0 + cbase;
#pragma unroll
        for (int b = 0; b < C::TN; ++b) cin[b][v] = (gi < M && colok[b]) ? cirow[b * 32] : 0.f;
      }
    }
    float ad[C::TN][16];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int rl = rbase + 8 * (v >> 2) + (v & 3);
      const int64_t gi = m0 + rl;
      const float srow = sc_row[rl];
      float* crow = ep.C + gi * ep.ldc + n0 + cbase;
#pragma unroll
      for (int b = 0; b < C::TN; ++b) {
        const int iv = acc[a][b][v];
        const float d = (float)iv * (srow * scol[b]);
        ad[b][v] = fabsf(d);
        if (gi < M && colok[b]) {
          if (DBG && ep.D_int) ep.D_int[gi * ep.ldd + n0 + cbase + b * 32] = iv;
          if (DBG && first && ep.D_F_copy) ep.D_F_copy[gi * ep.ldd + n0 + cbase + b * 32] = d;
          float out = first ? d : old[b][v] + d;
          if (ep.final_scale) {
            out = ep.alpha * out;
            if (has_beta) out = out + ep.beta * cin[b][v];
          }
          crow[b * 32] = out;
        } else {
          ad[b][v] = 0.f;
        }
      }
    }
    if (sums) {
      // Row sums: r[v] is this lane's share of row v of the band.  A reduce-scatter butterfly
      // over the 32 lanes of the half-wave (halving the live values at each exchange) leaves
      // the total of row v = cl >> 1 in lanes cl and cl ^ 1: 16 shuffles instead of 80.
      float r[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        if (C::TN == 4) r[v] = (ad[0][v] + ad[1][v]) + (ad[2][v] + ad[3][v]);
        else r[v] = ad[0][v] + ad[C::TN - 1][v];
      }
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
      if (!(cl & 1)) red[wn * RED + rbase + 8 * (v >> 2) + (v & 3)] = (double)r[0];
#pragma unroll
      for (int b = 0; b < C::TN; ++b) {
        float t8[8], t4[4];
#pragma unroll
        for (int i = 0; i < 8; ++i) t8[i] = ad[b][2 * i] + ad[b][2 * i + 1];
#pragma unroll
        for (int i = 0; i < 4; ++i) t4[i] = t8[2 * i] + t8[2 * i + 1];
        colsum[b] += (double)((t4[0] + t4[1]) + (t4[2] + t4[3]));
      }
    }
  }
  if (sums) {
    __syncthreads();
    for (int t = tid; t < BM; t += 256)
      if (m0 + t < M) ep.row_part[tile_n * (ep.part_ld_m ? ep.part_ld_m : M) + m0 + t] = red[t] + red[RED + t];
    __syncthreads();
#pragma unroll
    for (int b = 0; b < C::TN; ++b) {
      double c = colsum[b];
      c += __shfl_xor(c, 32, 64);                 // the two half-waves hold different rows
      if (half == 0) red[wm * RED + cbase + b * 32] = c;
    }
    __syncthreads();
    for (int t = tid; t < BN; t += 256)
      if (n0 + t < N) ep.col_part[tile_m * (ep.part_ld_n ? ep.part_ld_n : N) + n0 + t] = red[t] + red[RED + t];
  }
}

// C = alpha*C + beta*Cin when no product term carries the final scaling
__global__ void scale_only_kernel(int64_t M, int64_t N, GemmEpilogue ep) {
  int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= N || guard_tripped(ep)) return;
  for (int64_t i = blockIdx.y; i < M; i += gridDim.y) {
    float out = ep.alpha * ep.C[i * ep.ldc + j];
    if (ep.beta != 0.f) out = out + ep.beta * ep.Cin[i * ep.ldcin + j];
    ep.C[i * ep.ldc + j] = out;
  }
}

template <int BM, int BN, int BK>
hipError_t launch_cfg(int64_t M, int64_t N, int64_t K, const int8_t* Qa, int64_t lda, const int8_t* Qb,
                      int64_t ldb, const GemmEpilogue& ep, bool fast, hipStream_t st) {
  using C = Cfg<BM, BN, BK>;
  int64_t tm = (M + BM - 1) / BM, tn = (N + BN - 1) / BN;
  dim3 grid((unsigned)(tm * tn));
  size_t lds_bytes = C::kLds + (BM + BN) * sizeof(float);
  const size_t red_bytes = 2 * sizeof(double) * (BM > BN ? BM : BN);
  if (lds_bytes < red_bytes) lds_bytes = red_bytes;
  // the raw INT32 / pre-correction outputs are only wanted by parity checks: they get their
  // own instantiation so the timed kernel does not carry their code and registers
  const bool dbg = ep.D_int != nullptr || ep.D_F_copy != nullptr;
  auto kern = dbg ? (fast ? gemm_i8_kernel<BM, BN, BK, true, true> : gemm_i8_kernel<BM, BN, BK, false, true>)
                  : (fast ? gemm_i8_kernel<BM, BN, BK, true, false> : gemm_i8_kernel<BM, BN, BK, false, false>);
  if (lds_bytes > 64 * 1024) {
    hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), (int)lds_bytes);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(kern, grid, dim3(256), lds_bytes, st, M, N, K, Qa, lda, Qb, ldb, tm, tn, ep);
  return hipGetLastError();
}

// tile height / width used for an M x N problem (also sizes the partial-sum buffers)
inline bool use_big_tiles(int64_t M, int64_t N) {
  return ((M + 255) / 256) * ((N + 255) / 256) >= 256;   // at least one big tile per compute unit
}

}  // namespace

int gemm_tile_m() { return 128; }   // smallest tile: the partial-sum buffers are sized for it
int gemm_tile_n() { return 128; }
int64_t gemm_tiles_m(int64_t M, int64_t N) { int t = use_big_tiles(M, N) ? 256 : 128; return (M + t - 1) / t; }
int64_t gemm_tiles_n(int64_t M, int64_t N) { int t = use_big_tiles(M, N) ? 256 : 128; return (N + t - 1) / t; }

// A large problem whose M or N is not a multiple of 256: the largest block of whole 256 x 256
// tiles [0, M0) x [0, N0) can still take the persistent kernel, and the plain kernel (128 x 128
// tiles) then only multiplies the strip of columns [N0, N) and the strip of rows [M0, M).
static bool split_ok(int64_t M, int64_t N, int64_t K, const int8_t* Qa, int64_t lda, const int8_t* Qb, int64_t ldb,
                     const GemmEpilogue& ep, int64_t* M0, int64_t* N0) {
  *M0 = M / 256 * 256;
  *N0 = N / 256 * 256;
  if (*M0 <= 0 || *N0 <= 0 || (*M0 == M && *N0 == N)) return false;
  return gemm_persistent_ok(*M0, *N0, K, Qa, lda, Qb, ldb, ep);
}

void gemm_sum_parts(int64_t M, int64_t N, int64_t K, const int8_t* Qa, int64_t lda, const int8_t* Qb, int64_t ldb,
                    const GemmEpilogue& ep, int64_t* parts_n, int64_t* parts_m) {
  int64_t M0, N0;
  // (the persistent and the small-tile kernel leave one partial per 128 columns resp. rows; so does
  // the split, whose strips run with 128 x 128 tiles)
  const bool per128 = gemm_persistent_ok(M, N, K, Qa, lda, Qb, ldb, ep) ||
                      gemm_small_ok(M, N, K, Qa, lda, Qb, ldb, ep) || split_ok(M, N, K, Qa, lda, Qb, ldb, ep, &M0, &N0);
  *parts_n = per128 ? (N + 127) / 128 : gemm_tiles_n(M, N);
  *parts_m = per128 ? (M + 127) / 128 : gemm_tiles_m(M, N);
}

hipError_t launch_gemm_i8(int64_t M, int64_t N, int64_t K, const int8_t* Qa, int64_t lda,
                          const int8_t* Qb, int64_t ldb, const GemmEpilogue& ep, hipStream_t st) {
  if (M <= 0 || N <= 0) return hipSuccess;
  if (gemm_persistent_ok(M, N, K, Qa, lda, Qb, ldb, ep))
    return launch_gemm_i8_persistent(M, N, K, Qa, lda, Qb, ldb, ep, st);
  if (gemm_small_ok(M, N, K, Qa, lda, Qb, ldb, ep)) return launch_gemm_i8_small(M, N, K, Qa, lda, Qb, ldb, ep, st);
  // fast path: every 16-byte piece is aligned and inside [0,K)
  bool fast = ((reinterpret_cast<uintptr_t>(Qa) | reinterpret_cast<uintptr_t>(Qb)) & 15) == 0 &&
              (lda % 16) == 0 && (ldb % 16) == 0 && K > 0 && (K % 64) == 0;
  int64_t M0, N0;
  if (split_ok(M, N, K, Qa, lda, Qb, ldb, ep, &M0, &N0)) {
    GemmEpilogue e = ep;                            // partial sums keep the strides of the whole product
    e.part_ld_m = ep.part_ld_m ? ep.part_ld_m : M;
    e.part_ld_n = ep.part_ld_n ? ep.part_ld_n : N;
    hipError_t err = launch_gemm_i8_persistent(M0, N0, K, Qa, lda, Qb, ldb, e, st);
    if (err != hipSuccess) return err;
    if (N0 < N) {                                   // columns [N0, N), every row
      GemmEpilogue r = e;
      r.s_col = ep.s_col + N0;
      r.C = ep.C + N0;
      if (ep.Cin) r.Cin = ep.Cin + N0;
      if (ep.row_part) r.row_part = ep.row_part + (N0 / 128) * e.part_ld_m;
      if (ep.col_part) r.col_part = ep.col_part + N0;
      err = launch_cfg<128, 128, 64>(M, N - N0, K, Qa, lda, Qb + N0 * ldb, ldb, r, fast, st);
      if (err != hipSuccess) return err;
    }
    if (M0 < M) {                                   // rows [M0, M) of the columns [0, N0)
      GemmEpilogue b = e;
      b.s_row = ep.s_row + M0;
      b.C = ep.C + M0 * ep.ldc;
      if (ep.Cin) b.Cin = ep.Cin + M0 * ep.ldcin;
      if (ep.row_part) b.row_part = ep.row_part + M0;
      if (ep.col_part) b.col_part = ep.col_part + (M0 / 128) * e.part_ld_n;
      err = launch_cfg<128, 128, 64>(M - M0, N0, K, Qa + M0 * lda, lda, Qb, ldb, b, fast, st);
    }
    return err;
  }
  if (use_big_tiles(M, N)) {
    if (fast && K % 128 == 0) return launch_cfg<256, 256, 128>(M, N, K, Qa, lda, Qb, ldb, ep, fast, st);
    return launch_cfg<256, 256, 64>(M, N, K, Qa, lda, Qb, ldb, ep, fast, st);
  }
  return launch_cfg<128, 128, 64>(M, N, K, Qa, lda, Qb, ldb, ep, fast, st);
}

bool gemm_pair_ok(int64_t M, int64_t N, int64_t K, const int8_t* Qa, int64_t lda, const int8_t* Qb, int64_t ldb,
                  const GemmSecond& sec, const GemmEpilogue& ep) {
  if (ep.mode != kGemmAccum || !sec.Qa || !sec.Qb) return false;
  if (gemm_persistent_ok(M, N, K, Qa, lda, Qb, ldb, ep))
    return gemm_persistent_ok(M, N, K, sec.Qa, sec.lda, sec.Qb, sec.ldb, ep);
  return gemm_small_ok(M, N, K, Qa, lda, Qb, ldb, ep) && gemm_small_ok(M, N, K, sec.Qa, sec.lda, sec.Qb, sec.ldb, ep);
}

hipError_t launch_gemm_i8_pair(int64_t M, int64_t N, int64_t K, const int8_t* Qa, int64_t lda, const int8_t* Qb,
                               int64_t ldb, const GemmSecond& sec, const GemmEpilogue& ep, hipStream_t st) {
  if (gemm_persistent_ok(M, N, K, Qa, lda, Qb, ldb, ep))
    return launch_gemm_i8_persistent(M, N, K, Qa, lda, Qb, ldb, ep, st, &sec);
  return launch_gemm_i8_small(M, N, K, Qa, lda, Qb, ldb, ep, st, &sec);
}

hipError_t launch_scale_only(int64_t M, int64_t N, const GemmEpilogue& ep, hipStream_t st) {
  if (M <= 0 || N <= 0) return hipSuccess;
  dim3 grid((unsigned)((N + 255) / 256), (unsigned)(M < 32768 ? M : 32768));
  hipLaunchKernelGGL(scale_only_kernel, grid, dim3(256), 0, st, M, N, ep);
  return hipGetLastError();
}

}  // namespace srq
