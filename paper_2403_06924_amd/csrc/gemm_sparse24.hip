// Persistent INT8 product whose first operand is in 2:4 form (see sparse24.hip), on the sparse
// matrix-core instruction v_smfmac_i32_32x32x64_i8: per instruction and wave a 32 x 32 block of
// the output advances by 64 k, from 16 bytes of kept codes + 32 bits of positions per lane on
// the sparse side and 32 bytes per lane on the dense side.  Same structure as the dense
// persistent kernel (256 x 256 tile per 4-wave workgroup, 128 x 128 per wave, K staged 128 k at
// a time through two LDS stages filled by direct global -> LDS loads, one workgroup per compute
// unit walking several tiles) with, per staged K-tile,
//   sparse operand: 256 rows x 64 bytes of codes (16-byte pieces XOR-swizzled with (row>>2)&3)
//                   + 256 rows x 16 bytes of position nibbles, each one contiguous piece of the
//                   K-tile-major layout compress24 writes,
//   dense operand:  256 rows x 128 bytes (pieces swizzled with (row>>1)&7),
// i.e. 52 KiB instead of 64 KiB, and half the matrix-core instructions.
// Accumulate mode only: C += dequant(product), optionally followed by alpha / beta.
// TRANS: the sparse operand's vectors are the columns of C (term 2, RA . B': the product is
// formed transposed, B'^T . RA^T, and a lane adds four consecutive columns of one row of C).
#include "srq_internal.h"
#include "gemm_tiles.h"

namespace srq {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int BM = 256, BN = 256, BK = 128, KS = BK / 64;
constexpr int kVals = BM * BK / 2;                  // 16 KiB of kept codes
constexpr int kNibs = BM * BK / 8;                  // 4 KiB of positions
constexpr int kDense = BN * BK;                     // 32 KiB
constexpr int kStage = kVals + kNibs + kDense;      // 52 KiB
constexpr int TM = 4, TN = 4;
constexpr int kLdsScales = 2 * kStage;              // float[BM + BN]
constexpr int kLdsBytes = kLdsScales + (BM + BN) * 4;

template <bool TRANS, bool SCALE>
__global__ __launch_bounds__(256) void gemm_i8_sparse24_kernel(int64_t M, int64_t N, int64_t K,
                                                               const int8_t* __restrict__ Av,
                                                               const uint8_t* __restrict__ An,
                                                               const int8_t* __restrict__ Qb, int64_t ldb,
                                                               int64_t tiles_m, int64_t tiles_n, GemmEpilogue ep) {
  extern __shared__ __attribute__((aligned(1024))) int8_t lds[];
  if (guard_tripped(ep)) return;                              // the whole grid leaves together
  float* sc_m = reinterpret_cast<float*>(lds + kLdsScales);   // scale of the sparse operand's vectors
  float* sc_n = sc_m + BM;                                    // scale of the dense operand's vectors
  const uint32_t lds0 = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) int8_t*)lds);
  const float* s_m = TRANS ? ep.s_col : ep.s_row;
  const float* s_n = TRANS ? ep.s_row : ep.s_col;

  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));                     // keeps per-thread offsets from being hoisted out of the tile loop
  const int lane = tid & 63, w = tid >> 6, wm = w >> 1, wn = w & 1;
  const int64_t total = tiles_m * tiles_n, G = gridDim.x, nk = K / BK;

  // ---- loader.  Wave w fetches rows 64w .. 64w+63 of each operand tile.
  //  codes:     4 loads of 16 rows; lane l covers row 16j + l/4 and LDS slot l%4, which holds the
  //             logical piece (l%4) ^ ((row >> 2) & 3) = (l%4) ^ ((l >> 4) & 3)
  //  positions: 1 load, a quarter of the tile's 4 KiB (word planes, see sparse24.hip)
  //  dense:     8 loads of 8 rows as in the dense kernel
  // (the 2:4 operand is stored K-tile-major per block of 256 vectors: a staged tile is one
  // contiguous piece of memory, 64 resp. 16 bytes per vector)
  const int64_t goff_v = (int64_t)(lane >> 2) * (BK / 2) + 16 * ((lane & 3) ^ ((lane >> 4) & 3));
  const int64_t goff_n = (int64_t)lane * 16;        // the 4 KiB of nibbles of a tile are copied as they are
  const int lrow = lane >> 3;
  const int64_t goff_b0 = (int64_t)lrow * ldb + 16 * ((lane & 7) ^ ((lane >> 4) & 7));
  const int64_t goff_b1 = (int64_t)lrow * ldb + 16 * ((lane & 7) ^ (((lane >> 4) + 4) & 7));
  int64_t vba = blockIdx.x, kta = 0;                // cursor of the K-tile being fetched
  const int8_t *pv, *pb;
  const uint8_t* pn;
  auto point = [&]() {
    int64_t tm, tn;
    tile_of(vba, tiles_m, tiles_n, tm, tn);
    pv = Av + ((tm * nk + kta) * BM + 64 * w) * (BK / 2);
    pn = An + (tm * nk + kta) * kNibs + 1024 * w;
    pb = Qb + (tn * BN + 64 * w) * ldb + kta * BK;
  };
  auto advance = [&]() {
    if (kta + 1 < nk) {
      ++kta;
      pv += BM * (BK / 2);
      pn += BM * (BK / 8);
      pb += BK;
    } else if (vba + G < total) {
      vba += G;
      kta = 0;
      point();
    }                                               // else stay on the last K-tile (harmless re-fetch)
  };
  // load i (0..12) of the K-tile at the cursor into LDS buffer `stage`
  auto issue_load = [&](int stage, int i) {
    // (wave-uniform by construction; readfirstlane tells the compiler so: the addresses feed M0)
    const uint32_t base = lds0 + stage * kStage;
    const uint32_t lv = __builtin_amdgcn_readfirstlane(base + (64 * w) * (BK / 2));
    const uint32_t ln = __builtin_amdgcn_readfirstlane(base + kVals + (64 * w) * (BK / 8));
    const uint32_t lb = __builtin_amdgcn_readfirstlane(base + kVals + kNibs + (64 * w) * BK);
    if (i < 4)
      load_to_lds(pv + (16 * i) * (BK / 2) + goff_v, lv + 16 * i * (BK / 2));
    else if (i == 4)
      load_to_lds(reinterpret_cast<const int8_t*>(pn + goff_n), ln);
    else {
      const int j = i - 5;
      load_to_lds(pb + (int64_t)(8 * j) * ldb + ((j & 1) ? goff_b1 : goff_b0), lb + 8 * j * BK);
    }
  };
  auto issue_loads = [&](int stage) {
#pragma unroll
    for (int i = 0; i < 13; ++i) issue_load(stage, i);
  };

  // ---- fragment reads of lane (frow, kh) at step s of a K-tile (64 k per step)
  const int frow = lane & 31, kh = lane >> 5;
  const int key_v = (frow >> 2) & 3, key_b = (frow >> 1) & 7;
  const int v_row = (wm * (BM / 2) + frow) * (BK / 2);
  // (position words: plane-major, vectors of the odd planes rotated by 32; plane = 2 step + kh)
  const int n_row = kVals + 4 * ((wm * (BM / 2) + frow) ^ (32 * kh));
  const int b_row = kVals + kNibs + (wn * (BN / 2) + frow) * BK;
  int xv[KS], xn[KS], xb0[KS], xb1[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    xv[s] = 16 * ((2 * s + kh) ^ key_v);
    xn[s] = 4 * 256 * (2 * s + kh);
    xb0[s] = 16 * ((4 * s + 2 * kh) ^ key_b);
    xb1[s] = 16 * ((4 * s + 2 * kh + 1) ^ key_b);
  }
  v4i fa[2][TM];
  int fi[2][TM];
  v8i fb[2][TN];
  auto fread = [&](int stage, int step, int slot) {
    const int8_t* base = lds + stage * kStage;
#pragma unroll
    for (int t = 0; t < TM; ++t) {
      fa[slot][t] = *reinterpret_cast<const v4i*>(base + v_row + t * 32 * (BK / 2) + xv[step]);
      fi[slot][t] = *reinterpret_cast<const int*>(base + (n_row ^ (4 * 32 * (t & 1))) + 4 * 32 * (t & ~1) + xn[step]);
    }
#pragma unroll
    for (int t = 0; t < TN; ++t) {
      const v4i lo = *reinterpret_cast<const v4i*>(base + b_row + t * 32 * BK + xb0[step]);
      const v4i hi = *reinterpret_cast<const v4i*>(base + b_row + t * 32 * BK + xb1[step]);
      fb[slot][t] = v8i{lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
    }
  };

  int64_t vb = blockIdx.x, tile_m, tile_n;
  tile_of(vb, tiles_m, tiles_n, tile_m, tile_n);
  float sreg_m = s_m[tile_m * BM + tid], sreg_n = s_n[tile_n * BN + tid];

  point();
  issue_loads(0);
  advance();
  wait_loads();
  __syncthreads();
  issue_loads(1);
  advance();
  fread(0, 0, 0);

  v16i acc[TM][TN];
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0;

  const int64_t my_tiles = (total - blockIdx.x + G - 1) / G;
  int g = 0;                                        // parity of the K-tile stream across tiles
  for (int64_t tile = 0; tile < my_tiles; ++tile) {
    for (int64_t kt = 0; kt < nk; ++kt, ++g) {
      const int cur = g & 1;
      // step 0: the fragments of step 1 are read while step 0 multiplies
      fread(cur, 1, 1);
#pragma unroll
      for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
          acc[a][b] = __builtin_amdgcn_smfmac_i32_32x32x64_i8(fa[0][a], fb[0][b], acc[a][b], fi[0][a], 0, 0);
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      // step 1: K-tile g+1 (loads issued one whole K-tile ago) must have landed; after the
      // barrier everybody is also done reading buffer `cur`, which takes K-tile g+2
      wait_loads();
      __syncthreads();
      fread(cur ^ 1, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b) {
          acc[a][b] = __builtin_amdgcn_smfmac_i32_32x32x64_i8(fa[1][a], fb[1][b], acc[a][b], fi[1][a], 0, 0);
          if (a * TN + b < 13) issue_load(cur, a * TN + b);
          __builtin_amdgcn_sched_barrier(0);
        }
      advance();
    }

    // ================= epilogue of tile (tile_m, tile_n); tiles are full
    sc_m[tid] = sreg_m;
    sc_n[tid] = sreg_n;
    __syncthreads();
    const int64_t m0 = tile_m * BM, n0 = tile_n * BN;
    const int half = lane >> 5, cl = lane & 31;
    const int cbase = wn * (BN / 2) + cl;           // dense-side vector of this lane, plus 32 b
    float scn[TN];
#pragma unroll
    for (int b = 0; b < TN; ++b) scn[b] = sc_n[cbase + b * 32];
#pragma unroll
    for (int a = 0; a < TM; ++a) {
      const int rbase = wm * (BM / 2) + a * 32 + 4 * half;   // sparse-side vector, plus 8 (v>>2) + (v&3)
      if (!TRANS) {
        // C[m0 + row][n0 + col]: a lane adds to one column, rows 8 (v>>2) + (v&3)
        float* cband = ep.C + (m0 + rbase) * ep.ldc + n0 + cbase;
        float x[TN][16];
#pragma unroll
        for (int v = 0; v < 16; ++v)
#pragma unroll
          for (int b = 0; b < TN; ++b)
            x[b][v] = __builtin_nontemporal_load(&cband[(int64_t)(8 * (v >> 2) + (v & 3)) * ep.ldc + b * 32]);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int ro = 8 * (v >> 2) + (v & 3);
          const float sm = sc_m[rbase + ro];
#pragma unroll
          for (int b = 0; b < TN; ++b) {
            float out = x[b][v] + (float)acc[a][b][v] * (sm * scn[b]);
            if (SCALE) {
              out = ep.alpha * out;
              if (ep.beta != 0.f) out = out + ep.beta * ep.Cin[(m0 + rbase + ro) * ep.ldcin + n0 + cbase + b * 32];
            }
            __builtin_nontemporal_store(out, &cband[(int64_t)ro * ep.ldc + b * 32]);
            acc[a][b][v] = 0;
          }
        }
      } else {
        // C[n0 + col][m0 + row]: the four rows (v&3) of the product are four consecutive columns of C
        typedef float f4v __attribute__((ext_vector_type(4)));
#pragma unroll
        for (int b = 0; b < TN; ++b) {
          const int64_t ci = n0 + cbase + b * 32;                        // row of C
          f4v x[4];
#pragma unroll
          for (int q = 0; q < 4; ++q)
            x[q] = __builtin_nontemporal_load(reinterpret_cast<const f4v*>(ep.C + ci * ep.ldc + m0 + rbase + 8 * q));
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            f4v o = x[q];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
              // (the scale product is taken row scale of C first, as everywhere else)
              float out = o[t] + (float)acc[a][b][4 * q + t] * (scn[b] * sc_m[rbase + 8 * q + t]);
              if (SCALE) {
                out = ep.alpha * out;
                if (ep.beta != 0.f) out = out + ep.beta * ep.Cin[ci * ep.ldcin + m0 + rbase + 8 * q + t];
              }
              o[t] = out;
              acc[a][b][4 * q + t] = 0;
            }
            __builtin_nontemporal_store(o, reinterpret_cast<f4v*>(ep.C + ci * ep.ldc + m0 + rbase + 8 * q));
          }
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    // next output tile of this workgroup
    vb += G;
    if (vb < total) {
      tile_of(vb, tiles_m, tiles_n, tile_m, tile_n);
      sreg_m = s_m[tile_m * BM + tid];
      sreg_n = s_n[tile_n * BN + tid];
    }
    // (sc_m / sc_n are rewritten by the next epilogue: a whole K loop and its barriers lie between)
  }
  wait_loads();                                     // nothing may still be writing LDS when the wave ends
}

}  // namespace

// Mv, Nv: vectors of the sparse / dense operand (multiples of 256); K a multiple of 128
bool gemm_sparse24_ok(int64_t Mv, int64_t Nv, int64_t K, const int8_t* Av, const uint8_t* An, const int8_t* Qb,
                      int64_t ldb, bool trans, const GemmEpilogue& ep) {
  if (ep.D_int || ep.D_F_copy) return false;
  if (Mv <= 0 || Nv <= 0 || K <= 0 || (Mv % BM) || (Nv % BN) || (K % BK)) return false;
  if (((reinterpret_cast<uintptr_t>(Av) | reinterpret_cast<uintptr_t>(An) | reinterpret_cast<uintptr_t>(Qb)) & 15) ||
      (ldb % 16))
    return false;
  // the transposed epilogue adds to C sixteen bytes at a time
  if (trans && ((reinterpret_cast<uintptr_t>(ep.C) & 15) || (ep.ldc % 4))) return false;
  return true;
}

hipError_t launch_gemm_i8_sparse24(int64_t Mv, int64_t Nv, int64_t K, const int8_t* Av, const uint8_t* An,
                                   const int8_t* Qb, int64_t ldb, bool trans, const GemmEpilogue& ep,
                                   hipStream_t st) {
  int num_cu = 0;
  hipError_t e = gemm_device_cus(&num_cu);
  if (e != hipSuccess) return e;
  const int64_t tm = Mv / BM, tn = Nv / BN;
  int64_t wgs = num_cu / 8 * 8;                              // one workgroup per CU, a multiple of the 8 XCDs
  if (wgs < 8) wgs = 8;
  if (wgs > tm * tn) wgs = tm * tn;
  const bool scale = ep.final_scale != 0;
  void (*kern)(int64_t, int64_t, int64_t, const int8_t*, const uint8_t*, const int8_t*, int64_t, int64_t, int64_t,
               GemmEpilogue);
  kern = trans ? (scale ? gemm_i8_sparse24_kernel<true, true> : gemm_i8_sparse24_kernel<true, false>)
               : (scale ? gemm_i8_sparse24_kernel<false, true> : gemm_i8_sparse24_kernel<false, false>);
  e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), kLdsBytes);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3((unsigned)wgs), dim3(256), kLdsBytes, st, Mv, Nv, K, Av, An, Qb, ldb, tm, tn, ep);
  return hipGetLastError();
}

}  // namespace srq
