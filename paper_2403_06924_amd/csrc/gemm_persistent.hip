// Persistent variant of the INT8 GEMM for full, aligned problems (M, N multiples of 256, K a
// multiple of 128, 16-byte aligned operands): the shape of every large workload.
//
// Same output tile as gemm_i8_kernel (256 x 256 per 4-wave workgroup, 128 x 128 per wave,
// v_mfma_i32_32x32x32_i8) with three differences made for gfx950:
//
//  * operand tiles go from global memory straight into LDS (global_load_lds_dwordx4): no
//    staging registers and no ds_write instructions.  The hardware writes the 64 lanes of one
//    load to 1 KiB of consecutive LDS bytes, so the tile rows are unpadded (128 B) and bank
//    conflicts of the 16-byte fragment reads are avoided by an XOR swizzle instead: the 16-byte
//    piece s of row r sits at position s ^ ((r >> 1) & 7), applied on the global-address side
//    when loading and on the LDS-address side when reading;
//  * a workgroup walks over several output tiles and the stream of staged K-tiles never drains
//    between them: while one tile's epilogue runs, the first K-tiles of the next are already
//    landing in LDS (they need no registers), and the epilogue's stores retire while the next
//    tile is multiplied.  A one-tile-per-workgroup launch pays launch, prologue latency and
//    drain once per tile - four times per CU at 8192^3, since only one workgroup fits a CU;
//  * LDS holds three buffers for the tiles of A and two for the tiles of B (5 x 32 KiB, all of a
//    CU's LDS).  The sixteen loads that a wave issues per K-tile are spread evenly over its four
//    steps: the CU's vector-memory path takes a 1 KiB load about every 20 clocks, and a wave
//    whose load cannot be accepted yet also holds back the MFMAs behind it (with all sixteen in
//    the one step that follows the hand-over of a buffer, that step took 2.3 times as long as
//    the others).  The third A buffer is what makes room for that: the A tile of K-tile g+2 is
//    fetched during the middle steps of K-tile g, one K-tile earlier than a two-buffer scheme
//    could, so those loads also have twice as long to land, which matters when the operands
//    come from HBM rather than from the caches.
#include <atomic>
#include <mutex>
#include <type_traits>
#include <utility>
#include <vector>
#include "srq_internal.h"
#include "gemm_tiles.h"

namespace srq {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int BM = 256, BN = 256, BK = 128, KS = BK / 32;
constexpr int kOperand = BM * BK;                   // 32 KiB per operand tile
constexpr int TM = 4, TN = 4;                       // 32x32 MFMA tiles per wave
constexpr int kABufs = 3, kBBufs = 2;               // LDS buffers of the A tiles and of the B tiles
constexpr int kLdsB = kABufs * kOperand;            // the B buffers follow the A buffers
constexpr int kLdsBytes = kLdsB + kBBufs * kOperand;   // 160 KiB; the epilogue's scales borrow a free A buffer
constexpr int kLoads = 8;                           // loads per wave, operand and K-tile

template <int MODE, bool SUMS, bool SCALE>
__global__ __launch_bounds__(256) void gemm_i8_persistent_kernel(int64_t M, int64_t N, int64_t K,
                                                                 const int8_t* __restrict__ Qa, int64_t lda,
                                                                 const int8_t* __restrict__ Qb, int64_t ldb,
                                                                 int64_t tiles_m, int64_t tiles_n,
                                                                 GemmEpilogue ep, GemmSecond sec) {
  extern __shared__ __attribute__((aligned(1024))) int8_t lds[];
  if (MODE == kGemmAccum && guard_tripped(ep)) return;   // the whole grid leaves together
  // LDS byte address of the first stage (an address-space-3 pointer is a 32-bit offset)
  const uint32_t lds0 = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) int8_t*)lds);

  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));                     // keeps per-thread offsets from being hoisted out of the tile loop
  const int lane = tid & 63, w = tid >> 6, wm = w >> 1, wn = w & 1;
  const int64_t total = tiles_m * tiles_n, G = gridDim.x, nk = K / BK;
  // accumulate mode may carry a second product over the same tiles (sec.Qa != null): a workgroup
  // then runs product 0 and product 1 of a tile back to back, so that the tile of C written by
  // the first is still in the caches when the second adds to it
  const int nprod = (MODE == kGemmAccum && sec.Qa) ? 2 : 1;
  int p_lo, p_hi;                                   // the products this launch runs (device-side decision)
  pair_range(ep, nprod, p_lo, p_hi);

  // ---- loader: wave w fetches rows 64w .. 64w+63 of each operand tile, eight rows per load.
  // Lane l of load j covers row 64w + 8j + l/8 and LDS piece l%8, which holds the logical piece
  // (l%8) ^ ((row >> 1) & 7); (row >> 1) & 7 = ((l >> 4) + 4j) & 7 depends on j only through
  // its parity.
  const int lrow = lane >> 3;
  int64_t vba = blockIdx.x;                         // cursor of the K-tile being fetched: output tile,
  int kta = 0;                                      // ... K-tile within it
  int proda = p_lo;                                 // ... and the product it belongs to
  const int nk32 = (int)nk;
  const int8_t *pa, *pb;                            // row 64w of that K-tile in A and in B
  int64_t cur_lda = lda, cur_ldb = ldb;
  int64_t goff_a0 = 0, goff_a1 = 0, goff_b0 = 0, goff_b1 = 0;
  auto point = [&]() {
    int64_t tm, tn;
    tile_of(vba, tiles_m, tiles_n, tm, tn);
    const int8_t* A0 = proda ? sec.Qa : Qa;
    const int8_t* B0 = proda ? sec.Qb : Qb;
    cur_lda = proda ? sec.lda : lda;
    cur_ldb = proda ? sec.ldb : ldb;
    goff_a0 = (int64_t)lrow * cur_lda + 16 * ((lane & 7) ^ ((lane >> 4) & 7));
    goff_a1 = (int64_t)lrow * cur_lda + 16 * ((lane & 7) ^ (((lane >> 4) + 4) & 7));
    goff_b0 = (int64_t)lrow * cur_ldb + 16 * ((lane & 7) ^ ((lane >> 4) & 7));
    goff_b1 = (int64_t)lrow * cur_ldb + 16 * ((lane & 7) ^ (((lane >> 4) + 4) & 7));
    pa = A0 + (tm * BM + 64 * w) * cur_lda + (int64_t)kta * BK;
    pb = B0 + (tn * BN + 64 * w) * cur_ldb + (int64_t)kta * BK;
  };
  int kstep = BK;                                   // 0 once the cursor has reached the end of the launch
  auto advance = [&]() {
    if (kta + 1 < nk32) {
      kta += kstep ? 1 : 0;
      pa += kstep;
      pb += kstep;
    } else if (proda < p_hi) {
      ++proda;
      kta = 0;
      point();
    } else if (vba + G < total) {
      vba += G;
      proda = p_lo;
      kta = 0;
      point();
    } else {
      kstep = 0;                                    // stay on the last K-tile (harmless re-fetch)
    }
  };
  // The same where the caller knows that the cursor stays inside its output tile (or has reached
  // the end): no branch, and so no point where the compiler, having seen the reloads of spilled
  // registers on the other path, would wait for every load in flight.
  auto advance_within = [&]() {
    kta += kstep ? 1 : 0;
    pa += kstep;
    pb += kstep;
  };
  // load j (0..7) of the A resp. B tile at the cursor into buffer `buf` of that operand
  auto issue_a = [&](int buf, int j) {
    // wave-uniform by construction; readfirstlane tells the compiler so (it feeds M0)
    const uint32_t la = __builtin_amdgcn_readfirstlane(lds0 + buf * kOperand + (64 * w) * BK);
    load_to_lds(pa + (int64_t)(8 * j) * cur_lda + ((j & 1) ? goff_a1 : goff_a0), la + j * 8 * BK);
  };
  auto issue_b = [&](int buf, int j) {
    const uint32_t la = __builtin_amdgcn_readfirstlane(lds0 + kLdsB + buf * kOperand + (64 * w) * BK);
    load_to_lds(pb + (int64_t)(8 * j) * cur_ldb + ((j & 1) ? goff_b1 : goff_b0), la + j * 8 * BK);
  };

  // ---- fragment reads: lane (frow, kh) reads logical piece 2*step + kh of its rows
  const int frow = lane & 31, kh = lane >> 5, key = (frow >> 1) & 7;
  const int a_row = (wm * (BM / 2) + frow) * BK;
  const int b_row = kLdsB + (wn * (BN / 2) + frow) * BK;
  int xoff[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s) xoff[s] = 16 * ((2 * s + kh) ^ key);
  v4i fa[2][TM], fb[2][TN];
  auto fread = [&](int abuf, int bbuf, int step, int slot) {
    const int8_t* As = lds + abuf * kOperand + a_row + xoff[step];
    const int8_t* Bs = lds + bbuf * kOperand + b_row + xoff[step];
#pragma unroll
    for (int t = 0; t < TM; ++t) fa[slot][t] = *reinterpret_cast<const v4i*>(As + t * 32 * BK);
#pragma unroll
    for (int t = 0; t < TN; ++t) fb[slot][t] = *reinterpret_cast<const v4i*>(Bs + t * 32 * BK);
  };

  // read r of a step's eight fragment reads: 0..3 -> A tiles, 4..7 -> B tiles
  auto fread1 = [&](int abuf, int bbuf, int step, int slot, int r) {
    if (r < TM)
      fa[slot][r] = *reinterpret_cast<const v4i*>(lds + abuf * kOperand + a_row + xoff[step] + r * 32 * BK);
    else
      fb[slot][r - TM] = *reinterpret_cast<const v4i*>(lds + bbuf * kOperand + b_row + xoff[step] + (r - TM) * 32 * BK);
  };

  // ---- the output tile being multiplied
  int64_t vb = blockIdx.x, tile_m, tile_n;
  tile_of(vb, tiles_m, tiles_n, tile_m, tile_n);
  float sreg_row = (p_lo ? sec.s_row : ep.s_row)[tile_m * BM + tid];
  float sreg_col = (p_lo ? sec.s_col : ep.s_col)[tile_n * BN + tid];

  // K-tile 0, the A tile of K-tile 1 and the first half of its B tile
  point();
#pragma unroll
  for (int j = 0; j < kLoads; ++j) issue_a(0, j);
#pragma unroll
  for (int j = 0; j < kLoads; ++j) issue_b(0, j);
  advance();
#pragma unroll
  for (int j = 0; j < kLoads; ++j) issue_a(1, j);
#pragma unroll
  for (int j = 0; j < kLoads / 2; ++j) issue_b(1, j);
  wait_loads_but<kLoads + kLoads / 2>();            // K-tile 0 has landed
  __syncthreads();
  fread(0, 0, 0, 0);

  v16i acc[TM][TN];
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0;

  // Accumulate mode reads the tile of C it adds to.  Every compute unit reaches its epilogue at
  // about the same time, so loads issued there arrive as one burst per round while the memory
  // system idles in between: the first band of the tile (the lane's 16 rows x TN columns of the
  // first 32 rows of its wave tile) is therefore fetched during the K loop instead, a few K-tiles
  // before the last one, and waits in registers.  All its loads go out in one K-tile and straight
  // into their registers: nothing in the K loop reads a register that a load is still to fill
  // (the compiler, which does not see the operand loads, would wait there for all of them).
  constexpr int kPfBands = 1;                       // bands fetched ahead (of TM); two cost more in spills than they hide
  const bool pf_on = MODE == kGemmAccum && !SCALE && nk >= 8;   // (alpha / beta need the registers)
  const int64_t pf0 = nk - 4;                       // K-tile that issues the loads
  float pre[kPfBands][TN][16];
#pragma unroll
  for (int a = 0; a < kPfBands; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) pre[a][b][v] = 0.f;
  const int half = lane >> 5, cl = lane & 31;
  const int cbase = wn * (BN / 2) + cl;

  const int64_t my_tiles = (total - blockIdx.x + G - 1) / G;
  int g = 0;                                        // position in the K-tile stream across tiles
  int abuf = 0;                                     // A buffer of K-tile g (g mod 3)
  int prod = p_lo;                                  // product being multiplied (pairs: 0, 1, 0, 1, ...)
  const bool two = p_lo != p_hi;
  for (int64_t tile = 0; tile < my_tiles * (p_hi - p_lo + 1); ++tile) {
  auto ktile = [&](int64_t kt, auto crossing) {
    // Loads of this K-tile's four steps, four in each:
    //   step 0: second half of the B tile of K-tile g+1 (its buffer was handed over by the
    //           barrier of the step before); then the cursor moves on to K-tile g+2;
    //   steps 1, 2: the A tile of K-tile g+2, into the buffer that K-tile g-1 left;
    //   step 3, after the barrier: first half of the B tile of K-tile g+2, into this K-tile's.
    const int bbuf = g & 1;
    const int anext = abuf == kABufs - 1 ? 0 : abuf + 1, aload = anext == kABufs - 1 ? 0 : anext + 1;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      if (s == KS - 1) {
        // K-tile g+1 must have landed: everything but the eight loads of the A tile of K-tile
        // g+2.  After the barrier everybody is also done reading this K-tile's buffers.
        wait_loads_but<kLoads>();
        __syncthreads();
        fread(anext, bbuf ^ 1, 0, (s + 1) & 1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
          for (int b = 0; b < TN; ++b) {
            acc[a][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[s & 1][a], fb[s & 1][b], acc[a][b], 0, 0, 0);
            if (b == TN - 1) issue_b(bbuf, a);
            __builtin_amdgcn_sched_barrier(0);
          }
        if (MODE == kGemmAccum && pf_on && kt == pf0) {
          // the first band of C: rows 8 (v >> 2) + (v & 3) of the lane's 32-row band
          const float* cband0 = ep.C + (tile_m * BM + wm * (BM / 2) + 4 * half) * ep.ldc + tile_n * BN + cbase;
          if (p_lo != p_hi && prod == 1) {            // the first product of the pair left the tile in the caches
#pragma unroll
            for (int v = 0; v < 16; ++v)
#pragma unroll
              for (int b = 0; b < TN; ++b) pre[0][b][v] = cband0[(int64_t)(8 * (v >> 2) + (v & 3)) * ep.ldc + b * 32];
          } else {
#pragma unroll
            for (int v = 0; v < 16; ++v)
#pragma unroll
              for (int b = 0; b < TN; ++b)
                pre[0][b][v] = __builtin_nontemporal_load(&cband0[(int64_t)(8 * (v >> 2) + (v & 3)) * ep.ldc + b * 32]);
          }
        }
      } else {
        // the fragments of the next step: one read after each of the first eight MFMAs
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
          for (int b = 0; b < TN; ++b) {
            acc[a][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[s & 1][a], fb[s & 1][b], acc[a][b], 0, 0, 0);
            if (a * TN + b < 8) fread1(abuf, bbuf, s + 1, (s + 1) & 1, a * TN + b);
            // ... and one load after every second MFMA of the other eight
            if (a * TN + b >= 8 && !(b & 1)) {
              const int n = (a * TN + b - 8) >> 1;
              if (s == 0) issue_b(bbuf ^ 1, kLoads / 2 + n);
              if (s == 1) issue_a(aload, n);
              if (s == 2) issue_a(aload, kLoads / 2 + n);
            }
            __builtin_amdgcn_sched_barrier(0);
          }
        if (s == 0) {
          if (decltype(crossing)::value) advance();
          else advance_within();
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    abuf = anext;
    ++g;
  };
  // The cursor is two K-tiles ahead and moves on in the first step of a K-tile: it leaves its
  // output tile (or product) in K-tile nk - 2 and nowhere else.
  if (nk >= 3) {
    for (int64_t kt = 0; kt < nk - 2; ++kt) ktile(kt, std::false_type());
    ktile(nk - 2, std::true_type());
    ktile(nk - 1, std::false_type());
  } else {
    for (int64_t kt = 0; kt < nk; ++kt) ktile(kt, std::true_type());
  }

    // ================= epilogue of tile (tile_m, tile_n); no bounds checks: tiles are full
    // The scales are staged in the A buffer that the last K-tile has just left (everybody passed
    // that K-tile's barrier after its last read); the next loads into it go out in the second
    // step of the next K-tile, which the barrier at the end of the epilogue holds back.
    float* sc_row = reinterpret_cast<float*>(lds + (abuf == 0 ? kABufs - 1 : abuf - 1) * kOperand);
    float* sc_col = sc_row + BM;
    sc_row[tid] = sreg_row;
    sc_col[tid] = sreg_col;
    __syncthreads();
    const int64_t m0 = tile_m * BM, n0 = tile_n * BN;
    double colsum[TN];
    float scol[TN];
#pragma unroll
    for (int b = 0; b < TN; ++b) {
      colsum[b] = 0.0;
      scol[b] = sc_col[cbase + b * 32];
    }
    // C goes around the caches (it would evict the FP32 operands the next stages stream), except
    // between the two products of a pair: the first leaves its tile cached for the second
    const bool do_scale = SCALE && prod == nprod - 1;
    // (alpha, beta and the stride of Cin are read here, not kept in registers through the K loop)
    const float alpha = SCALE ? ep.alpha : 1.f, beta = SCALE ? ep.beta : 0.f;
    const bool has_beta = SCALE && do_scale && beta != 0.f;
    const int64_t ldcin = SCALE ? ep.ldcin : 0;
    auto bands = [&](auto cached_load_tag, auto cached_store_tag) {
    constexpr bool CLOAD = decltype(cached_load_tag)::value, CSTORE = decltype(cached_store_tag)::value;
#pragma unroll
    for (int a = 0; a < TM; ++a) {
      const int rbase = wm * (BM / 2) + a * 32 + 4 * half;
      float* cband = ep.C + (m0 + rbase) * ep.ldc + n0 + cbase;
      float x[TN][16];
      float cin[TN][16];                              // the band of Cin, all loads in flight at once
      if (SCALE && has_beta) {
        const float* cinband = ep.Cin + (m0 + rbase) * ldcin + n0 + cbase;
#pragma unroll
        for (int v = 0; v < 16; ++v)
#pragma unroll
          for (int b = 0; b < TN; ++b)
            cin[b][v] = __builtin_nontemporal_load(&cinband[(int64_t)(8 * (v >> 2) + (v & 3)) * ldcin + b * 32]);
      }
      if (MODE == kGemmAccum) {
        if (a < kPfBands && pf_on) {
#pragma unroll
          for (int v = 0; v < 16; ++v)
#pragma unroll
            for (int b = 0; b < TN; ++b) x[b][v] = pre[a < kPfBands ? a : 0][b][v];
        } else {
#pragma unroll
          for (int v = 0; v < 16; ++v)
#pragma unroll
            for (int b = 0; b < TN; ++b) {
              const float* src = &cband[(int64_t)(8 * (v >> 2) + (v & 3)) * ep.ldc + b * 32];
              x[b][v] = CLOAD ? *src : __builtin_nontemporal_load(src);
            }
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
        for (int v = 0; v < 16; ++v) r[v] = (x[0][v] + x[1][v]) + (x[2][v] + x[3][v]);
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
        // each wave leaves its own partial (its 128 columns of the tile): no exchange through LDS
        // and no barrier, so a wave that is done starts on the next tile
        if (!(cl & 1)) ep.row_part[(2 * tile_n + wn) * (ep.part_ld_m ? ep.part_ld_m : M) + m0 + rbase + 8 * (v >> 2) + (v & 3)] =
              (double)r[0];
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
#pragma unroll
      for (int b = 0; b < TN; ++b) {
        double c = colsum[b];
        c += __shfl_xor(c, 32, 64);
        if (half == 0) ep.col_part[(2 * tile_m + wm) * (ep.part_ld_n ? ep.part_ld_n : N) + n0 + cbase + b * 32] = c;
      }
    }
    // everybody has read its scales: the A buffer that held them may be loaded again (a bare
    // barrier: the stores of C stay in flight)
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" : : : "memory");
    // next product of this tile, or the next output tile of this workgroup
    if (prod < p_hi) {
      prod = 1;
      sreg_row = sec.s_row[tile_m * BM + tid];
      sreg_col = sec.s_col[tile_n * BN + tid];
    } else {
      prod = p_lo;
      vb += G;
      if (vb < total) {
        tile_of(vb, tiles_m, tiles_n, tile_m, tile_n);
        sreg_row = (p_lo ? sec.s_row : ep.s_row)[tile_m * BM + tid];
        sreg_col = (p_lo ? sec.s_col : ep.s_col)[tile_n * BN + tid];
      }
    }
  }
  wait_loads();                                     // nothing may still be writing LDS when the wave ends
}

}  // namespace

bool gemm_persistent_ok(int64_t M, int64_t N, int64_t K, const int8_t* Qa, int64_t lda, const int8_t* Qb,
                        int64_t ldb, const GemmEpilogue& ep) {
  if (ep.D_int || ep.D_F_copy) return false;                 // parity-check outputs use the plain kernel
  if (M <= 0 || N <= 0 || K <= 0 || (M % BM) || (N % BN) || (K % BK)) return false;
  if (((reinterpret_cast<uintptr_t>(Qa) | reinterpret_cast<uintptr_t>(Qb)) & 15) || (lda % 16) || (ldb % 16))
    return false;
  return (M / BM) * (N / BN) >= 256;                        // at least one tile per compute unit
}

// Compute units of the current device, looked up once per device (srq_create primes it, so
// that no property query happens inside a caller's stream capture).
hipError_t gemm_device_cus(int* cus) {
  static std::atomic<int> cached[64];               // zero-initialised; a racing first query stores the same value
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  int n = (dev >= 0 && dev < 64) ? cached[dev].load(std::memory_order_relaxed) : 0;
  if (!n) {
    hipDeviceProp_t prop;
    e = hipGetDeviceProperties(&prop, dev);
    if (e != hipSuccess) return e;
    n = prop.multiProcessorCount;
    if (dev >= 0 && dev < 64) cached[dev].store(n, std::memory_order_relaxed);
  }
  *cus = n;
  return hipSuccess;
}

hipError_t ensure_dynamic_lds(const void* kernel, int bytes) {
  static std::mutex mu;
  static std::vector<std::pair<int, const void*>> done;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  std::lock_guard<std::mutex> lock(mu);
  for (const auto& d : done)
    if (d.first == dev && d.second == kernel) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess) done.emplace_back(dev, kernel);
  return e;
}

hipError_t launch_gemm_i8_persistent(int64_t M, int64_t N, int64_t K, const int8_t* Qa, int64_t lda,
                                     const int8_t* Qb, int64_t ldb, const GemmEpilogue& ep, hipStream_t st,
                                     const GemmSecond* second) {
  int num_cu = 0;
  hipError_t e = gemm_device_cus(&num_cu);
  if (e != hipSuccess) return e;
  const int64_t tm = M / BM, tn = N / BN;
  int64_t wgs = num_cu / 8 * 8;                              // one workgroup per CU, a multiple of the 8 XCDs
  if (wgs < 8) wgs = 8;
  if (wgs > tm * tn) wgs = tm * tn;
  const bool sums = ep.mode == kGemmFirst && ep.row_part != nullptr;
  const bool scale = ep.final_scale != 0;
  void (*kern)(int64_t, int64_t, int64_t, const int8_t*, int64_t, const int8_t*, int64_t, int64_t, int64_t,
               GemmEpilogue, GemmSecond);
  GemmSecond sec = {nullptr, nullptr, 0, 0, nullptr, nullptr};
  if (second && ep.mode == kGemmAccum) sec = *second;
  if (ep.mode == kGemmFirst) {
    kern = sums ? (scale ? gemm_i8_persistent_kernel<kGemmFirst, true, true>
                         : gemm_i8_persistent_kernel<kGemmFirst, true, false>)
                : (scale ? gemm_i8_persistent_kernel<kGemmFirst, false, true>
                         : gemm_i8_persistent_kernel<kGemmFirst, false, false>);
  } else {
    kern = scale ? gemm_i8_persistent_kernel<kGemmAccum, false, true>
                 : gemm_i8_persistent_kernel<kGemmAccum, false, false>;
  }
  e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), kLdsBytes);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3((unsigned)wgs), dim3(256), kLdsBytes, st, M, N, K, Qa, lda, Qb, ldb, tm, tn, ep,
                     sec);
  return hipGetLastError();
}

}  // namespace srq
