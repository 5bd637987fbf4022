// Persistent INT8 product whose first operand is in 2:4 form (P1 + P2, see sparse24.hip), on the
// sparse matrix-core instruction v_smfmac_i32_32x32x64_i8: per instruction and wave a 32 x 32 block
// of the output advances by 64 k, from 16 bytes of kept codes + 32 bits of positions per lane on
// the sparse side and 32 bytes per lane on the dense side.  Same structure as the dense
// persistent kernel (256 x 256 tile per workgroup, K staged 128 k at a time through two LDS stages
// filled by direct global -> LDS loads, one workgroup per compute unit walking several tiles) but
// EIGHT waves of 64 x 128 each: the sparse instruction takes its accumulator from ordinary vector
// registers only, and a 128 x 128 accumulator (256 registers) would leave none for anything else;
// with 128 per wave everything fits in 256 registers and two waves share a SIMD.  Per staged
// K-tile,
//   sparse operand: 256 rows x 64 bytes of codes (16-byte pieces XOR-swizzled with (row>>2)&3)
//                   + 256 rows x 16 bytes of position nibbles, each one contiguous piece of the
//                   K-tile-major layout the compaction pass writes,
//   dense operand:  256 rows x 128 bytes (pieces swizzled with (row>>1)&7),
// i.e. 52 KiB instead of 64 KiB, and half the matrix-core instructions.
// The overflow operand P2 (third and fourth code of a group of four k) has the same layout and
// its own 20 KiB per stage, but is staged and multiplied only where the flag word of the
// (block of 256 vectors, K-tile) says it holds something: bit 2 b + s for the 32 vectors b in
// step s.  The flag words of an output tile's band sit in LDS (one row of K / 128 words, fetched
// together with the tile's first K-tile, whose P2 is therefore staged unconditionally).  P1 and
// P2 feed the same accumulators, so the integer sums are those of the whole reduced operand and
// C comes out bit-identical to the dense execution.
// Accumulate mode only: C += dequant(product), optionally followed by alpha / beta.
// A launch carries one product or both correction terms of Algorithm 1 line 12:
//   product 0 (term 1, A'.RB):  the sparse operand's vectors are rows of C;
//   product 1 (term 2, RA.B'):  its vectors are the COLUMNS of C: the product is formed
//       transposed, B'^T . RA^T, and a lane adds four consecutive columns of one row of C.
// With both, a workgroup runs the two products of an output tile back to back, so that the tile
// of C the first one wrote is still in the caches when the second adds to it.
#include <type_traits>
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
constexpr int kP2 = kVals + kNibs + kDense;         // offset of the overflow operand inside a stage
constexpr int kStage = kP2 + kVals + kNibs;         // 72 KiB
constexpr int TM = 2, TN = 4;                       // 32 x 32 output blocks per wave (64 x 128)
constexpr int kThreads = 512;
constexpr int kLdsScales = 2 * kStage;              // float[BM + BN]
constexpr int kLdsFlags = kLdsScales + (BM + BN) * 4;   // 2 rows of flag words (two (tile, product) pairs in flight)
constexpr int kLdsBytes = kLdsFlags + 2 * kSparse24MaxKTiles * 4;
constexpr int kLoads = 9;                           // wave-wide loads per wave and staged K-tile

// The overflow products of one block of 32 vectors in one step of 64 k: if bit BIT of `flags` is
// set, read the block's P2 fragment from LDS (16 code bytes + 32 position bits per lane) and add
// its four products to the block's accumulators.  One piece of inline assembly with the test and
// the branch inside: to the compiler it is a straight-line instruction that updates the four
// accumulators in place, so it neither copies them around a conditional block nor keeps fragment
// registers alive across the loop.  A matrix-core result may not be touched by a
// non-matrix instruction for some cycles, and nothing inserts those wait states around inline
// assembly: the block ends with them.
template <int BIT, int CODES_OFF, int POS_OFF>
__device__ __forceinline__ void overflow_products(v16i& c0, v16i& c1, v16i& c2, v16i& c3, const v8i& d0,
                                                  const v8i& d1, const v8i& d2, const v8i& d3, uint32_t codes_addr,
                                                  uint32_t pos_addr, uint32_t flags) {
  v4i codes;
  int pos;
  asm volatile(
      "s_bitcmp0_b32 %[fl], %[bit]\n\t"
      "s_cbranch_scc1 .Lno_overflow%=\n\t"
      "ds_read_b128 %[codes], %[ca] offset:%[co]\n\t"
      "ds_read_b32 %[pos], %[pa] offset:%[po]\n\t"
      "s_waitcnt lgkmcnt(0)\n\t"
      "v_smfmac_i32_32x32x64_i8 %[c0], %[codes], %[d0], %[pos]\n\t"
      "v_smfmac_i32_32x32x64_i8 %[c1], %[codes], %[d1], %[pos]\n\t"
      "v_smfmac_i32_32x32x64_i8 %[c2], %[codes], %[d2], %[pos]\n\t"
      "v_smfmac_i32_32x32x64_i8 %[c3], %[codes], %[d3], %[pos]\n\t"
      "s_nop 15\n\t"
      "s_nop 3\n"
      ".Lno_overflow%=:"
      : [c0] "+v"(c0), [c1] "+v"(c1), [c2] "+v"(c2), [c3] "+v"(c3), [codes] "=&v"(codes), [pos] "=&v"(pos)
      : [d0] "v"(d0), [d1] "v"(d1), [d2] "v"(d2), [d3] "v"(d3), [ca] "v"(codes_addr), [pa] "v"(pos_addr),
        [fl] "s"(flags), [bit] "n"(BIT), [co] "n"(CODES_OFF), [po] "n"(POS_OFF)
      : "memory", "scc");
}

template <bool TRANS0, bool PAIR, bool SCALE>
__global__ __launch_bounds__(kThreads) void gemm_i8_sparse24_kernel(int64_t K, Sparse24Operand op0, Sparse24Operand op1,
                                                               int64_t tiles_m, int64_t tiles_n, GemmEpilogue ep) {
  extern __shared__ __attribute__((aligned(1024))) int8_t lds[];
  if (guard_tripped(ep)) return;                              // the whole grid leaves together
  float* sc_m = reinterpret_cast<float*>(lds + kLdsScales);   // scale of the sparse operand's vectors
  float* sc_n = sc_m + BM;                                    // scale of the dense operand's vectors
  const uint32_t* fl_lds = reinterpret_cast<const uint32_t*>(lds + kLdsFlags);
  const uint32_t lds0 = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) int8_t*)lds);

  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));                     // keeps per-thread offsets from being hoisted out of the tile loop
  // (the wave number is the same in every lane: saying so keeps everything derived from it,
  // the flag tests of the overflow operand above all, in scalar registers and scalar branches)
  // wave w of eight owns rows 64 (w / 2) .. +63 and columns 128 (w % 2) .. +127 of the tile
  const int lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6), wm = w >> 1, wn = w & 1;
  const int64_t total = tiles_m * tiles_n, G = gridDim.x, nk = K / BK;
  constexpr int nprod = PAIR ? 2 : 1;
  // tiles_m x tiles_n are the tiles of C; a product whose sparse vectors are columns of C takes its
  // band of the sparse operand from the tile's column and its dense rows from the tile's row
  auto trans_of = [&](int prod) { return PAIR ? prod == 1 : TRANS0; };

  // ---- loader.  Wave w fetches rows 32w .. 32w+31 of each operand tile (one block of 32 vectors).
  //  codes:     2 loads of 16 rows; lane l covers row 16j + l/4 and LDS slot l%4, which holds the
  //             logical piece (l%4) ^ ((row >> 2) & 3) = (l%4) ^ ((l >> 4) & 3)
  //  positions: the tile's 4 KiB are four word planes of 1 KiB (see sparse24.hip): waves 0-3
  //             fetch P1's plane w, waves 4-7 P2's plane w - 4 (if the flags say it holds anything)
  //  dense:     4 loads of 8 rows as in the dense kernel
  //  overflow:  the same 2 loads from P2's codes, only if the flags say block w holds anything
  // (the 2:4 operands are stored K-tile-major per block of 256 vectors: a staged tile is one
  // contiguous piece of memory, 64 resp. 16 bytes per vector)
  const int64_t goff_v = (int64_t)(lane >> 2) * (BK / 2) + 16 * ((lane & 3) ^ ((lane >> 4) & 3));
  const int64_t goff_n = (int64_t)lane * 16;        // the 4 KiB of nibbles of a tile are copied as they are
  const int lrow = lane >> 3;
  int64_t vba = blockIdx.x, kta = 0;                // cursor of the K-tile being fetched
  int proda = 0, orda = 0;                          // ... the product it belongs to, and the ordinal of its (tile, product)
  int64_t cur_ldb = 0, goff_b0 = 0, goff_b1 = 0;
  const int8_t *pv1, *pv2, *pb;
  const uint8_t *pn1, *pn2;
  const uint32_t* pfl;                              // flag row of the cursor's band
  auto point = [&]() {
    int64_t tm, tn;
    tile_of(vba, tiles_m, tiles_n, tm, tn);
    const Sparse24Operand& op = proda ? op1 : op0;
    const int64_t band = trans_of(proda) ? tn : tm, drow = trans_of(proda) ? tm : tn;
    const int64_t off_v = ((band * nk + kta) * BM + 32 * w) * (BK / 2);
    const int64_t off_n = (band * nk + kta) * kNibs + 1024 * (w & 3);
    pv1 = op.vals1 + off_v; pv2 = op.vals2 + off_v;
    pn1 = op.nib1 + off_n; pn2 = op.nib2 + off_n;
    pfl = op.flags + band * sparse24_flag_stride(K);
    cur_ldb = op.ldb;
    goff_b0 = (int64_t)lrow * cur_ldb + 16 * ((lane & 7) ^ ((lane >> 4) & 7));
    goff_b1 = (int64_t)lrow * cur_ldb + 16 * ((lane & 7) ^ (((lane >> 4) + 4) & 7));
    pb = op.Qb + (drow * BN + 32 * w) * cur_ldb + kta * BK;
  };
  auto advance = [&]() {
    if (kta + 1 < nk) {
      ++kta;
      pv1 += BM * (BK / 2); pv2 += BM * (BK / 2);
      pn1 += BM * (BK / 8); pn2 += BM * (BK / 8);
      pb += BK;
    } else if (proda + 1 < nprod) {
      ++proda; ++orda;
      kta = 0;
      point();
    } else if (vba + G < total) {
      vba += G;
      proda = 0; ++orda;
      kta = 0;
      point();
    }                                               // else stay on the last K-tile (harmless re-fetch)
  };
  // load i (0..8) of the K-tile at the cursor into LDS buffer `stage`; fl = flag word of that
  // K-tile (all ones for the first K-tile of a tile, whose flag row is fetched alongside)
  auto issue_load = [&](int stage, int i, uint32_t fl) {
    // (wave-uniform by construction; readfirstlane tells the compiler so: the addresses feed M0)
    const uint32_t base = lds0 + stage * kStage;
    const uint32_t lv = __builtin_amdgcn_readfirstlane(base + (32 * w) * (BK / 2));
    const uint32_t ln = __builtin_amdgcn_readfirstlane(base + kVals + 1024 * (w & 3));
    const uint32_t lb = __builtin_amdgcn_readfirstlane(base + kVals + kNibs + (32 * w) * BK);
    if (i < 2) {
      load_to_lds(pv1 + (16 * i) * (BK / 2) + goff_v, lv + 16 * i * (BK / 2));
    } else if (i == 2) {
      if (w < 4) {
        load_to_lds(reinterpret_cast<const int8_t*>(pn1 + goff_n), ln);
      } else if (fl & (0x5555u << ((w & 3) >> 1))) {
        // plane w - 4 of P2's positions: step (w - 4) / 2, all eight blocks
        load_to_lds(reinterpret_cast<const int8_t*>(pn2 + goff_n), ln + kP2);
      }
    } else if (i < 7) {
      const int j = i - 3;
      load_to_lds(pb + (int64_t)(8 * j) * cur_ldb + ((j & 1) ? goff_b1 : goff_b0), lb + 8 * j * BK);
    } else {
      // rows 32w + 16j .. +15 of P2's codes: block w
      const int j = i - 7;
      if ((fl >> (2 * w)) & 3u)
        load_to_lds(pv2 + (16 * j) * (BK / 2) + goff_v, lv + kP2 + 16 * j * (BK / 2));
    }
  };
  // the flag row of the cursor's band (wave 0 fetches it with the tile's first K-tile): 1 KiB,
  // K / 128 of its words are flags (the array is padded so that the whole read is in bounds)
  auto issue_flag_row = [&]() {
    if (w == 0)
      load_to_lds(reinterpret_cast<const int8_t*>(pfl) + goff_n,
                  __builtin_amdgcn_readfirstlane(lds0 + kLdsFlags + (orda & 1) * kSparse24MaxKTiles * 4));
  };
  auto issue_loads_first = [&](int stage) {         // a tile's first K-tile: everything, and the flag row
#pragma unroll
    for (int i = 0; i < kLoads; ++i) issue_load(stage, i, 0xffffu);
    issue_flag_row();
  };

  // ---- fragment reads of lane (frow, kh) at step s of a K-tile (64 k per step)
  const int frow = lane & 31, kh = lane >> 5;
  const int key_v = (frow >> 2) & 3, key_b = (frow >> 1) & 7;
  const int v_row = (wm * 64 + frow) * (BK / 2);
  // (position words: plane-major, vectors of the odd planes rotated by 32; plane = 2 step + kh)
  const int n_row = kVals + 4 * ((wm * 64 + frow) ^ (32 * kh));
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
  v16i acc[TM][TN];
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0;

  // overflow fragments of block t at `step` live at the same offsets inside the P2 part of a stage;
  // LDS addresses for overflow_products (block t adds t * 32 * 64 bytes to the codes' address and
  // 128 * (t & ~1) to the positions', whose row is rotated for odd t)
  auto p2_codes_addr = [&](int stage, int step) { return lds0 + stage * kStage + kP2 + v_row + xv[step]; };
  auto p2_pos_addr = [&](int stage, int step, int odd) {
    return lds0 + stage * kStage + kP2 + (n_row ^ (4 * 32 * odd)) + xn[step];
  };
  // block T of the wave's two, step STEP of the K-tile staged in `stage`; fw: the K-tile's flag
  // word shifted so that bit 2 t + step belongs to the wave's block t
  auto overflow_block = [&](auto t_tag, auto step_tag, int stage, uint32_t fw, const v8i (&d)[TN]) {
    constexpr int T = decltype(t_tag)::value, STEP = decltype(step_tag)::value;
    overflow_products<2 * T + STEP, T * 32 * (BK / 2), 0>(
        acc[T][0], acc[T][1], acc[T][2], acc[T][3], d[0], d[1], d[2], d[3], p2_codes_addr(stage, STEP),
        p2_pos_addr(stage, STEP, T & 1), fw);
  };

  // ---- the output tile and product being multiplied
  int64_t vb = blockIdx.x, tile_m, tile_n;
  tile_of(vb, tiles_m, tiles_n, tile_m, tile_n);
  int prod = 0, ord = 0;
  auto scales_of = [&](float& sm, float& sn) {
    const bool tr = trans_of(prod);
    const float* s_row = prod ? op1.s_row : ep.s_row;
    const float* s_col = prod ? op1.s_col : ep.s_col;
    // sparse-side vectors are columns of C when transposed
    // (threads 0-255 fetch the sparse side's scales, 256-511 the dense side's)
    const int t = tid & 255;
    const bool dense_side = tid >= 256;
    const bool from_cols = tr != dense_side;        // sparse vectors are columns of C when transposed
    sm = from_cols ? s_col[tile_n * BN + t] : s_row[tile_m * BM + t];
    sn = sm;
  };
  float sreg_m, sreg_n;
  scales_of(sreg_m, sreg_n);

  // flag word of the K-tile at the cursor, as the loader wants it
  auto cursor_flags = [&]() -> uint32_t {
    if (kta == 0) return 0xffffu;
    return __builtin_amdgcn_readfirstlane(fl_lds[(orda & 1) * kSparse24MaxKTiles + kta]);
  };

  point();
  issue_loads_first(0);
  advance();
  wait_loads();
  __syncthreads();
  {
    // second K-tile of the stream (or, if K is a single K-tile, the first of the next tile)
    const uint32_t fl = cursor_flags();
    if (kta == 0) {
      issue_loads_first(1);
    } else {
#pragma unroll
      for (int i = 0; i < kLoads; ++i) issue_load(1, i, fl);
    }
  }
  advance();
  fread(0, 0, 0);
  uint32_t fc = __builtin_amdgcn_readfirstlane(fl_lds[0]);   // flags of the K-tile being multiplied (ordinal 0, K-tile 0)

  const int64_t my_tiles = (total - blockIdx.x + G - 1) / G;
  int g = 0;                                        // parity of the K-tile stream across tiles
  typedef std::integral_constant<int, 0> I0;
  typedef std::integral_constant<int, 1> I1;
  for (int64_t tile = 0; tile < my_tiles * nprod; ++tile) {
    for (int64_t kt = 0; kt < nk; ++kt, ++g) {
      const int cur = g & 1;
      const uint32_t fw = fc >> (4 * wm);           // bit 2 t + step: the wave's block t
      // step 0: the fragments of step 1 are read while step 0 multiplies.  The overflow products
      // of a block of 32 vectors follow its four regular ones at once (same accumulators).
      fread(cur, 1, 1);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int b = 0; b < TN; ++b)
        acc[0][b] = __builtin_amdgcn_smfmac_i32_32x32x64_i8(fa[0][0], fb[0][b], acc[0][b], fi[0][0], 0, 0);
      overflow_block(I0(), I0(), cur, fw, fb[0]);
#pragma unroll
      for (int b = 0; b < TN; ++b)
        acc[1][b] = __builtin_amdgcn_smfmac_i32_32x32x64_i8(fa[0][1], fb[0][b], acc[1][b], fi[0][1], 0, 0);
      overflow_block(I1(), I0(), cur, fw, fb[0]);
      __builtin_amdgcn_sched_barrier(0);
      // the overflow products of step 1 come before its regular ones: their fragments must be
      // read from buffer `cur` before the barrier below hands it to the loader
      overflow_block(I0(), I1(), cur, fw, fb[1]);
      overflow_block(I1(), I1(), cur, fw, fb[1]);
      __builtin_amdgcn_sched_barrier(0);
      // step 1: K-tile g+1 (loads issued one whole K-tile ago) must have landed; after the
      // barrier everybody is also done reading buffer `cur`, which takes K-tile g+2
      wait_loads();
      __syncthreads();
      fread(cur ^ 1, 0, 0);
      // flag words: of the K-tile at the load cursor, and of the K-tile multiplied next
      const uint32_t fl = cursor_flags();
      const bool first_of_tile = kta == 0;
      const bool last_kt = kt + 1 == nk;
      const int ord_next = last_kt ? ord + 1 : ord;
      const uint32_t fc_next =
          __builtin_amdgcn_readfirstlane(fl_lds[(ord_next & 1) * kSparse24MaxKTiles + (last_kt ? 0 : kt + 1)]);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b) {
          acc[a][b] = __builtin_amdgcn_smfmac_i32_32x32x64_i8(fa[1][a], fb[1][b], acc[a][b], fi[1][a], 0, 0);
          const int i = a * TN + b;
          issue_load(cur, i, fl);
          if (i + TM * TN < kLoads) issue_load(cur, i + TM * TN, fl);
          __builtin_amdgcn_sched_barrier(0);
        }
      if (first_of_tile) issue_flag_row();
      fc = fc_next;
      advance();
    }

    // ================= epilogue of tile (tile_m, tile_n), product `prod`; tiles are full
    sc_m[tid] = sreg_m;                             // (sc_n follows sc_m: thread 256 + t writes sc_n[t])
    __syncthreads();
    const int64_t m0 = tile_m * BM, n0 = tile_n * BN;
    const int half = lane >> 5, cl = lane & 31;
    const int cbase = wn * (BN / 2) + cl;           // dense-side vector of this lane, plus 32 b
    const bool do_scale = SCALE && prod == nprod - 1;
    float scn[TN];
#pragma unroll
    for (int b = 0; b < TN; ++b) scn[b] = sc_n[cbase + b * 32];
    // C goes around the caches, except between the two products of a pair: the first leaves its
    // tile cached for the second
    auto bands = [&](auto trans_tag, auto cached_load_tag, auto cached_store_tag) {
    constexpr bool TR = decltype(trans_tag)::value, CLOAD = decltype(cached_load_tag)::value,
                   CSTORE = decltype(cached_store_tag)::value;
#pragma unroll
    for (int a = 0; a < TM; ++a) {
      const int rbase = wm * 64 + a * 32 + 4 * half;         // sparse-side vector, plus 8 (v>>2) + (v&3)
      if (!TR) {
        // C[m0 + row][n0 + col]: a lane adds to one column, rows 8 (v>>2) + (v&3)
        float* cband = ep.C + (m0 + rbase) * ep.ldc + n0 + cbase;
        float x[TN][16];
#pragma unroll
        for (int v = 0; v < 16; ++v)
#pragma unroll
          for (int b = 0; b < TN; ++b) {
            const float* src = &cband[(int64_t)(8 * (v >> 2) + (v & 3)) * ep.ldc + b * 32];
            x[b][v] = CLOAD ? *src : __builtin_nontemporal_load(src);
          }
        const bool has_beta = SCALE && do_scale && ep.beta != 0.f;
        float cin[TN][16];                            // the band of Cin, all loads in flight at once
        if (has_beta) {
          const float* cinband = ep.Cin + (m0 + rbase) * ep.ldcin + n0 + cbase;
#pragma unroll
          for (int v = 0; v < 16; ++v)
#pragma unroll
            for (int b = 0; b < TN; ++b)
              cin[b][v] = __builtin_nontemporal_load(&cinband[(int64_t)(8 * (v >> 2) + (v & 3)) * ep.ldcin + b * 32]);
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int ro = 8 * (v >> 2) + (v & 3);
          const float sm = sc_m[rbase + ro];
#pragma unroll
          for (int b = 0; b < TN; ++b) {
            float out = x[b][v] + (float)acc[a][b][v] * (sm * scn[b]);
            if (SCALE && do_scale) {
              out = ep.alpha * out;
              if (has_beta) out = out + ep.beta * cin[b][v];
            }
            if (CSTORE) cband[(int64_t)ro * ep.ldc + b * 32] = out;
            else __builtin_nontemporal_store(out, &cband[(int64_t)ro * ep.ldc + b * 32]);
            acc[a][b][v] = 0;
          }
        }
      } else {
        // C[m0 + col][n0 + row]: the four rows (v&3) of the product are four consecutive columns of C
        typedef float f4v __attribute__((ext_vector_type(4)));
#pragma unroll
        for (int b = 0; b < TN; ++b) {
          const int64_t ci = m0 + cbase + b * 32;                        // row of C
          f4v x[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const f4v* src = reinterpret_cast<const f4v*>(ep.C + ci * ep.ldc + n0 + rbase + 8 * q);
            x[q] = CLOAD ? *src : __builtin_nontemporal_load(src);
          }
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            f4v o = x[q];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
              // (the scale product is taken row scale of C first, as everywhere else)
              float out = o[t] + (float)acc[a][b][4 * q + t] * (scn[b] * sc_m[rbase + 8 * q + t]);
              if (SCALE && do_scale) {
                out = ep.alpha * out;
                if (ep.beta != 0.f) out = out + ep.beta * ep.Cin[ci * ep.ldcin + n0 + rbase + 8 * q + t];
              }
              o[t] = out;
              acc[a][b][4 * q + t] = 0;
            }
            f4v* dst = reinterpret_cast<f4v*>(ep.C + ci * ep.ldc + n0 + rbase + 8 * q);
            if (CSTORE) *dst = o;
            else __builtin_nontemporal_store(o, dst);
          }
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    };
    if (PAIR) {
      if (prod == 0) bands(std::false_type(), std::false_type(), std::true_type());
      else bands(std::true_type(), std::true_type(), std::false_type());
    } else {
      bands(std::integral_constant<bool, TRANS0>(), std::false_type(), std::false_type());
    }
    // next product of this tile, or the next output tile of this workgroup
    ++ord;
    if (prod + 1 < nprod) {
      prod = 1;
      scales_of(sreg_m, sreg_n);
    } else {
      prod = 0;
      vb += G;
      if (vb < total) {
        tile_of(vb, tiles_m, tiles_n, tile_m, tile_n);
        scales_of(sreg_m, sreg_n);
      }
    }
    // (sc_m / sc_n are rewritten by the next epilogue: a whole K loop and its barriers lie between)
  }
  wait_loads();                                     // nothing may still be writing LDS when the wave ends
}

}  // namespace

// One product: M x N = rows x columns of C.  op.Qb: the dense operand, K-contiguous, N rows
// (trans: M rows) of leading dimension op.ldb.  The sparse operand has M (trans: N) vectors.
bool gemm_sparse24_ok(int64_t M, int64_t N, int64_t K, const Sparse24Operand& op, bool trans, const GemmEpilogue& ep) {
  if (ep.D_int || ep.D_F_copy) return false;
  if (M <= 0 || N <= 0 || K <= 0 || (M % BM) || (N % BN) || (K % BK)) return false;
  if (K / BK > kSparse24MaxKTiles) return false;             // one flag row must fit one wave-wide load
  const uintptr_t bits = reinterpret_cast<uintptr_t>(op.vals1) | reinterpret_cast<uintptr_t>(op.nib1) |
                         reinterpret_cast<uintptr_t>(op.vals2) | reinterpret_cast<uintptr_t>(op.nib2) |
                         reinterpret_cast<uintptr_t>(op.flags) | reinterpret_cast<uintptr_t>(op.Qb);
  if ((bits & 15) || (op.ldb % 16)) return false;
  // the transposed epilogue adds to C sixteen bytes at a time
  if (trans && ((reinterpret_cast<uintptr_t>(ep.C) & 15) || (ep.ldc % 4))) return false;
  return true;
}

// second == null: one product (op, trans); else both terms of a pair: op = term 1 (not
// transposed, scales ep.s_row / ep.s_col), *second = term 2 (transposed, its own scales)
hipError_t launch_gemm_i8_sparse24(int64_t M, int64_t N, int64_t K, const Sparse24Operand& op, bool trans,
                                   const Sparse24Operand* second, const GemmEpilogue& ep, hipStream_t st) {
  int num_cu = 0;
  hipError_t e = gemm_device_cus(&num_cu);
  if (e != hipSuccess) return e;
  const int64_t tm = M / BM, tn = N / BN;
  int64_t wgs = num_cu / 8 * 8;                              // one workgroup per CU, a multiple of the 8 XCDs
  if (wgs < 8) wgs = 8;
  if (wgs > tm * tn) wgs = tm * tn;
  const bool scale = ep.final_scale != 0;
  void (*kern)(int64_t, Sparse24Operand, Sparse24Operand, int64_t, int64_t, GemmEpilogue);
  if (second)
    kern = scale ? gemm_i8_sparse24_kernel<false, true, true> : gemm_i8_sparse24_kernel<false, true, false>;
  else
    kern = trans ? (scale ? gemm_i8_sparse24_kernel<true, false, true> : gemm_i8_sparse24_kernel<true, false, false>)
                 : (scale ? gemm_i8_sparse24_kernel<false, false, true> : gemm_i8_sparse24_kernel<false, false, false>);
  e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), kLdsBytes);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3((unsigned)wgs), dim3(kThreads), kLdsBytes, st, K, op, second ? *second : op, tm, tn,
                     ep);
  return hipGetLastError();
}

}  // namespace srq
