// 2:4-structured execution of a sparse correction product (Algorithm 1 line 12 on the sparse
// matrix cores; the structured-sparsity direction of the paper's closing section).
//
// compress24_kernel splits the zero-filled INT8 expansion of a reduced operand (vector-major,
// K contiguous) into
//   * a 2:4 operand: of every four consecutive k the first two non-zero codes, as two bytes,
//     plus their positions inside the group as one nibble (first position in bits 1:0, second
//     in bits 3:2).  A group with fewer than two non-zeros is padded with zero-valued slots;
//   * a spill list: the third and fourth non-zero of a group, as (index, value) pairs of the
//     vector, with explicit begin / end offsets per vector (vectors reserve their piece of the
//     list with one atomic add, so pieces follow each other in no particular order; inside a
//     piece the indices ascend).
// Layout of the 2:4 operand: K-tile-major inside blocks of 256 vectors, the unit the matrix-core
// kernel stages: the 64 code bytes (16 nibble bytes) that vector v holds for the K-tile t of
// 128 k sit at ((v / 256) * (kc / 128) + t) * 256 * 64 + (v % 256) * 64, so that one staged tile
// is one contiguous 16 KiB piece of memory; the 4 KiB of nibbles of a tile are stored as four
// planes of 256 32-bit words, plane c holding the positions of code bytes 16c .. 16c+15 of every
// vector, vector r at word r ^ 32 in the odd planes (the 64 lanes of a wave, which read the
// words of 32 consecutive vectors from two neighbouring planes, then hit 64 different LDS
// banks).  The vector count is padded to a multiple of 256 by the caller's buffers.
// Byte order of the 2:4 operand inside every block of 64 k: the four groups of k 0-15, then
// those of k 32-47, 16-31, 48-63 (eight bytes each; the nibbles in the same order).  This is
// the order in which v_smfmac_i32_32x32x64_i8 consumes them: the lane that holds row r and
// half h of a 64-k block takes sixteen consecutive bytes, of which the first eight pair with
// k 16h .. 16h+15 of the dense operand and the last eight with k 32+16h .. 32+16h+15.
#include "srq_internal.h"

namespace srq {
namespace {

// one wave per vector, sixteen codes (four groups) per lane and step
__global__ __launch_bounds__(256) void compress24_kernel(const int8_t* __restrict__ dense, int64_t ldd,
                                                         int64_t nvec, int64_t kc,       // kc: multiple of 128
                                                         int8_t* __restrict__ vals,
                                                         uint8_t* __restrict__ nib,
                                                         int32_t* __restrict__ sp_begin,
                                                         int32_t* __restrict__ sp_end,
                                                         int32_t* __restrict__ sp_idx, int8_t* __restrict__ sp_val,
                                                         int64_t sp_capacity,
                                                         unsigned long long* __restrict__ sp_total) {
  const int lane = threadIdx.x & 63;
  const int64_t v = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (v >= nvec) return;                                           // whole waves leave together
  const int8_t* src = dense + v * ldd;
  typedef unsigned u4v __attribute__((ext_vector_type(4)));
  auto spills_of = [](const u4v& w) {
    const unsigned g[4] = {w.x, w.y, w.z, w.w};
    int extra = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int nz = ((g[q] & 0xffu) != 0) + ((g[q] & 0xff00u) != 0) + ((g[q] & 0xff0000u) != 0) +
                     ((g[q] & 0xff000000u) != 0);
      extra += nz > 2 ? nz - 2 : 0;
    }
    return extra;
  };
  // vectors of up to 8192 codes are read once and held in registers (all loads in flight
  // together); longer ones are read twice
  constexpr int kHeld = 8;
  const bool held = kc <= 1024 * kHeld;
  u4v wreg[kHeld];
  // pass 1: how many entries of this vector spill
  int extra = 0;
  if (held) {
#pragma unroll
    for (int it = 0; it < kHeld; ++it) {
      const int64_t k0 = 16 * lane + 1024 * it;
      wreg[it] = u4v{0u, 0u, 0u, 0u};
      if (k0 < kc) wreg[it] = *reinterpret_cast<const u4v*>(src + k0);
    }
#pragma unroll
    for (int it = 0; it < kHeld; ++it) extra += spills_of(wreg[it]);
  } else {
    for (int64_t k0 = 16 * lane; k0 < kc; k0 += 1024) extra += spills_of(*reinterpret_cast<const u4v*>(src + k0));
  }
  int total = extra;
  for (int off = 32; off > 0; off >>= 1) total += __shfl_xor(total, off, 64);
  // the vector's piece of the spill list
  unsigned long long base = 0;
  if (lane == 0) {
    base = total ? atomicAdd(sp_total, (unsigned long long)total) : 0ull;
    const long long b = (long long)base < (long long)sp_capacity ? (long long)base : (long long)sp_capacity;
    const long long e = (long long)(base + total) < (long long)sp_capacity ? (long long)(base + total)
                                                                            : (long long)sp_capacity;
    sp_begin[v] = (int32_t)b;
    sp_end[v] = (int32_t)e;
  }
  base = __shfl((long long)base, 0, 64);
  int64_t pos = (int64_t)base;                                     // next free slot of this vector's piece
  // pass 2: one step of 1024 codes (sixteen per lane)
  auto step = [&](int64_t k0, const u4v& w) {
    const bool in = k0 < kc;
    const unsigned g[4] = {w.x, w.y, w.z, w.w};
    unsigned out_lo = 0, out_hi = 0, nibs = 0;
    int mine = 0;                                                  // spilled entries of this lane in this step
    unsigned spill_pos = 0;                                        // up to 8 entries: 4-bit offsets
    // (a lane spills at most 2 per group, 8 per step: offsets inside its 16 codes, 4 bits each;
    //  values kept in two words)
    unsigned sv0 = 0, sv1 = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      // positions of the non-zero codes of the group, lowest first (bit tricks: no indexed array)
      const unsigned m = ((g[q] & 0xffu) ? 1u : 0u) | ((g[q] & 0xff00u) ? 2u : 0u) |
                         ((g[q] & 0xff0000u) ? 4u : 0u) | ((g[q] & 0xff000000u) ? 8u : 0u);
      const unsigned m1 = m & (m - 1u), m2 = m1 & (m1 - 1u);
      int p0 = m ? __ffs((int)m) - 1 : 0;
      int p1 = m1 ? __ffs((int)m1) - 1 : 3;
      if (!m) p1 = 1;                               // empty group: slots (0, 1), both zero
      else if (!m1 && p0 == 3) p0 = 0;              // single non-zero at 3: slots (0, 3); else (p0, 3)
      const unsigned v0 = (g[q] >> (8 * p0)) & 0xffu, v1 = (g[q] >> (8 * p1)) & 0xffu;
      const unsigned pair = v0 | (v1 << 8);
      if (q < 2) out_lo |= pair << (16 * q); else out_hi |= pair << (16 * (q - 2));
      nibs |= (unsigned)(p0 | (p1 << 2)) << (4 * q);
      unsigned rest = m2;                           // third and fourth non-zero spill
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        if (rest) {
          const int pe = __ffs((int)rest) - 1;
          rest &= rest - 1u;
          const unsigned val = (g[q] >> (8 * pe)) & 0xffu;
          spill_pos |= (unsigned)(4 * q + pe) << (4 * mine);
          if (mine < 4) sv0 |= val << (8 * mine); else sv1 |= val << (8 * (mine - 4));
          ++mine;
        }
      }
    }
    if (in) {
      // where this lane's sixteen k sit inside their block of 64
      const int64_t blk = k0 >> 6;
      const int sub = (int)((k0 >> 4) & 3);
      const int ord = sub == 0 ? 0 : sub == 2 ? 1 : sub == 1 ? 2 : 3;
      typedef unsigned u2v __attribute__((ext_vector_type(2)));
      const u2v o = {out_lo, out_hi};
      // K-tile t = blk / 2 of this vector's block of 256 vectors; half (blk & 1) of its 64 bytes
      const int64_t tile = (v >> 8) * (kc >> 7) + (blk >> 1);
      const int64_t in_tile = v & 255;
      *reinterpret_cast<u2v*>(vals + (tile * 256 + in_tile) * 64 + 32 * (blk & 1) + 8 * ord) = o;
      // positions: word c = 2 (blk & 1) + ord / 2 of the vector, stored word-plane-major with the
      // vectors of the odd planes rotated by 32 (see the layout note above)
      const int c = 2 * (int)(blk & 1) + (ord >> 1);
      const int64_t word = c * 256 + (in_tile ^ ((c & 1) << 5));
      *reinterpret_cast<uint16_t*>(nib + tile * 4096 + 4 * word + 2 * (ord & 1)) = (uint16_t)nibs;
    }
    if (!total) return;                                            // (wave-uniform) nothing of this vector spills
    // spilled entries in ascending k: lanes in order, then position
    int incl = mine;
    for (int d = 1; d < 64; d <<= 1) {
      const int y = __shfl_up(incl, d, 64);
      if (lane >= d) incl += y;
    }
    int64_t p = pos + incl - mine;
    pos += __shfl(incl, 63, 64);
    for (int e = 0; e < mine; ++e) {
      if (p < sp_capacity) {
        sp_idx[p] = (int32_t)(k0 + ((spill_pos >> (4 * e)) & 0xfu));
        sp_val[p] = (int8_t)((e < 4 ? sv0 >> (8 * e) : sv1 >> (8 * (e - 4))) & 0xffu);
      }
      ++p;
    }
  };
  if (held) {
#pragma unroll
    for (int it = 0; it < kHeld; ++it)
      if ((int64_t)1024 * it < kc) step(16 * lane + 1024 * it, wreg[it]);
  } else {
    for (int64_t k0 = 16 * lane; k0 - 16 * lane < kc; k0 += 1024) {
      u4v w = {0u, 0u, 0u, 0u};
      if (k0 < kc) w = *reinterpret_cast<const u4v*>(src + k0);
      step(k0, w);
    }
  }
}

}  // namespace

// dense: nvec x kc zero-filled codes (ld = ldd, 16-byte aligned rows; kc a multiple of 128);
// vals: ceil(nvec / 256) * 256 * kc / 2 bytes, nib: ... * kc / 8 bytes, in the tiled layout above;
// *sp_total must be zero on entry and holds the number of spilled entries afterwards (which may
// exceed sp_capacity: entries past the capacity are dropped and the per-vector ranges clipped)
hipError_t launch_compress24(const int8_t* dense, int64_t ldd, int64_t nvec, int64_t kc, int8_t* vals,
                             uint8_t* nib, int32_t* sp_begin, int32_t* sp_end, int32_t* sp_idx,
                             int8_t* sp_val, int64_t sp_capacity, unsigned long long* sp_total, hipStream_t st) {
  if (nvec <= 0 || kc <= 0) return hipSuccess;
  hipLaunchKernelGGL(compress24_kernel, dim3((unsigned)((nvec + 3) / 4)), dim3(256), 0, st, dense, ldd, nvec, kc,
                     vals, nib, sp_begin, sp_end, sp_idx, sp_val, sp_capacity, sp_total);
  return hipGetLastError();
}

}  // namespace srq
