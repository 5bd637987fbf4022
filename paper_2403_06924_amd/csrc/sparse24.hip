// 2:4-structured form of a reduced operand, written straight from the keep-mask by the
// compaction pass (Algorithm 1 lines 8-10 emitting, next to the CSR / CSC arrays, the operand of
// line 12 in the layout the sparse matrix-core instruction consumes; the structured-sparsity
// direction of the paper's closing section).
//
// Every group of four consecutive k of a vector holds at most four kept, non-zero codes.  They
// are split over TWO operands of 2:4 form:
//   P1: the first two non-zero codes of the group,
//   P2: the third and fourth, if any (an unstructured operand of density d overflows "two of
//       four" in about 4 d^3 of its groups).
// Each operand stores per group two code bytes plus one nibble of positions (first position in
// bits 1:0, second in bits 3:2; missing codes are zero-valued slots with distinct positions).
// A' = P1 + P2 exactly, so A'.R = P1.R + P2.R in integers.  P2 is almost empty: a bit per
// (block of 32 vectors, step of 64 k) says whether P2 holds anything there, and the product
// kernel stages and multiplies P2 only where it does.
//
// Layout of either operand: K-tile-major inside blocks of 256 vectors, the unit the matrix-core
// kernel stages: the 64 code bytes (16 nibble bytes) that vector v holds for the K-tile t of
// 128 k sit at ((v / 256) * (kc / 128) + t) * 256 * 64 + (v % 256) * 64, so that one staged tile
// is one contiguous 16 KiB piece of memory; the 4 KiB of nibbles of a tile are stored as four
// planes of 256 32-bit words, plane c holding the positions of code bytes 16c .. 16c+15 of every
// vector, vector r at word r ^ 32 in the odd planes (the 64 lanes of a wave, which read the
// words of 32 consecutive vectors from two neighbouring planes, then hit 64 different LDS
// banks).  The vector count is a multiple of 256.
// Byte order inside every block of 64 k: the four groups of k 0-15, then those of k 32-47,
// 16-31, 48-63 (eight bytes each; the nibbles in the same order).  This is the order in which
// v_smfmac_i32_32x32x64_i8 consumes them: the lane that holds row r and half h of a 64-k block
// takes sixteen consecutive bytes, of which the first eight pair with k 16h .. 16h+15 of the
// dense operand and the last eight with k 32+16h .. 32+16h+15.
// Flags: one 32-bit word per (block of 256 vectors, K-tile), rows of sparse24_flag_stride(kc)
// words per block; bit 2 * (vector % 256 / 32) + step is set when P2 is non-empty for those 32
// vectors in step (k / 64) % 2 of the K-tile.
#include "srq_internal.h"

namespace srq {
namespace {

// two codes + position nibble of one group from the positions in `m` (bit p: code p is taken),
// lowest two first; fewer than two: zero-valued slots at distinct positions
__device__ __forceinline__ void pick_two(unsigned g, unsigned m, unsigned& pair, unsigned& nib) {
  const unsigned m1 = m & (m - 1u);
  int p0 = m ? __ffs((int)m) - 1 : 0;
  int p1 = m1 ? __ffs((int)m1) - 1 : 3;
  if (!m) p1 = 1;                               // empty: slots (0, 1), both zero
  else if (!m1 && p0 == 3) p0 = 0;              // single code at 3: slots (0, 3); else (p0, 3)
  // (a slot that names a position whose code is not taken must read as zero)
  const unsigned v0 = ((m >> p0) & 1u) ? (g >> (8 * p0)) & 0xffu : 0u;
  const unsigned v1 = ((m >> p1) & 1u) ? (g >> (8 * p1)) & 0xffu : 0u;
  pair = v0 | (v1 << 8);
  nib = (unsigned)(p0 | (p1 << 2));
}

// One block per vector, a quarter of the vector's kc codes per wave, sixteen codes per lane and
// step (one 16-byte code load, one 16-bit piece of the mask).  Emits the compressed arrays as
// scatter_mask16_kernel does, and P1 / P2 / flags as described above.  Reads the codes up to kc:
// the columns past veclen hold zeros, and so do the mask bits.
__global__ __launch_bounds__(256) void scatter24_kernel(const uint64_t* __restrict__ mask, int64_t words,
                                                        int64_t veclen, int64_t kc, const int8_t* __restrict__ Q,
                                                        int64_t ldq, const int32_t* __restrict__ ptr,
                                                        int32_t* __restrict__ idx, int8_t* __restrict__ val,
                                                        int64_t capacity, int8_t* __restrict__ vals1,
                                                        uint8_t* __restrict__ nib1, int8_t* __restrict__ vals2,
                                                        uint8_t* __restrict__ nib2, uint32_t* __restrict__ flags) {
  __shared__ int wsum[4];
  const int64_t v = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const uint16_t* mv16 = reinterpret_cast<const uint16_t*>(mask + v * words);
  const uint64_t* mv = mask + v * words;
  const int8_t* qv = Q + v * ldq;                        // 16-byte aligned (checked by the launcher)
  const int64_t nchunks = (kc + 1023) >> 10;
  const int64_t cpw = (nchunks + 3) >> 2;
  const int64_t c0 = w * cpw < nchunks ? w * cpw : nchunks;
  const int64_t c1 = c0 + cpw < nchunks ? c0 + cpw : nchunks;
  int mine = 0;
  for (int64_t i = c0 * 16 + lane; i < c1 * 16 && i < words; i += 64) {
    uint64_t m = mv[i];
    const int64_t left = veclen - i * 64;                 // bits at and past veclen do not count
    if (left < 64) m &= left > 0 ? (1ull << left) - 1ull : 0ull;
    mine += __popcll(m);
  }
  for (int off = 32; off > 0; off >>= 1) mine += __shfl_xor(mine, off, 64);
  if (lane == 0) wsum[w] = mine;
  __syncthreads();
  int64_t pos = ptr[v];
  for (int i = 0; i < w; ++i) pos += wsum[i];
  const uint64_t lower = (1ull << lane) - 1ull;
  const int64_t in_tile = v & 255, band = v >> 8, nk = kc >> 7;
  typedef unsigned u4v __attribute__((ext_vector_type(4)));
  typedef unsigned u2v __attribute__((ext_vector_type(2)));
  for (int64_t c = c0; c < c1; ++c) {
    const int64_t e = c * 1024 + 16 * lane;
    const bool in = e < kc;                               // kc is a multiple of 16
    const int64_t left = veclen - e;
    unsigned m = 0;
    if (left > 0) {
      m = mv16[e >> 4];
      if (left < 16) m &= (1u << left) - 1u;
    }
    unsigned cw[4] = {0u, 0u, 0u, 0u};
    if (in) {
      const u4v t = *reinterpret_cast<const u4v*>(qv + e);
      cw[0] = t.x; cw[1] = t.y; cw[2] = t.z; cw[3] = t.w;
    }
    if (in) {
      unsigned lo1 = 0, hi1 = 0, n1 = 0, lo2 = 0, hi2 = 0, n2 = 0;
      bool spill = false;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const unsigned g = cw[q];
        // kept AND non-zero codes of the group (a kept zero code adds nothing to any product)
        const unsigned keep = (m >> (4 * q)) & 0xfu;
        const unsigned nz = ((g & 0xffu) ? 1u : 0u) | ((g & 0xff00u) ? 2u : 0u) | ((g & 0xff0000u) ? 4u : 0u) |
                            ((g & 0xff000000u) ? 8u : 0u);
        const unsigned mk = keep & nz;
        const unsigned first = mk & (0u - mk), r1 = mk & (mk - 1u), second = r1 & (0u - r1);
        const unsigned m_p1 = first | second, m_p2 = mk & ~m_p1;
        unsigned pair, nb;
        pick_two(g, m_p1, pair, nb);
        if (q < 2) lo1 |= pair << (16 * q); else hi1 |= pair << (16 * (q - 2));
        n1 |= nb << (4 * q);
        pick_two(g, m_p2, pair, nb);
        if (q < 2) lo2 |= pair << (16 * q); else hi2 |= pair << (16 * (q - 2));
        n2 |= nb << (4 * q);
        spill |= m_p2 != 0u;
      }
      // where this lane's sixteen k sit inside their block of 64
      const int64_t blk = e >> 6;
      const int sub = (int)((e >> 4) & 3);
      const int ord = sub == 0 ? 0 : sub == 2 ? 1 : sub == 1 ? 2 : 3;
      const int64_t tile = band * nk + (blk >> 1);
      const int64_t voff = (tile * 256 + in_tile) * 64 + 32 * (blk & 1) + 8 * ord;
      const int cpl = 2 * (int)(blk & 1) + (ord >> 1);
      const int64_t noff = tile * 4096 + 4 * (cpl * 256 + (in_tile ^ ((cpl & 1) << 5))) + 2 * (ord & 1);
      *reinterpret_cast<u2v*>(vals1 + voff) = u2v{lo1, hi1};
      *reinterpret_cast<uint16_t*>(nib1 + noff) = (uint16_t)n1;
      *reinterpret_cast<u2v*>(vals2 + voff) = u2v{lo2, hi2};
      *reinterpret_cast<uint16_t*>(nib2 + noff) = (uint16_t)n2;
      if (spill)
        atomicOr(&flags[band * sparse24_flag_stride(kc) + (blk >> 1)], 1u << (2 * (int)(in_tile >> 5) + (int)(blk & 1)));
    }
    // compressed arrays: position of the lane's first kept entry from ballots of its count
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

}  // namespace

// Codes Q[nvec x kc] (ld = ldq, 16-byte aligned rows, zeros in the columns veclen .. kc-1; kc a
// multiple of 128, nvec a multiple of 256), keep-mask with mask_words(veclen) words per vector.
// vals1 / vals2: nvec * kc / 2 bytes each, nib1 / nib2: nvec * kc / 8 bytes each, flags:
// sparse24_flag_words(nvec, kc) words, which must be ZERO on entry.
bool scatter24_ok(int64_t nvec, int64_t kc, const int8_t* Q, int64_t ldq) {
  return nvec > 0 && kc > 0 && (nvec % 256) == 0 && (kc % 128) == 0 && (ldq % 16) == 0 && ldq >= kc &&
         (reinterpret_cast<uintptr_t>(Q) & 15) == 0;
}

hipError_t launch_scatter24(const uint64_t* mask, int64_t nvec, int64_t veclen, int64_t kc, const int8_t* Q,
                            int64_t ldq, const int32_t* ptr, int32_t* idx, int8_t* val, int64_t capacity,
                            int8_t* vals1, uint8_t* nib1, int8_t* vals2, uint8_t* nib2, uint32_t* flags,
                            hipStream_t st) {
  if (nvec <= 0 || kc <= 0) return hipSuccess;
  hipLaunchKernelGGL(scatter24_kernel, dim3((unsigned)nvec), dim3(256), 0, st, mask, mask_words(veclen), veclen, kc,
                     Q, ldq, ptr, idx, val, capacity, vals1, nib1, vals2, nib2, flags);
  return hipGetLastError();
}

}  // namespace srq
