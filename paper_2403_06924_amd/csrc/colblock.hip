// Column-block execution of a reduced operand (the block-structured direction of the paper's
// closing section; Algorithm 1 line 12 computed in two parts that add up to the same integers).
//
// A reduced operand whose selection is dominated by a few whole "k-columns" (an index k kept in
// nearly every vector: the outlier columns of an activation matrix) is split into
//   * a dense strip: up to kStripK such k, gathered into a K-contiguous code matrix of width
//     kStripK (zero-padded; entries the selection dropped stay zero), multiplied on the matrix
//     cores with the same k gathered from the dense residual codes of the other operand;
//   * the remainder: the compressed operand without those k, on the vector ALUs (the sparse
//     kernel skips entries whose index is flagged).
// Nothing is approximated: strip + remainder hold exactly the kept entries, so the two integer
// products sum to the sparse product of the whole reduced operand.
#include "srq_internal.h"

namespace srq {
namespace {

// kept entries per k from the keep-mask (one 64-bit word per 64 k of a vector): a wave owns one
// word-column and a slice of the vectors, 64 vectors at a time (one word per lane); bit b of the
// 64 words is counted with one ballot, lane b keeping the running count of k = 64 wc + b
__global__ __launch_bounds__(256) void colcount_kernel(const uint64_t* __restrict__ mask, int64_t words,
                                                       int64_t nvec, int32_t* __restrict__ count) {
  const int lane = threadIdx.x & 63;
  const int64_t wc = blockIdx.x;
  const int64_t slices = (int64_t)gridDim.y * 4;
  const int64_t slice = (int64_t)blockIdx.y * 4 + (threadIdx.x >> 6);
  const int64_t per = ((nvec + slices - 1) / slices + 63) / 64 * 64;
  const int64_t v0 = slice * per, v1 = v0 + per < nvec ? v0 + per : nvec;
  int c = 0;
  for (int64_t vb = v0; vb < v1; vb += 64) {
    const int64_t v = vb + lane;
    const uint64_t word = v < v1 ? mask[v * words + wc] : 0ull;
    if (!__ballot(word != 0ull)) continue;
#pragma unroll 16
    for (int bit = 0; bit < 64; ++bit) {
      const int n = __popcll(__ballot((word >> bit) & 1ull));
      if (lane == bit) c += n;
    }
  }
  if (c) atomicAdd(&count[wc * 64 + lane], c);            // integer adds: order does not matter
}

// One block: the k whose count reaches `need` become the strip, in ascending order, at most
// kStripK of them.  klist[kStripK] (-1 past the end), kflag = bitmap over k (32 per word), nstrip.
__global__ __launch_bounds__(1024) void colpick_kernel(const int32_t* __restrict__ count, int64_t K, int32_t need,
                                                       int32_t* __restrict__ klist, uint32_t* __restrict__ kflag,
                                                       int32_t* __restrict__ nstrip) {
  __shared__ int wave_cnt[16];
  __shared__ int base;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  if (tid == 0) base = 0;
  if (tid < kStripK) klist[tid] = -1;
  __syncthreads();
  for (int64_t k0 = 0; k0 < K; k0 += 1024) {
    const int64_t k = k0 + tid;
    const bool hit = k < K && count[k] >= need;
    const unsigned long long m = __ballot(hit);
    if (lane == 0) wave_cnt[w] = __popcll(m);
    __syncthreads();
    int pos = base + __popcll(m & ((1ull << lane) - 1ull));
    for (int i = 0; i < w; ++i) pos += wave_cnt[i];
    const bool take = hit && pos < kStripK;
    if (take) klist[pos] = (int32_t)k;
    // flag words: 32 consecutive k = half a wave
    const unsigned long long t = __ballot(take);
    if (k < K && (lane & 31) == 0) kflag[k >> 5] = (uint32_t)(t >> (lane & 32));
    __syncthreads();
    if (tid == 0) {
      int add = 0;
      for (int i = 0; i < 16; ++i) add += wave_cnt[i];
      base += add;
    }
    __syncthreads();
  }
  if (tid == 0) *nstrip = base < kStripK ? base : kStripK;
}

// strip[v][c] = keep-bit(v, klist[c]) ? Q[v][klist[c]] : 0  (mask == null: every entry is taken,
// the dense residual codes of the other operand); columns past the strip's end are zero
__global__ __launch_bounds__(256) void strip_gather_kernel(const int8_t* __restrict__ Q, int64_t ldq,
                                                           const uint64_t* __restrict__ mask, int64_t words,
                                                           int64_t nvec, const int32_t* __restrict__ klist,
                                                           int8_t* __restrict__ strip) {
  const int c = threadIdx.x & (kStripK - 1);
  const int64_t v = (int64_t)blockIdx.x * (256 / kStripK) + (threadIdx.x / kStripK);
  if (v >= nvec) return;
  const int k = klist[c];
  int8_t out = 0;
  if (k >= 0 && (!mask || ((mask[v * words + (k >> 6)] >> (k & 63)) & 1ull))) out = Q[v * ldq + k];
  strip[v * kStripK + c] = out;
}

}  // namespace

hipError_t launch_colblock_pick(const uint64_t* mask, int64_t nvec, int64_t K, double min_keep_ratio,
                                int32_t* count, int32_t* klist, uint32_t* kflag, int32_t* nstrip,
                                hipStream_t st) {
  if (nvec <= 0 || K <= 0) return hipSuccess;
  const int64_t words = mask_words(K);
  hipError_t e = launch_fill_u32(reinterpret_cast<uint32_t*>(count), words * 64, 0, st);
  if (e != hipSuccess) return e;
  int64_t gy = (nvec + 1023) / 1024;                      // about 256 vectors per wave
  if (gy < 1) gy = 1;
  if (gy > 64) gy = 64;
  hipLaunchKernelGGL(colcount_kernel, dim3((unsigned)words, (unsigned)gy), dim3(256), 0, st, mask, words, nvec,
                     count);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  int64_t need = (int64_t)(min_keep_ratio * (double)nvec + 0.999999);
  if (need < 1) need = 1;
  hipLaunchKernelGGL(colpick_kernel, dim3(1), dim3(1024), 0, st, count, K, (int32_t)need, klist, kflag, nstrip);
  return hipGetLastError();
}

hipError_t launch_strip_gather(const int8_t* Q, int64_t ldq, const uint64_t* mask, int64_t K, int64_t nvec,
                               const int32_t* klist, int8_t* strip, hipStream_t st) {
  if (nvec <= 0) return hipSuccess;
  const int per = 256 / kStripK;
  hipLaunchKernelGGL(strip_gather_kernel, dim3((unsigned)((nvec + per - 1) / per)), dim3(256), 0, st, Q, ldq, mask,
                     mask_words(K), nvec, klist, strip);
  return hipGetLastError();
}

}  // namespace srq
