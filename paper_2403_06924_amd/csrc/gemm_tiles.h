// Pieces shared by the persistent matrix-core kernels (dense and 2:4): the launch-order -> tile
// mapping and the direct global -> LDS load.
#ifndef SRQ_GEMM_TILES_H_
#define SRQ_GEMM_TILES_H_
#include "srq_internal.h"

namespace srq {

// tile coordinates of the vb-th tile in launch order: XCD-contiguous bands, groups of 8 rows
static __device__ __forceinline__ void tile_of(int64_t vb, int64_t tiles_m, int64_t tiles_n, int64_t& tm, int64_t& tn) {
  const int64_t total = tiles_m * tiles_n, per = total / 8;
  int64_t bid = vb;
  if (per > 0 && bid < per * 8) bid = (bid & 7) * per + (bid >> 3);
  const int64_t g = 8;
  int64_t grp = bid / (g * tiles_n), first = grp * g;
  int64_t rows_in = tiles_m - first < g ? tiles_m - first : g;
  int64_t in = bid - grp * g * tiles_n;
  tm = first + in % rows_in;
  tn = in / rows_in;
}

// One wave-wide 16-byte-per-lane load from global memory into LDS: lane l's bytes land at
// lds_base + 16*l.  Issued as inline assembly so that its completion is waited for explicitly
// (wait_loads) right before the barrier that publishes the tile, not before every LDS read.
static __device__ __forceinline__ void load_to_lds(const int8_t* gptr, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_base), "v"(gptr) : "memory", "m0");
}
static __device__ __forceinline__ void wait_loads() { asm volatile("s_waitcnt vmcnt(0)" : : : "memory"); }
// All but the newest N vector-memory operations of this wave have completed.  (Loads complete in
// the order they were issued; stores may overtake them, so a count is only relied on where the
// loads to be waited for are older than N younger LOADS.)
template <int N>
static __device__ __forceinline__ void wait_loads_but() {
  asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

}  // namespace srq

#endif  // SRQ_GEMM_TILES_H_
