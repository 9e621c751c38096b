// Tile list: the replacement for the paper's length groups and per-group
// streams (Section IV-A-2).  Every sequence is cut into 128-row tiles; tiles
// are emitted longest sequence first so that one launch, whose workgroups the
// hardware hands out in index order, finishes the expensive tiles early and
// fills the tail with cheap ones.
#pragma once
#include "kernel_args.h"

namespace fmha {

constexpr int kSchedThreads = 1024;
constexpr int kSchedBuckets = 128;  // bucket = ceil(keys / 8), clipped; bucket 0 = longest

__device__ __forceinline__ int sched_bucket(int nkeys) {
  int b = (nkeys + 7) >> 3;
  b = b > kSchedBuckets - 1 ? kSchedBuckets - 1 : b;
  return kSchedBuckets - 1 - b;
}

// One workgroup.  count <- number of tiles, list[0..count) <- tiles.  `cap`
// bounds the list (total_tokens/128 + batch always suffices).
__global__ __launch_bounds__(kSchedThreads) void schedule_kernel(const int32_t* __restrict__ cu,
                                                                 const int32_t* __restrict__ seqused,
                                                                 int batch, int32_t* count,
                                                                 TileItem* list, int cap, uint32_t* feed_counters) {
  __shared__ int cursor[kSchedBuckets];
  const int tid = threadIdx.x;
  if (tid < kFeedWords) feed_counters[tid] = 0u;  // the item feed's counters start at zero
  static_assert(kFeedWords <= kSchedThreads, "one thread per word");
  if (tid < kSchedBuckets) cursor[tid] = 0;
  __syncthreads();
  // The thread's first sequence stays in registers for the second sweep (one memory
  // round trip less on the usual batch of at most 1024 sequences).
  int r0_first = 0, len_first = 0, nk_first = 0;
  for (int i = tid; i < batch; i += kSchedThreads) {
    const int r0 = cu[i];
    const int len = cu[i + 1] - r0;
    const int nk = len <= 0 ? 0 : (seqused ? min(max(seqused[i], 0), len) : len);
    if (i == tid) {
      r0_first = r0;
      len_first = len;
      nk_first = nk;
    }
    if (len <= 0) continue;
    atomicAdd(&cursor[sched_bucket(nk)], (len + kTileRows - 1) / kTileRows);
  }
  __syncthreads();
  // exclusive prefix sum over the 128 buckets: two wavefronts scan 64 each, the
  // second then adds the first one's total
  __shared__ int half_total;
  int incl = 0, mine = 0;
  if (tid < kSchedBuckets) {
    const int lane = tid & 63;
    mine = cursor[tid];
    incl = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int up = __shfl_up(incl, d, 64);
      if (lane >= d) incl += up;
    }
    if (tid == 63) half_total = incl;
  }
  __syncthreads();
  if (tid < kSchedBuckets) {
    const int excl = incl - mine + (tid >= 64 ? half_total : 0);
    cursor[tid] = excl;
    if (tid == kSchedBuckets - 1) {
      const int run = excl + mine;
      *count = run < cap ? run : cap;
    }
  }
  __syncthreads();
  for (int i = tid; i < batch; i += kSchedThreads) {
    int r0 = r0_first, len = len_first, nk = nk_first;
    if (i != tid) {
      r0 = cu[i];
      len = cu[i + 1] - r0;
      nk = len <= 0 ? 0 : (seqused ? min(max(seqused[i], 0), len) : len);
    }
    if (len <= 0) continue;
    const int nt = (len + kTileRows - 1) / kTileRows;
    int at = atomicAdd(&cursor[sched_bucket(nk)], nt);
    for (int t = 0; t < nt; t++)
      if (at + t < cap) list[at + t] = TileItem{r0, len, nk, t * kTileRows};
  }
}

}  // namespace fmha
