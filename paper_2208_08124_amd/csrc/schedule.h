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

// A sequence as the kernels may use it: whatever the device arrays hold, the rows
// [r0, r0 + len) lie inside the packed tensors of total_tokens rows (arrays that disagree
// with the sizes the host passed can then only give wrong numbers, never addresses out of
// range), and at most len keys are attended.
struct SchedSeq {
  int r0, len, nk;
};
__device__ __forceinline__ SchedSeq sched_seq(const int32_t* __restrict__ cu, const int32_t* __restrict__ seqused,
                                              int i, int total_tokens) {
  SchedSeq s;
  s.r0 = min(max(cu[i], 0), total_tokens);
  s.len = min(max(cu[i + 1] - s.r0, 0), total_tokens - s.r0);
  s.nk = s.len <= 0 ? 0 : (seqused ? min(max(seqused[i], 0), s.len) : s.len);
  return s;
}

// One workgroup.  count <- number of tiles, list[0..count) <- tiles.  `cap`
// bounds the list (total_tokens/128 + batch always suffices).
__global__ __launch_bounds__(kSchedThreads) void schedule_kernel(const int32_t* __restrict__ cu,
                                                                 const int32_t* __restrict__ seqused,
                                                                 int batch, int total_tokens, int32_t* count,
                                                                 TileItem* list, int cap, uint32_t* feed_counters) {
  __shared__ int cursor[kSchedBuckets];
  const int tid = threadIdx.x;
  if (tid < kFeedWords) feed_counters[tid] = 0u;  // the item feed's counters start at zero
  static_assert(kFeedWords <= kSchedThreads, "one thread per word");
  if (tid < kSchedBuckets) cursor[tid] = 0;
  __syncthreads();
  // The thread's first sequence stays in registers for the second sweep (one memory
  // round trip less on the usual batch of at most 1024 sequences).
  SchedSeq first = {0, 0, 0};
  for (int i = tid; i < batch; i += kSchedThreads) {
    const SchedSeq s = sched_seq(cu, seqused, i, total_tokens);
    if (i == tid) first = s;
    if (s.len <= 0) continue;
    atomicAdd(&cursor[sched_bucket(s.nk)], (s.len + kTileRows - 1) / kTileRows);
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
    const SchedSeq s = i == tid ? first : sched_seq(cu, seqused, i, total_tokens);
    if (s.len <= 0) continue;
    const int nt = (s.len + kTileRows - 1) / kTileRows;
    const int at = atomicAdd(&cursor[sched_bucket(s.nk)], nt);
    for (int t = 0; t < nt; t++)
      if (at + t < cap) list[at + t] = TileItem{s.r0, s.len, s.nk, t * kTileRows};
  }
}

}  // namespace fmha
