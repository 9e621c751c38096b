// Hand-out of (tile, head) work items to persistent workgroups - the scheduler that stands
// in for the paper's length groups on separate streams (Section IV-A-2).
//
// Items are numbered in list order (longest sequences first, head fastest).  Item i belongs
// to class i % 8; a workgroup only takes items of class blockIdx % 8, so with the hardware's
// round-robin placement of workgroups on the 8 dies all tiles of a (sequence, head) whose
// head count is a multiple of 8 are computed on one die and share its L2 (a placement
// heuristic: nothing depends on it for correctness).
//
// Within a class, positions k = i / 8 are handed out in chunks of `chunk` consecutive
// positions.  The first three chunks of every workgroup are fixed: chunk number = its rank in
// the class, then the mirrored rank (so that every workgroup starts with a similar load), then
// the rank again; all later ones are claimed from a counter per class with an atomic add, so
// that workgroups that run faster - on a SIMD the older wavefront is favoured, measured 15
// against 22 us per item - take more items, and the expensive items, which come first, are
// never left for the end.  A claim is requested two items before it is needed (its latency
// never shows; the first one when the workgroup has finished its first item, so that the
// claims are ordered by progress and not by launch time) by the first lane of the workgroup
// and reaches the other wavefronts through a word of LDS at a barrier the kernels have anyway.
//
// The counters live in the workspace; the tile-list kernel zeroes them, and every kernel
// that uses them leaves them zero: the last workgroup to finish clears them (told by exit
// counters in two levels - per class, then one for the classes - so that workgroups ending
// together do not queue on one address).  Kernels that share a workspace must therefore not
// overlap in time.  All atomics are relaxed, at device scope: nothing but the counters
// themselves is communicated through them, and an acquire or release at that scope would
// write back and invalidate the die's whole L2 at every use (measured: the forward kernel
// took 103 instead of 60 us with an acquire-release exit counter).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fmha {

constexpr int kFeedClasses = 8;
constexpr int kFeedClassWords = 64;                       // one 256-byte line per class: [0] claims, [1] exits
constexpr int kFeedWords = kFeedClasses * kFeedClassWords;  // 2 KB

struct FeedArgs {
  uint32_t* counters;  // kFeedWords words, zero at launch
  int32_t chunk;       // positions per chunk, >= 1
};

struct ItemFeed {
  int cls;           // class of this workgroup
  int kpos, kend;    // next position and end of the current chunk
  int rank, per_class;
  int chunk;
  int stage;         // chunks started so far, minus one
  int pending;       // start of the next claimed chunk, relative to the end of the fixed ones (all wavefronts)
  bool want;         // the pending claim was used up (or none was made yet): request another
  uint32_t claimed;  // first lane of the workgroup: the claim last requested

  static constexpr int kFixed = 3;  // chunks per workgroup that are not claimed

  // grid must be a multiple of 8.  Returns the workgroup's first item.
  __device__ __forceinline__ int init(const FeedArgs& f, int block, int grid) {
    cls = block & 7;
    chunk = f.chunk;
    per_class = grid >> 3;
    rank = block >> 3;
    kpos = chunk * rank;
    kend = kpos + chunk;
    stage = 0;
    pending = 0;
    claimed = 0;
    want = true;
    return (kpos++) * kFeedClasses + cls;
  }
  // Request the next chunk if the last one received has been used.  Call it where the
  // answer has time to arrive before the next publish().
  __device__ __forceinline__ void request(const FeedArgs& f) {
    if (want) {
      if (threadIdx.x == 0)
        claimed = __hip_atomic_fetch_add(f.counters + cls * kFeedClassWords, (uint32_t)chunk, __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_AGENT);
      want = false;
    }
  }
  // Once per item, around a workgroup barrier: the first lane publishes the claim it holds,
  // everybody picks it up after the barrier.
  __device__ __forceinline__ void publish(uint32_t* mailbox) const {
    if (threadIdx.x == 0) *mailbox = claimed;
  }
  __device__ __forceinline__ void receive(const uint32_t* mailbox) {
    pending = __builtin_amdgcn_readfirstlane((int)*mailbox);
  }
  // Next item of this workgroup (may lie beyond the end of the list: then the workgroup is
  // done).  Uniform over the workgroup.  After init(), call it once before the first
  // receive() and then once after each receive(), followed by request().
  __device__ __forceinline__ int next() {
    if (kpos >= kend) {
      stage++;
      if (stage == 1) {
        kpos = chunk * (2 * per_class - 1 - rank);
      } else if (stage < kFixed) {
        kpos = chunk * (stage * per_class + rank);
      } else {
        kpos = chunk * kFixed * per_class + pending;
        want = true;
      }
      kend = kpos + chunk;
    }
    return (kpos++) * kFeedClasses + cls;
  }
  // Last act of a workgroup (all its claims have returned: they were published): the last
  // one of a class to finish leaves the class's counters zero for the next kernel.
  __device__ __forceinline__ void finish(const FeedArgs& f, int grid) const {
    if (threadIdx.x == 0) {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the claims have been performed
      uint32_t* mine = f.counters + cls * kFeedClassWords;
      const uint32_t per_class = (uint32_t)grid >> 3;
      if (__hip_atomic_fetch_add(mine + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == per_class - 1u) {
        __hip_atomic_store(mine, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(mine + 1, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }
};

}  // namespace fmha
