// Arguments shared by the host launcher and the kernels (plain data).
#pragma once
#include <stdint.h>

#include "item_feed.h"

namespace fmha {

constexpr int kHeadDim = 64;
constexpr int kTileRows = 128;  // rows (queries, or keys in the dK/dV pass) per work tile
constexpr int kBlockKeys = 64;  // rows staged in LDS per inner step
constexpr int kThreads = 256;   // 4 wavefronts; each owns 32 rows of the tile

// One unit of work: a tile of up to 128 rows of one sequence, with everything a
// kernel needs to know about that sequence, so that starting a tile costs one
// (prefetchable) 16-byte load instead of a chain of dependent ones.
struct TileItem {
  int32_t r0;    // packed row at which the sequence starts
  int32_t len;   // rows of the sequence (queries)
  int32_t nk;    // keys attended: len, or min(seqused, len)
  int32_t row0;  // first row of the tile within the sequence
};

struct Problem {
  const int32_t* n_tiles;  // device scalar written by the schedule kernel
  const TileItem* tiles;   // tile list, longest sequences first
  int32_t heads;
  int32_t total_tokens;
  float scale;
};

// Dropout on the attention probabilities (see dropout.h).
struct DropArgs {
  uint32_t thr;     // an element is dropped iff its random byte is < thr; 0 = dropout off
  uint32_t k0, k1;  // generator key = the two halves of the seed
  float rp;         // 256 / (256 - thr), multiplies what is kept
};

struct FwdArgs {
  Problem pb;
  DropArgs drop;
  FeedArgs feed;
  const uint16_t *q, *k, *v;
  uint16_t* o;
  float* lse;  // [H, T]
  int64_t q_stride, k_stride, v_stride, o_stride;
};

struct BwdArgs {
  Problem pb;
  DropArgs drop;
  FeedArgs feed;
  const uint16_t *q, *k, *v, *o, *d_o;
  const float* lse;  // [H, T]
  float* dsum;       // [H, T] rowsum(dO o O), workspace (written by the dQ pass)
  float* lse2;       // [H, T] lse * log2(e), workspace (written by the dQ pass)
  uint16_t *dq, *dk, *dv;
  int64_t q_stride, k_stride, v_stride, o_stride, do_stride, dq_stride, dk_stride, dv_stride;
};

// The tile list and its count were written by an earlier kernel and are only
// read here.  Reading them through the constant address space lets the compiler
// use scalar loads (wave-uniform, tracked by their own counter) instead of vector
// loads, whose completion would otherwise be awaited together with - and so
// serialise - whatever else the wavefront has in flight on the vector memory path.
typedef const __attribute__((address_space(4))) int32_t* ConstInt;
__device__ __forceinline__ TileItem load_tile(const Problem& pb, int i) {
  ConstInt p = (ConstInt)(uintptr_t)(pb.tiles + i);
  return TileItem{p[0], p[1], p[2], p[3]};
}
__device__ __forceinline__ int tile_count(const Problem& pb) { return *(ConstInt)(uintptr_t)pb.n_tiles; }

}  // namespace fmha
