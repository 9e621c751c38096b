// Arguments shared by the host launcher and the kernels (plain data).
#pragma once
#include <stdint.h>

namespace fmha {

constexpr int kHeadDim = 64;
constexpr int kTileRows = 128;  // rows (queries, or keys in the dK/dV pass) per work tile
constexpr int kBlockKeys = 64;  // rows staged in LDS per inner step
constexpr int kThreads = 256;   // 4 wavefronts; each owns 32 rows of the tile

struct TileItem {
  int32_t seq;   // sequence index
  int32_t row0;  // first row of the tile within the sequence
};

struct Problem {
  const int32_t* cu;       // [B+1]
  const int32_t* seqused;  // [B] or null
  const int32_t* n_tiles;  // device scalar written by the schedule kernel
  const TileItem* tiles;   // tile list, longest sequences first
  int32_t heads;
  int32_t total_tokens;
  float scale;
};

struct FwdArgs {
  Problem pb;
  const uint16_t *q, *k, *v;
  uint16_t* o;
  float* lse;  // [H, T]
  int64_t q_stride, k_stride, v_stride, o_stride;
};

struct BwdArgs {
  Problem pb;
  const uint16_t *q, *k, *v, *o, *d_o;
  const float* lse;  // [H, T]
  float* dsum;       // [H, T] rowsum(dO o O), workspace (written by the dQ pass)
  float* lse2;       // [H, T] lse * log2(e), workspace (written by the dQ pass)
  uint16_t *dq, *dk, *dv;
  int64_t q_stride, k_stride, v_stride, o_stride, do_stride, dq_stride, dk_stride, dv_stride;
};

}  // namespace fmha
