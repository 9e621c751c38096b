// Writes out the dropout keep mask exactly as the attention kernels see it,
// through the same per-tile routine (keep_bytes) in either of its two
// orientations, so that tests can compare it bit for bit with an independent
// implementation of the mask's definition.  Not part of the hot path.
#pragma once
#include "dropout.h"
#include "kernel_args.h"

namespace fmha {

// mask[(h * T + t) * row_bytes + k] = 1 if element (query row t, key k of the same
// sequence) of head h is kept, 0 if dropped, for k < L of that sequence; other bytes
// are not written.  TRANSPOSED selects the S (column = key) form of keep_bytes.
template <bool TRANSPOSED>
__global__ __launch_bounds__(kThreads) void keep_mask_kernel(const Problem pb, const DropArgs d, uint8_t* mask,
                                                             int row_bytes) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int g = lane >> 5, ln = lane & 31;
  const int heads = pb.heads;
  const int n_items = tile_count(pb) * heads;
  for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
    const int head = item % heads;
    const TileItem ti = load_tile(pb, item / heads);
    const int len = ti.len;
    if (ti.row0 + 32 * wave >= len) continue;  // uniform over the wavefront
    const int col = ti.row0 + 32 * wave + ln;
    for (int rb = 0; rb < len; rb += 32) {
      uint32_t kb[4];
      keep_bytes<TRANSPOSED>(kb, col >> 2, (rb >> 2) + g, ln, ti.r0, head, d);
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const int row = rb + 8 * (r >> 2) + 4 * g + (r & 3);
        const int q = TRANSPOSED ? row : col, k = TRANSPOSED ? col : row;
        if (q < len && k < len && k < row_bytes)
          mask[((int64_t)head * pb.total_tokens + ti.r0 + q) * row_bytes + k] = kept(kb, r, d.thr) ? 1 : 0;
      }
    }
  }
}

}  // namespace fmha
