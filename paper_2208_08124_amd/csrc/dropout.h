// Dropout on the attention probabilities, regenerated from (seed, position) in
// every kernel that needs it (forward, both backward passes).
//
// The mask (the same definition the public header gives): the 4 x 4 block
// (Q4, K4) = (q >> 2, k >> 2) of the score matrix of the sequence starting at
// packed row r0, head h, owns one Philox4x32-10 call (Salmon et al., SC 2011)
// with counter (K4, Q4, r0, h) and the 64-bit seed as key.  Its 16 output bytes
// B[x][y] (byte y of word x) serve the 16 elements: element (q, k) reads
//   x = ((q & 3) - (k >> 3)) & 3,   y = ((k & 3) - (q >> 3)) & 3
// and is kept iff that byte is >= thr = round(256 p).
//
// Why this shape.  In the MFMA result layout a lane holds, for its one column,
// rows 8j + 4g + e (j, e = 0..3): four runs of four.  With S^T tiles (forward,
// dQ pass) the column is a query and the rows are keys; with S tiles (dK/dV
// pass) it is the other way round.  Either way the four lanes of a quad
// (columns 4m .. 4m+3) cover, for each j, exactly one 4 x 4 block - so each
// lane makes ONE call (the block j = lane & 3) and the quad trades words:
// 16 elements per lane per call in both orientations, no call made twice.
// The two index twists above are what make the trade cheap: lane b needs from
// lane j word (b - j) & 3, so step i of the exchange (quad rotation by i)
// always moves register i, and the remaining differences are one rotation of
// the bytes within each word and one of the four words, both by lane-constant
// amounts.
#pragma once
#include "kernel_args.h"
#include "mfma_tiles.h"

namespace fmha {

static __device__ __forceinline__ u32x4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                      uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; r++) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return u32x4{c0, c1, c2, c3};
}

// lane b of each quad receives the value lane (b - I) & 3 holds
template <int I>
static __device__ __forceinline__ uint32_t quad_rotate(uint32_t x) {
  constexpr int ctrl = ((0 - I) & 3) | (((1 - I) & 3) << 2) | (((2 - I) & 3) << 4) | (((3 - I) & 3) << 6);
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, ctrl, 0xf, 0xf, false);
}

// Keep-mask bytes for the 16 registers of one 32 x 32 result tile.
//   col4   : (this lane's column index within the sequence) >> 2   (query for S^T, key for S)
//   row4   : (first row of the 32-row tile) >> 2 + g               (key block for S^T, query block for S)
//   ln     : lane & 31
// TRANSPOSED = false for S^T tiles (column = query), true for S tiles (column = key).
// Returns four words; byte e of word j belongs to register 4j + e.
// All 64 lanes must be active.
template <bool TRANSPOSED>
static __device__ __forceinline__ void keep_bytes(uint32_t (&out)[4], int col4, int row4, int ln, int r0,
                                                  int head, const DropArgs& d) {
  const int b = ln & 3;         // position in the quad = which block this lane generates
  const int c = (ln >> 3) & 3;  // (column >> 3) & 3: tile bases are multiples of 32
  const int blk = row4 + 2 * b;
  // (the key schedule is ten scalar additions per call; the empty asm keeps the compiler
  // from forming all twenty round keys once per kernel and holding them in scalar registers)
  uint32_t k0 = d.k0, k1 = d.k1;
  asm volatile("" : "+s"(k0), "+s"(k1));
  const u32x4 w = TRANSPOSED ? philox4x32_10(col4, blk, r0, head, k0, k1)
                             : philox4x32_10(blk, col4, r0, head, k0, k1);
  uint32_t s[4] = {w[0], w[1], w[2], w[3]};
  if (TRANSPOSED) {
    // 4 x 4 byte transpose: s[y] byte n = w[n] byte y
    const uint32_t a0 = __builtin_amdgcn_perm(w[1], w[0], 0x05010400u);
    const uint32_t a1 = __builtin_amdgcn_perm(w[1], w[0], 0x07030602u);
    const uint32_t b0 = __builtin_amdgcn_perm(w[3], w[2], 0x05010400u);
    const uint32_t b1 = __builtin_amdgcn_perm(w[3], w[2], 0x07030602u);
    s[0] = __builtin_amdgcn_perm(b0, a0, 0x05040100u);
    s[1] = __builtin_amdgcn_perm(b0, a0, 0x07060302u);
    s[2] = __builtin_amdgcn_perm(b1, a1, 0x05040100u);
    s[3] = __builtin_amdgcn_perm(b1, a1, 0x07060302u);
  }
  // got[i] comes from lane (b - i) & 3, i.e. it is the word for block j = (b - i) & 3
  uint32_t got[4] = {s[0], quad_rotate<1>(s[1]), quad_rotate<2>(s[2]), quad_rotate<3>(s[3])};
  // byte e of the result must be byte (e - c) & 3 of what arrived: rotate left by c bytes
  const uint32_t rot = (32u - 8u * c) & 31u;
#pragma unroll
  for (int i = 0; i < 4; i++) got[i] = __builtin_amdgcn_alignbit(got[i], got[i], rot);
  // out[j] = got[(b - j) & 3]: with h[j] = got[(-j) & 3] that is h rotated by b
  const uint32_t h[4] = {got[0], got[3], got[2], got[1]};
  uint32_t r1[4];
#pragma unroll
  for (int j = 0; j < 4; j++) r1[j] = (b & 1) ? h[(j + 3) & 3] : h[j];
#pragma unroll
  for (int j = 0; j < 4; j++) out[j] = (b & 2) ? r1[(j + 2) & 3] : r1[j];
}

static __device__ __forceinline__ bool kept(const uint32_t (&kb)[4], int r, uint32_t thr) {
  return ((kb[r >> 2] >> (8 * (r & 3))) & 0xffu) >= thr;
}

}  // namespace fmha
