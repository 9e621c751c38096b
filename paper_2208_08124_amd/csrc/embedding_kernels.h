// Backward of the embedding lookup (Section IV-C-3 of the paper): row t of the output
// gradient is added onto row indices[t] of the weight gradient.  Rows that share an index
// collide; as in the paper the collisions are resolved by the memory system's atomic add on
// PACKED pairs of 16-bit values (global_atomic_pk_add_f16 / _bf16: two adjacent columns per
// operation), with a fine work split: one wavefront per token row, each atomic instruction
// covering 256 contiguous bytes of the weight-gradient row.
//
// What is specific to this chip: its eight dies (XCDs) have an L2 each, and a line that is
// updated from several dies migrates between them on every update.  Workgroups are handed to
// the dies round-robin (workgroup b runs on die b mod 8), so in the die-aware variant
// workgroup b only takes the tokens with indices[t] mod 8 == b mod 8: all updates of one
// weight row then come from one die and stay in its L2.  Every die scans all indices
// (4 bytes per token) but reads only its own share of the gradient rows.  This is a placement
// heuristic only: the result does not depend on where a workgroup actually runs.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fmha {

constexpr int kEmbThreads = 256;

typedef _Float16 emb_h2 __attribute__((ext_vector_type(2)));
typedef short emb_s2 __attribute__((ext_vector_type(2)));

template <bool BF16>
static __device__ __forceinline__ void pk_add(uint32_t* p, uint32_t v) {
  if (BF16)
    __builtin_amdgcn_global_atomic_fadd_v2bf16((__attribute__((address_space(1))) emb_s2*)p,
                                               __builtin_bit_cast(emb_s2, v));
  else
    __builtin_amdgcn_global_atomic_fadd_v2f16((__attribute__((address_space(1))) emb_h2*)p,
                                              __builtin_bit_cast(emb_h2, v));
}

struct EmbArgs {
  const uint32_t* dy;      // [rows, pairs] packed pairs of 16-bit values
  const int32_t* indices;  // [rows]
  const int32_t* n_rows;   // device, may be null: rows actually present
  uint32_t* dw;            // [vocab, pairs]
  int32_t rows, pairs, vocab, padding_idx;
};

static __device__ __forceinline__ int emb_rows(const EmbArgs& a) {
  int n = a.rows;
  if (a.n_rows) n = min(max(*a.n_rows, 0), n);
  return n;
}

// one wavefront adds one gradient row (its columns [c_begin, c_end), counted in pairs) onto
// its weight row
template <bool BF16>
static __device__ __forceinline__ void add_row(const EmbArgs& a, int t, int v, int lane, int c_begin, int c_end) {
  const uint32_t* src = a.dy + (int64_t)t * a.pairs;
  uint32_t* dst = a.dw + (int64_t)v * a.pairs;
  for (int c0 = c_begin; c0 < c_end; c0 += 256) {  // four loads in flight, then four atomics
    uint32_t x[4];
#pragma unroll
    for (int u = 0; u < 4; u++) {
      const int c = c0 + 64 * u + lane;
      x[u] = c < c_end ? src[c] : 0u;
    }
#pragma unroll
    for (int u = 0; u < 4; u++) {
      const int c = c0 + 64 * u + lane;
      if (c < c_end) pk_add<BF16>(dst + c, x[u]);
    }
  }
}

// Plain variant: wavefront w takes tokens w, w + W, ...
template <bool BF16>
__global__ __launch_bounds__(kEmbThreads) void embedding_bwd_kernel(const EmbArgs a) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int rows = emb_rows(a);
  const int stride = gridDim.x * (kEmbThreads / 64);
  for (int t = blockIdx.x * (kEmbThreads / 64) + wave; t < rows; t += stride) {
    const int v = a.indices[t];  // uniform over the wavefront
    if (v < 0 || v >= a.vocab || v == a.padding_idx) continue;
    add_row<BF16>(a, t, v, lane, 0, a.pairs);
  }
}

// The rows named by `members` (NW sets of lanes, one per 64-token sub-window starting at
// t0 + 64k; all these tokens have index v) summed in fp32 and added onto weight row v with one
// set of atomics.
template <bool BF16, int NW>
static __device__ __forceinline__ void add_rows_grouped(const EmbArgs& a, int t0, const uint64_t (&members)[NW], int v,
                                                        int lane, int c_begin, int c_end) {
  uint32_t* dst = a.dw + (int64_t)v * a.pairs;
  for (int c0 = c_begin; c0 < c_end; c0 += 256) {
    float lo[4] = {0.f, 0.f, 0.f, 0.f}, hi[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k = 0; k < NW; k++) {
      uint64_t m = members[k];
      while (m) {  // uniform; up to four member rows per trip, all their loads in flight together
        int row[4];
#pragma unroll
        for (int j = 0; j < 4; j++) {
          row[j] = m ? t0 + 64 * k + __builtin_ctzll(m) : -1;
          m &= m - 1;  // 0 stays 0
        }
        uint32_t x[4][4];
#pragma unroll
        for (int j = 0; j < 4; j++) {
          const uint32_t* src = a.dy + (int64_t)(row[j] < 0 ? row[0] : row[j]) * a.pairs;
#pragma unroll
          for (int u = 0; u < 4; u++) {
            const int c = c0 + 64 * u + lane;
            x[j][u] = (row[j] >= 0 && c < c_end) ? src[c] : 0u;
          }
        }
#pragma unroll
        for (int j = 0; j < 4; j++)
#pragma unroll
          for (int u = 0; u < 4; u++) {
            if (BF16) {
              lo[u] += __builtin_bit_cast(float, x[j][u] << 16);
              hi[u] += __builtin_bit_cast(float, x[j][u] & 0xffff0000u);
            } else {
              lo[u] += (float)__builtin_bit_cast(_Float16, (uint16_t)(x[j][u] & 0xffffu));
              hi[u] += (float)__builtin_bit_cast(_Float16, (uint16_t)(x[j][u] >> 16));
            }
          }
      }
    }
#pragma unroll
    for (int u = 0; u < 4; u++) {
      const int c = c0 + 64 * u + lane;
      uint32_t w;
      if (BF16) {
        typedef __bf16 b2 __attribute__((ext_vector_type(2)));
        w = __builtin_bit_cast(uint32_t, b2{(__bf16)lo[u], (__bf16)hi[u]});
      } else {
        w = __builtin_bit_cast(uint32_t, emb_h2{(_Float16)lo[u], (_Float16)hi[u]});
      }
      if (c < c_end) pk_add<BF16>(dst + c, w);
    }
  }
}

// Default variant.  A workgroup looks at 64 * NW consecutive tokens at a time, NW indices per
// lane (each of its 4 wavefronts reads the same indices and takes a quarter of the columns).
// Tokens of the window that share an index are first summed in registers (fp32) and reach
// memory as ONE row of atomics: with word-piece ids a handful of indices take a large share of
// the tokens, and every atomic on the same address waits for the one before it.  NW = 1 for
// small batches (more workgroups), NW = 4 for large ones (more merging).
// DIE (gridDim.x a multiple of 8): workgroup b only takes the indices congruent to b modulo 8.
template <bool BF16, bool DIE, int NW>
__global__ __launch_bounds__(kEmbThreads) void embedding_bwd_window_kernel(const EmbArgs a) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int rows = emb_rows(a);
  const int die = blockIdx.x & 7;
  const int per = DIE ? (gridDim.x >> 3) : gridDim.x;  // workgroups sharing the windows
  const int me = DIE ? (blockIdx.x >> 3) : blockIdx.x;
  const int quarter = ((a.pairs + 4 * 64 - 1) / (4 * 64)) * 64;  // columns per wavefront, whole 256-byte runs
  const int c_begin = min(wave * quarter, a.pairs), c_end = min(c_begin + quarter, a.pairs);
  if (c_begin >= c_end) return;  // uniform over the wavefront; no barriers below
  constexpr int kWindow = 64 * NW;
  for (int64_t w0 = (int64_t)me * kWindow; w0 < rows; w0 += (int64_t)per * kWindow) {
    const int t0 = (int)w0;
    int v[NW];
    bool mine[NW];
    uint64_t todo[NW];
#pragma unroll
    for (int k = 0; k < NW; k++) {
      const int t = t0 + 64 * k + lane;
      v[k] = t < rows ? a.indices[t] : -1;
      mine[k] = v[k] >= 0 && v[k] < a.vocab && v[k] != a.padding_idx && (!DIE || (v[k] & 7) == die);
      todo[k] = __ballot(mine[k]);
    }
#pragma unroll
    for (int k0 = 0; k0 < NW; k0++) {
      while (todo[k0]) {  // uniform
        const int l = __builtin_ctzll(todo[k0]);
        const int vv = __shfl(v[k0], l, 64);
        uint64_t same[NW];
        int count = 0;
#pragma unroll
        for (int k = 0; k < NW; k++) {
          same[k] = k >= k0 ? __ballot(mine[k] && v[k] == vv) & todo[k] : 0ull;  // earlier sub-windows are done
          todo[k] &= ~same[k];
          count += __popcll(same[k]);
        }
        if (count == 1)
          add_row<BF16>(a, t0 + 64 * k0 + l, vv, lane, c_begin, c_end);  // alone in the window: its 16-bit values go as they are
        else
          add_rows_grouped<BF16, NW>(a, t0, same, vv, lane, c_begin, c_end);
      }
    }
  }
}

__global__ __launch_bounds__(256) void zero_fill_kernel(uint4* p, int64_t n16) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (int64_t)gridDim.x * blockDim.x)
    p[i] = make_uint4(0u, 0u, 0u, 0u);
}

}  // namespace fmha
