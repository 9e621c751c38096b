// Embedding backward without atomics, for callers that know the indices before the gradient
// arrives (the paper computes its index tensors once per mini-batch, Section IV-B-2, and
// names the colliding additions of Section IV-C-3 as the cost of this step): the token
// positions are ordered by index once (a stable radix sort, a call of its own), and the
// gradient rows of an index are then summed in fp32 in that order and written as ONE row.
//
// The sorted positions are cut into chunks of 256 entries, one workgroup each.  A workgroup
// walks its chunk run by run (a run = consecutive entries with the same index).  A run that
// begins and ends inside the chunk is finished on the spot: weight row = old row + sum,
// rounded once.  A run that reaches into the chunk from before ("head") or out of it at the
// end ("tail") leaves its fp32 partial sum in the workspace; a second kernel adds the partial
// sums of each such run in chunk order and writes the row.  Every weight row has exactly one
// writer and every sum a fixed order: results are identical from run to run.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fmha {

constexpr int kEmbChunk = 256;    // sorted entries per workgroup
constexpr int kEmbSortThreads = 128;

// What the two kernels pass through the workspace, per chunk.
struct EmbChunkInfo {
  int32_t head_key;    // index of the run that reaches in from the chunk before, or -1
  int32_t head_whole;  // 1 if that run covers the whole chunk and goes on into the next one
  int32_t tail_key;    // index of the run that goes on into the next chunk and began in this one, or -1
  int32_t pad;
};

struct EmbSortedArgs {
  const uint32_t* dy;     // [rows, pairs] packed pairs of 16-bit values
  const uint32_t* keys;   // [rows] sorted: index, or vocab for entries that are skipped (sorted last)
  const uint32_t* order;  // [rows] token position of each sorted entry
  EmbChunkInfo* info;     // [chunks]
  float* partial;         // [chunks][2][2 * pairs]: head and tail partial sums
  uint32_t* dw;           // [vocab, pairs]
  int32_t rows, pairs, vocab;
  int32_t accumulate;     // 1: add onto the weight rows that are there, 0: they are known to be zero
};

// keys[t] = indices[t] if the token counts (in range, not the padding index, t < *n_rows), else vocab
__global__ __launch_bounds__(256) void emb_keys_kernel(const int32_t* __restrict__ indices, const int32_t* __restrict__ n_rows,
                                                       int rows, int vocab, int padding_idx, uint32_t* __restrict__ keys,
                                                       uint32_t* __restrict__ positions) {
  int n = rows;
  if (n_rows) n = min(max(*n_rows, 0), rows);
  for (int t = blockIdx.x * blockDim.x + threadIdx.x; t < rows; t += gridDim.x * blockDim.x) {
    const int v = t < n ? indices[t] : -1;
    keys[t] = (v >= 0 && v < vocab && v != padding_idx) ? (uint32_t)v : (uint32_t)vocab;
    positions[t] = (uint32_t)t;
  }
}

// x (eight 16-bit values in four dwords) added onto eight fp32 sums
template <bool BF16>
static __device__ __forceinline__ void emb_add8(const uint4& x, float (&s)[8]) {
  const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
  for (int i = 0; i < 4; i++) {
    if (BF16) {
      s[2 * i] += __builtin_bit_cast(float, w[i] << 16);
      s[2 * i + 1] += __builtin_bit_cast(float, w[i] & 0xffff0000u);
    } else {
      s[2 * i] += (float)__builtin_bit_cast(_Float16, (uint16_t)(w[i] & 0xffffu));
      s[2 * i + 1] += (float)__builtin_bit_cast(_Float16, (uint16_t)(w[i] >> 16));
    }
  }
}

// the sums (plus the old weight values, if they count) rounded once to the 16-bit type
template <bool BF16>
static __device__ __forceinline__ uint4 emb_finish8(const uint4& old, float (&s)[8], bool accumulate) {
  if (accumulate) emb_add8<BF16>(old, s);
  uint32_t w[4];
#pragma unroll
  for (int i = 0; i < 4; i++) {
    if (BF16) {
      typedef __bf16 b2 __attribute__((ext_vector_type(2)));
      w[i] = __builtin_bit_cast(uint32_t, b2{(__bf16)s[2 * i], (__bf16)s[2 * i + 1]});
    } else {
      typedef _Float16 h2 __attribute__((ext_vector_type(2)));
      w[i] = __builtin_bit_cast(uint32_t, h2{(_Float16)s[2 * i], (_Float16)s[2 * i + 1]});
    }
  }
  return make_uint4(w[0], w[1], w[2], w[3]);
}

constexpr int kEmbAhead = 16;  // rows a thread has in flight

// One workgroup per chunk of `chunk` (<= kEmbChunk) sorted entries; thread i owns the columns
// 8i .. 8i+7 (and 8(i + 128) .. for rows wider than 1024 values) and walks the chunk's rows in
// order, sixteen 16-byte loads in flight.  What happens at the end of a run is worked out once
// per chunk (one entry per thread) and kept in LDS as index * 4 + action.
template <bool BF16>
__global__ __launch_bounds__(kEmbSortThreads) void emb_chunk_kernel(const EmbSortedArgs a, const int chunk) {
  __shared__ uint32_t s_code[kEmbChunk];  // index * 4 + {0: the run goes on, 1: head partial, 2: tail partial, 3: final row}
  __shared__ uint32_t s_pos[kEmbChunk];
  __shared__ int s_live;                  // entries of the chunk that count (skipped ones are sorted last)
  const int c = blockIdx.x, tid = threadIdx.x;
  const int base = c * chunk;
  const int n = min(chunk, a.rows - base);
  const uint32_t none = (uint32_t)a.vocab;
  const uint32_t first = a.keys[base], last = a.keys[base + n - 1];
  const uint32_t before = base > 0 ? a.keys[base - 1] : none, after = base + n < a.rows ? a.keys[base + n] : none;
  const bool head = first != none && before == first;  // the first run began before this chunk
  const bool tail = last != none && after == last;     // the last run goes on after it
  if (tid == 0) {
    EmbChunkInfo inf;
    inf.head_key = head ? (int32_t)first : -1;
    inf.head_whole = head && tail && first == last;
    inf.tail_key = (tail && !(head && first == last)) ? (int32_t)last : -1;
    inf.pad = 0;
    a.info[c] = inf;
    s_live = 0;
  }
  __syncthreads();
  for (int r = tid; r < n; r += kEmbSortThreads) {
    const uint32_t key = a.keys[base + r];
    const uint32_t next = r + 1 < n ? a.keys[base + r + 1] : after;
    uint32_t action = 0;
    if (key != none && (r == n - 1 || next != key)) {  // the run ends here, or leaves the chunk
      if (head && key == first)
        action = 1;  // (sorted: the run of `first` is the chunk's first run)
      else if (r == n - 1 && tail)
        action = 2;
      else
        action = 3;
    }
    s_code[r] = key * 4u + action;
    s_pos[r] = a.order[base + r];
    if (key != none && (r == n - 1 || next == none)) s_live = r + 1;  // exactly one entry qualifies
  }
  __syncthreads();
  const int live = s_live;
  const int hidden = 2 * a.pairs;
  float* part = a.partial + (int64_t)c * 2 * hidden;  // [head | tail][hidden]
  const uint16_t* dy = reinterpret_cast<const uint16_t*>(a.dy);
  uint16_t* dw = reinterpret_cast<uint16_t*>(a.dw);
  for (int col = 8 * tid; col < hidden; col += 8 * kEmbSortThreads) {
    float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int r0 = 0; r0 < live; r0 += kEmbAhead) {  // (uniform over the workgroup)
      uint4 x[kEmbAhead];
#pragma unroll
      for (int u = 0; u < kEmbAhead; u++)
        x[u] = *reinterpret_cast<const uint4*>(dy + (int64_t)s_pos[min(r0 + u, live - 1)] * hidden + col);
#pragma unroll
      for (int u = 0; u < kEmbAhead; u++) {
        const int r = r0 + u;
        if (r >= live) break;
        emb_add8<BF16>(x[u], s);
        const uint32_t code = s_code[r];
        if (code & 3u) {
          if ((code & 3u) == 3u) {
            uint4* w = reinterpret_cast<uint4*>(dw + (int64_t)(code >> 2) * hidden + col);
            *w = emb_finish8<BF16>(a.accumulate ? *w : make_uint4(0u, 0u, 0u, 0u), s, a.accumulate != 0);
          } else {
            float4* p = reinterpret_cast<float4*>(part + ((code & 3u) == 2u ? hidden : 0) + col);
            p[0] = make_float4(s[0], s[1], s[2], s[3]);
            p[1] = make_float4(s[4], s[5], s[6], s[7]);
          }
#pragma unroll
          for (int i = 0; i < 8; i++) s[i] = 0.f;
        }
      }
    }
  }
}

// One workgroup per chunk in which a run begins that goes on into later chunks: its partial
// sums are added in chunk order and the row is written.  Where the run ends is found first (a
// binary search in the sorted indices by one thread), so that the partial sums - up to a few
// hundred for the most frequent index of a large batch - can then be fetched four at a time
// instead of one after the other.
template <bool BF16>
__global__ __launch_bounds__(kEmbSortThreads) void emb_combine_kernel(const EmbSortedArgs a, const int chunk) {
  __shared__ int s_last;
  const int c = blockIdx.x;
  const int key = a.info[c].tail_key;
  if (key < 0) return;
  if (threadIdx.x == 0) {
    int lo = (c + 1) * chunk, hi = a.rows;  // first position after the run: keys[lo - 1] == key < keys[hi] (or hi == rows)
    while (lo < hi) {
      const int mid = lo + ((hi - lo) >> 1);
      if (a.keys[mid] <= (uint32_t)key)
        lo = mid + 1;
      else
        hi = mid;
    }
    s_last = (lo - 1) / chunk;  // the chunk the run ends in
  }
  __syncthreads();
  const int d_last = s_last;
  const int hidden = 2 * a.pairs;
  uint16_t* dw = reinterpret_cast<uint16_t*>(a.dw);
  for (int col = 8 * threadIdx.x; col < hidden; col += 8 * kEmbSortThreads) {
    const float4* p = reinterpret_cast<const float4*>(a.partial + ((int64_t)c * 2 + 1) * hidden + col);
    float s[8] = {p[0].x, p[0].y, p[0].z, p[0].w, p[1].x, p[1].y, p[1].z, p[1].w};
    for (int d0 = c + 1; d0 <= d_last; d0 += 4) {
      float4 t[4][2];
#pragma unroll
      for (int u = 0; u < 4; u++) {
        const float4* q = reinterpret_cast<const float4*>(a.partial + (int64_t)min(d0 + u, d_last) * 2 * hidden + col);
        t[u][0] = q[0];
        t[u][1] = q[1];
      }
#pragma unroll
      for (int u = 0; u < 4; u++) {
        if (d0 + u > d_last) break;
        s[0] += t[u][0].x, s[1] += t[u][0].y, s[2] += t[u][0].z, s[3] += t[u][0].w;
        s[4] += t[u][1].x, s[5] += t[u][1].y, s[6] += t[u][1].z, s[7] += t[u][1].w;
      }
    }
    uint4* w = reinterpret_cast<uint4*>(dw + (int64_t)key * hidden + col);
    *w = emb_finish8<BF16>(a.accumulate ? *w : make_uint4(0u, 0u, 0u, 0u), s, a.accumulate != 0);
  }
}

}  // namespace fmha
