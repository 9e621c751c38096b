// Host side of fmha_embedding_bwd (include/fmha_varlen.h): argument checks (host memory
// only) and launches on the caller's stream.  Nothing here allocates, copies to the host or waits.
#include <hip/hip_runtime.h>

#include <cstring>

#include <rocprim/device/device_radix_sort.hpp>

#include "../../include/fmha_varlen.h"
#include "embedding_kernels.h"
#include "embedding_sorted_kernels.h"
#include "host_error.h"

namespace {
using fmha_host::fail;
bool misaligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }
size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Chunk of sorted entries per workgroup: small batches get smaller chunks so that they still
// spread over the chip.
int sort_chunk(int rows) { return rows >= (1 << 17) ? fmha::kEmbChunk : 32; }

// Bits of the sort key: indices 0 .. vocab (vocab itself stands for "skipped").
unsigned key_bits(int vocab) {
  unsigned b = 1;
  while (b < 32 && ((uint64_t)1 << b) <= (uint64_t)vocab) b++;
  return b;
}

// Layout of the workspace of the sorted embedding backward (offsets in bytes).
struct SortSpace {
  size_t keys_in, pos_in, keys, order, info, partial, temp, temp_bytes, bytes;
  int chunks;
};
// Host arithmetic only (the sort's own temporary storage is sized by asking the sort).
bool sort_space(int rows, int hidden, SortSpace* out) {
  SortSpace s;
  const size_t n = (size_t)(rows > 0 ? rows : 1);
  s.chunks = (int)((n + sort_chunk(rows) - 1) / sort_chunk(rows));
  size_t at = 256;
  s.keys_in = at, at = round_up(at + 4 * n, 256);
  s.pos_in = at, at = round_up(at + 4 * n, 256);
  s.keys = at, at = round_up(at + 4 * n, 256);
  s.order = at, at = round_up(at + 4 * n, 256);
  s.info = at, at = round_up(at + sizeof(fmha::EmbChunkInfo) * (size_t)s.chunks, 256);
  s.partial = at, at = round_up(at + sizeof(float) * 2 * (size_t)hidden * (size_t)s.chunks, 256);
  s.temp = at;
  s.temp_bytes = 0;
  // The sort sizes its own temporary storage; where it cannot be asked (no device in this
  // process) the figure is an upper estimate: two more copies of keys and values plus its tables.
  uint32_t* none = nullptr;
  size_t asked = 0;
  const size_t estimate = 16 * n + ((size_t)1 << 20);
  if (rocprim::radix_sort_pairs(nullptr, asked, none, none, none, none, n, 0u, 32u, nullptr) != hipSuccess) asked = 0;
  s.temp_bytes = asked > estimate ? asked : estimate;
  s.bytes = round_up(at + s.temp_bytes, 256);
  *out = s;
  return true;
}
}  // namespace

extern "C" size_t fmha_embedding_sort_workspace_size(int32_t rows, int32_t hidden) {
  SortSpace s;
  if (rows < 0 || hidden <= 0 || !sort_space(rows, hidden, &s)) return 0;
  return s.bytes;
}

extern "C" int fmha_embedding_sort(const int32_t* indices, const int32_t* n_rows, int32_t rows, int32_t hidden,
                                   int32_t vocab, int32_t padding_idx, void* workspace, size_t workspace_bytes,
                                   void* stream) {
  if (rows < 0 || vocab <= 0) return fail(FMHA_ERR_INVALID_ARG, "rows=%d must not be negative and vocab=%d must be positive", rows, vocab);
  if (hidden <= 0 || (hidden & 7)) return fail(FMHA_ERR_INVALID_ARG, "hidden=%d must be a positive multiple of 8", hidden);
  if (rows > 0 && (!indices || misaligned(indices, 4))) return fail(FMHA_ERR_INVALID_ARG, "indices null or not 4-byte aligned");
  if (n_rows && misaligned(n_rows, 4)) return fail(FMHA_ERR_INVALID_ARG, "n_rows must be 4-byte aligned");
  SortSpace s;
  if (!sort_space(rows, hidden, &s)) return fail(FMHA_ERR_HIP, "sizing the sort's temporary storage failed");
  if (!workspace || misaligned(workspace, 256)) return fail(FMHA_ERR_WORKSPACE, "workspace is null or not 256-byte aligned (%zu bytes needed)", s.bytes);
  if (workspace_bytes < s.bytes) return fail(FMHA_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, s.bytes);
  fmha_host::g_err[0] = 0;
  if (rows == 0) return FMHA_OK;
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* w = static_cast<char*>(workspace);
  uint32_t* keys_in = reinterpret_cast<uint32_t*>(w + s.keys_in);
  uint32_t* pos_in = reinterpret_cast<uint32_t*>(w + s.pos_in);
  int64_t g = ((int64_t)rows + 255) / 256;
  if (g > 2048) g = 2048;
  fmha::emb_keys_kernel<<<(unsigned)g, 256, 0, st>>>(indices, n_rows, rows, vocab, padding_idx, keys_in, pos_in);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(FMHA_ERR_HIP, "key kernel launch failed: %s", hipGetErrorString(e));
  size_t temp_bytes = s.temp_bytes;
  e = rocprim::radix_sort_pairs(w + s.temp, temp_bytes, keys_in, reinterpret_cast<uint32_t*>(w + s.keys), pos_in,
                                reinterpret_cast<uint32_t*>(w + s.order), (size_t)rows, 0u, key_bits(vocab), st);
  if (e != hipSuccess) return fail(FMHA_ERR_HIP, "radix sort failed: %s", hipGetErrorString(e));
  return FMHA_OK;
}

extern "C" int fmha_embedding_bwd_sorted(const void* dy, void* workspace, size_t workspace_bytes, int32_t rows,
                                         int32_t hidden, int32_t vocab, int32_t dtype, uint32_t flags, void* dw,
                                         void* stream) {
  if (dtype != FMHA_F16 && dtype != FMHA_BF16) return fail(FMHA_ERR_UNSUPPORTED, "dtype=%d is neither FMHA_F16 nor FMHA_BF16", dtype);
  if (rows < 0 || vocab <= 0) return fail(FMHA_ERR_INVALID_ARG, "rows=%d must not be negative and vocab=%d must be positive", rows, vocab);
  if (hidden <= 0 || (hidden & 7)) return fail(FMHA_ERR_INVALID_ARG, "hidden=%d must be a positive multiple of 8", hidden);
  if (flags & ~FMHA_EMB_ZERO_FIRST) return fail(FMHA_ERR_INVALID_ARG, "flags=%u: only FMHA_EMB_ZERO_FIRST applies to the sorted variant", flags);
  if (!dw || misaligned(dw, 16)) return fail(FMHA_ERR_INVALID_ARG, "dw is null or not 16-byte aligned");
  if (rows > 0 && (!dy || misaligned(dy, 16))) return fail(FMHA_ERR_INVALID_ARG, "dy null or not 16-byte aligned");
  SortSpace s;
  if (!sort_space(rows, hidden, &s)) return fail(FMHA_ERR_HIP, "sizing the sort's temporary storage failed");
  if (!workspace || misaligned(workspace, 256)) return fail(FMHA_ERR_WORKSPACE, "workspace is null or not 256-byte aligned (%zu bytes needed)", s.bytes);
  if (workspace_bytes < s.bytes) return fail(FMHA_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, s.bytes);
  fmha_host::g_err[0] = 0;
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipError_t e;
  if (flags & FMHA_EMB_ZERO_FIRST) {
    const int64_t n16 = (int64_t)vocab * hidden * 2 / 16;
    int64_t g = (n16 + 255) / 256;
    if (g > 256 * 16) g = 256 * 16;
    fmha::zero_fill_kernel<<<(unsigned)g, 256, 0, st>>>(static_cast<uint4*>(dw), n16);
    if ((e = hipGetLastError()) != hipSuccess) return fail(FMHA_ERR_HIP, "zero fill launch failed: %s", hipGetErrorString(e));
  }
  if (rows == 0) return FMHA_OK;
  char* w = static_cast<char*>(workspace);
  fmha::EmbSortedArgs a;
  a.dy = static_cast<const uint32_t*>(dy);
  a.keys = reinterpret_cast<const uint32_t*>(w + s.keys);
  a.order = reinterpret_cast<const uint32_t*>(w + s.order);
  a.info = reinterpret_cast<fmha::EmbChunkInfo*>(w + s.info);
  a.partial = reinterpret_cast<float*>(w + s.partial);
  a.dw = static_cast<uint32_t*>(dw);
  a.rows = rows;
  a.pairs = hidden / 2;
  a.vocab = vocab;
  a.accumulate = (flags & FMHA_EMB_ZERO_FIRST) ? 0 : 1;
  const int chunk = sort_chunk(rows);
  if (dtype == FMHA_BF16) {
    fmha::emb_chunk_kernel<true><<<(unsigned)s.chunks, fmha::kEmbSortThreads, 0, st>>>(a, chunk);
    fmha::emb_combine_kernel<true><<<(unsigned)s.chunks, fmha::kEmbSortThreads, 0, st>>>(a, chunk);
  } else {
    fmha::emb_chunk_kernel<false><<<(unsigned)s.chunks, fmha::kEmbSortThreads, 0, st>>>(a, chunk);
    fmha::emb_combine_kernel<false><<<(unsigned)s.chunks, fmha::kEmbSortThreads, 0, st>>>(a, chunk);
  }
  if ((e = hipGetLastError()) != hipSuccess) return fail(FMHA_ERR_HIP, "sorted embedding backward launch failed: %s", hipGetErrorString(e));
  return FMHA_OK;
}

extern "C" int fmha_embedding_bwd(const void* dy, const int32_t* indices, const int32_t* n_rows, int32_t rows,
                                  int32_t hidden, int32_t vocab, int32_t padding_idx, int32_t dtype, uint32_t flags,
                                  void* dw, void* stream) {
  if (dtype != FMHA_F16 && dtype != FMHA_BF16) return fail(FMHA_ERR_UNSUPPORTED, "dtype=%d is neither FMHA_F16 nor FMHA_BF16", dtype);
  if (rows < 0 || vocab <= 0) return fail(FMHA_ERR_INVALID_ARG, "rows=%d must not be negative and vocab=%d must be positive", rows, vocab);
  if (hidden <= 0 || (hidden & 7)) return fail(FMHA_ERR_INVALID_ARG, "hidden=%d must be a positive multiple of 8", hidden);
  if (!dw || misaligned(dw, 16)) return fail(FMHA_ERR_INVALID_ARG, "dw is null or not 16-byte aligned");
  if (rows > 0 && (!dy || !indices || misaligned(dy, 4) || misaligned(indices, 4)))
    return fail(FMHA_ERR_INVALID_ARG, "dy / indices null or not 4-byte aligned");
  if (n_rows && misaligned(n_rows, 4)) return fail(FMHA_ERR_INVALID_ARG, "n_rows must be 4-byte aligned");
  fmha_host::g_err[0] = 0;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (flags & FMHA_EMB_ZERO_FIRST) {
    const int64_t n16 = (int64_t)vocab * hidden * 2 / 16;
    int64_t g = (n16 + 255) / 256;
    if (g > 256 * 16) g = 256 * 16;
    fmha::zero_fill_kernel<<<(unsigned)g, 256, 0, st>>>(static_cast<uint4*>(dw), n16);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(FMHA_ERR_HIP, "zero fill launch failed: %s", hipGetErrorString(e));
  }
  if (rows == 0) return FMHA_OK;
  fmha::EmbArgs a;
  a.dy = static_cast<const uint32_t*>(dy);
  a.indices = indices;
  a.n_rows = n_rows;
  a.dw = static_cast<uint32_t*>(dw);
  a.rows = rows;
  a.pairs = hidden / 2;
  a.vocab = vocab;
  a.padding_idx = padding_idx;
  const int per = fmha::kEmbThreads / 64;
  const bool bf16 = dtype == FMHA_BF16;
  if (flags & FMHA_EMB_PLAIN_SPLIT) {
    int64_t g = ((int64_t)rows + per - 1) / per;
    if (g > 256 * 8) g = 256 * 8;
    if (bf16)
      fmha::embedding_bwd_kernel<true><<<(unsigned)g, fmha::kEmbThreads, 0, st>>>(a);
    else
      fmha::embedding_bwd_kernel<false><<<(unsigned)g, fmha::kEmbThreads, 0, st>>>(a);
  } else {
    // 64-token windows while the batch is small (more workgroups), 256-token windows once
    // there are enough of them to fill the chip several times over (more merging; 128 and 512
    // were both slower on 527 340 Zipf-distributed rows: 0.74 / 0.65 / 0.82 ms)
    const int nw = rows >= (1 << 17) ? 4 : 1;
    const int window = 64 * nw;
    const bool die = !(flags & FMHA_EMB_NO_DIE_SPLIT);
    int64_t g = ((int64_t)rows + window - 1) / window;  // one window per workgroup and trip (per die, if split)
    const int64_t cap = die ? 256 : 256 * 8;
    if (g > cap) g = cap;
    if (g < 1) g = 1;
    if (die) g *= 8;
    const unsigned grid = (unsigned)g;
#define FMHA_EMB_LAUNCH(BF, DIE)                                                                          \
  do {                                                                                                    \
    if (nw == 4)                                                                                          \
      fmha::embedding_bwd_window_kernel<BF, DIE, 4><<<grid, fmha::kEmbThreads, 0, st>>>(a);               \
    else                                                                                                  \
      fmha::embedding_bwd_window_kernel<BF, DIE, 1><<<grid, fmha::kEmbThreads, 0, st>>>(a);               \
  } while (0)
    if (bf16) {
      if (die) FMHA_EMB_LAUNCH(true, true); else FMHA_EMB_LAUNCH(true, false);
    } else {
      if (die) FMHA_EMB_LAUNCH(false, true); else FMHA_EMB_LAUNCH(false, false);
    }
#undef FMHA_EMB_LAUNCH
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(FMHA_ERR_HIP, "embedding backward launch failed: %s", hipGetErrorString(e));
  return FMHA_OK;
}
