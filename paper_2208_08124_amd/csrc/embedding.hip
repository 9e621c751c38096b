// Host side of fmha_embedding_bwd (include/fmha_varlen.h): argument checks (host memory
// only) and launches on the caller's stream.  Nothing here allocates, copies to the host or waits.
#include <hip/hip_runtime.h>

#include "../../include/fmha_varlen.h"
#include "embedding_kernels.h"
#include "host_error.h"

namespace {
using fmha_host::fail;
bool misaligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }
}  // namespace

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
