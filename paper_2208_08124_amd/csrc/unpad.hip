// Host side of the padded <-> unpadded entry points declared in
// include/fmha_varlen.h: argument checks (host memory only) and launches on the
// caller's stream.  Nothing here allocates, copies to the host or waits.
#include <hip/hip_runtime.h>

#include "../../include/fmha_varlen.h"
#include "host_error.h"
#include "unpad_kernels.h"

namespace {

using fmha_host::fail;

int launched(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(FMHA_ERR_HIP, "%s launch failed: %s", what, hipGetErrorString(e));
  return FMHA_OK;
}

bool misaligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

int check_rows(const void* src, const void* dst, const int32_t* map, const int32_t* n_rows, int64_t src_rows,
               int64_t dst_rows, int64_t row_bytes) {
  if (!src || !dst || !map || !n_rows) return fail(FMHA_ERR_INVALID_ARG, "null pointer");
  if (misaligned(src, 16) || misaligned(dst, 16)) return fail(FMHA_ERR_INVALID_ARG, "row buffers must be 16-byte aligned");
  if (misaligned(map, 4) || misaligned(n_rows, 4)) return fail(FMHA_ERR_INVALID_ARG, "index arrays must be 4-byte aligned");
  if (row_bytes <= 0 || (row_bytes & 15)) return fail(FMHA_ERR_INVALID_ARG, "row_bytes=%lld must be a positive multiple of 16", (long long)row_bytes);
  if (row_bytes / 16 > 0x7fffffff) return fail(FMHA_ERR_INVALID_ARG, "row_bytes too large");
  if (src_rows < 0 || dst_rows < 0 || src_rows > 0x7fffffff || dst_rows > 0x7fffffff)
    return fail(FMHA_ERR_INVALID_ARG, "row counts must be in [0, 2^31)");
  return FMHA_OK;
}

unsigned copy_grid(int64_t rows, int64_t chunks) {
  const int64_t want = (rows * chunks + 1023) / 1024;  // four pieces per thread and trip
  const int64_t cap = 256 * 16;  // 16 workgroups per compute unit keep every memory channel busy
  return (unsigned)(want < 1 ? 1 : (want > cap ? cap : want));
}

}  // namespace

extern "C" {

int fmha_unpad_indices_host(const int32_t* input_mask, int32_t batch, int32_t seqlen, int32_t* nonzero_indices,
                            int32_t* inverse, int32_t* cu_seqlens, int32_t* max_seqlen) {
  if (batch < 0 || seqlen < 0) return fail(FMHA_ERR_INVALID_ARG, "batch=%d, seqlen=%d must not be negative", batch, seqlen);
  if ((int64_t)batch * seqlen > 0x7fffffff) return fail(FMHA_ERR_INVALID_ARG, "batch*seqlen exceeds 2^31-1");
  if (!cu_seqlens || (!input_mask && (int64_t)batch * seqlen > 0)) return fail(FMHA_ERR_INVALID_ARG, "null pointer");
  fmha_host::g_err[0] = 0;
  int32_t n = 0, longest = 0;
  cu_seqlens[0] = 0;
  for (int32_t b = 0; b < batch; b++) {
    const int32_t start = n;
    for (int32_t s = 0; s < seqlen; s++) {
      const int64_t pos = (int64_t)b * seqlen + s;
      const bool nz = input_mask[pos] != 0;
      if (nz && nonzero_indices) nonzero_indices[n] = (int32_t)pos;
      if (inverse) inverse[pos] = nz ? n : -1;
      n += nz;
    }
    cu_seqlens[b + 1] = n;
    if (n - start > longest) longest = n - start;
  }
  if (max_seqlen) *max_seqlen = longest;
  return FMHA_OK;
}

int fmha_unpad_indices(const int32_t* input_mask, int32_t batch, int32_t seqlen, int32_t* nonzero_indices,
                       int32_t* inverse, int32_t* cu_seqlens, void* stream) {
  if (batch < 0 || seqlen < 0) return fail(FMHA_ERR_INVALID_ARG, "batch=%d, seqlen=%d must not be negative", batch, seqlen);
  if ((int64_t)batch * seqlen > 0x7fffffff) return fail(FMHA_ERR_INVALID_ARG, "batch*seqlen exceeds 2^31-1");
  if (!cu_seqlens || ((!input_mask || !nonzero_indices) && (int64_t)batch * seqlen > 0))
    return fail(FMHA_ERR_INVALID_ARG, "null pointer");
  if (misaligned(input_mask, 4) || misaligned(nonzero_indices, 4) || misaligned(inverse, 4) || misaligned(cu_seqlens, 4))
    return fail(FMHA_ERR_INVALID_ARG, "arrays must be 4-byte aligned");
  fmha_host::g_err[0] = 0;
  hipStream_t st = static_cast<hipStream_t>(stream);
  int rc;
  const int per = fmha::kUnpadThreads / 64;
  const unsigned grid = (unsigned)((batch + per - 1) / per);
  if (batch == 0) {  // only cu[0] = 0 to write
    fmha::prefix_sum_kernel<<<1, fmha::kScanThreads, 0, st>>>(cu_seqlens, 0);
    return launched("prefix sum");
  }
  fmha::mask_count_kernel<<<grid, fmha::kUnpadThreads, 0, st>>>(input_mask, batch, seqlen, cu_seqlens);
  if ((rc = launched("mask count"))) return rc;
  fmha::prefix_sum_kernel<<<1, fmha::kScanThreads, 0, st>>>(cu_seqlens, batch);
  if ((rc = launched("prefix sum"))) return rc;
  fmha::mask_fill_kernel<<<grid, fmha::kUnpadThreads, 0, st>>>(input_mask, batch, seqlen, cu_seqlens, nonzero_indices, inverse);
  return launched("mask fill");
}

int fmha_gather_rows(const void* padded, int32_t padded_rows, const int32_t* nonzero_indices, const int32_t* n_rows,
                     int32_t packed_rows, int64_t row_bytes, void* packed, void* stream) {
  if (packed_rows == 0) {  // nothing can be written: the buffers may be null
    fmha_host::g_err[0] = 0;
    return FMHA_OK;
  }
  int rc = check_rows(padded, packed, nonzero_indices, n_rows, padded_rows, packed_rows, row_bytes);
  if (rc) return rc;
  fmha_host::g_err[0] = 0;
  const int chunks = (int)(row_bytes / 16);
  fmha::gather_rows_kernel<<<copy_grid(packed_rows, chunks), 256, 0, static_cast<hipStream_t>(stream)>>>(
      static_cast<const uint4*>(padded), nonzero_indices, n_rows, padded_rows, chunks, packed_rows,
      static_cast<uint4*>(packed));
  return launched("gather");
}

int fmha_scatter_rows(const void* packed, int32_t packed_rows, const int32_t* inverse, const int32_t* n_rows,
                      int32_t padded_rows, int64_t row_bytes, void* padded, void* stream) {
  if (padded_rows == 0) {  // nothing to write: the buffers may be null
    fmha_host::g_err[0] = 0;
    return FMHA_OK;
  }
  int rc = check_rows(packed, padded, inverse, n_rows, packed_rows, padded_rows, row_bytes);
  if (rc) return rc;
  fmha_host::g_err[0] = 0;
  const int chunks = (int)(row_bytes / 16);
  fmha::scatter_rows_kernel<<<copy_grid(padded_rows, chunks), 256, 0, static_cast<hipStream_t>(stream)>>>(
      static_cast<const uint4*>(packed), inverse, n_rows, packed_rows, chunks, padded_rows,
      static_cast<uint4*>(padded));
  return launched("scatter");
}

}  // extern "C"
