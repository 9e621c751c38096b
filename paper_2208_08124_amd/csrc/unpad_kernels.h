// Between the padded [batch, max_seq_len] input format and the paper's
// unpadded storage (Section IV-A-1): where the valid tokens are
// (nonzero_indices, Section IV-B-2), how many each sequence has (batch_offset),
// and the row copies in both directions (gather / scatter).  Integer and
// copy work only; all of it bound by HBM traffic, none of it by arithmetic.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fmha {

constexpr int kUnpadThreads = 256;  // 4 wavefronts, one mask row each
constexpr int kScanThreads = 1024;

// cu[row + 1] <- number of non-zero entries in row `row` of the mask.
__global__ __launch_bounds__(kUnpadThreads) void mask_count_kernel(const int32_t* __restrict__ mask, int batch,
                                                                   int seqlen, int32_t* __restrict__ cu) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int row = blockIdx.x * (kUnpadThreads / 64) + wave;
  if (row >= batch) return;  // uniform over the wavefront
  const int32_t* m = mask + (int64_t)row * seqlen;
  int count = 0;
  for (int s0 = 0; s0 < seqlen; s0 += 64) {
    const int s = s0 + lane;
    const bool nz = s < seqlen && m[s] != 0;
    count += __popcll(__ballot(nz));
  }
  if (lane == 0) cu[row + 1] = count;
}

// In place, one workgroup: cu[0] <- 0, cu[1..batch] <- inclusive prefix sums of itself.
__global__ __launch_bounds__(kScanThreads) void prefix_sum_kernel(int32_t* cu, int batch) {
  __shared__ int part[kScanThreads];
  const int tid = threadIdx.x;
  const int per = (batch + kScanThreads - 1) / kScanThreads;  // consecutive entries per thread
  const int lo = min(tid * per, batch), hi = min(lo + per, batch);
  int sum = 0;
  for (int i = lo; i < hi; i++) sum += cu[1 + i];
  part[tid] = sum;
  __syncthreads();
  for (int d = 1; d < kScanThreads; d <<= 1) {  // Hillis-Steele over the thread sums
    const int add = tid >= d ? part[tid - d] : 0;
    __syncthreads();
    part[tid] += add;
    __syncthreads();
  }
  if (tid == 0) cu[0] = 0;
  int run = part[tid] - sum;  // exclusive
  for (int i = lo; i < hi; i++) {
    run += cu[1 + i];
    cu[1 + i] = run;
  }
}

// With cu holding the prefix sums: the flat positions of the non-zero entries in
// ascending order, and for every flat position its rank among them (or -1).
__global__ __launch_bounds__(kUnpadThreads) void mask_fill_kernel(const int32_t* __restrict__ mask, int batch,
                                                                  int seqlen, const int32_t* __restrict__ cu,
                                                                  int32_t* __restrict__ nonzero_indices,
                                                                  int32_t* __restrict__ inverse) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int row = blockIdx.x * (kUnpadThreads / 64) + wave;
  if (row >= batch) return;
  const int32_t* m = mask + (int64_t)row * seqlen;
  int base = cu[row];
  for (int s0 = 0; s0 < seqlen; s0 += 64) {
    const int s = s0 + lane;
    const bool nz = s < seqlen && m[s] != 0;
    const uint64_t bal = __ballot(nz);
    const int rank = base + __popcll(bal & ((1ull << lane) - 1ull));
    const int64_t pos = (int64_t)row * seqlen + s;
    if (nz) nonzero_indices[rank] = (int32_t)pos;
    if (inverse && s < seqlen) inverse[pos] = nz ? rank : -1;
    base += __popcll(bal);
  }
}

// dst row j <- src row idx[j] for j < *n_rows; rows are `chunks` pieces of 16 bytes.
// An index outside [0, src_rows) yields a row of zeros instead of a wild read.
__global__ __launch_bounds__(256) void gather_rows_kernel(const uint4* __restrict__ src, const int32_t* __restrict__ idx,
                                                          const int32_t* __restrict__ n_rows, int src_rows,
                                                          int chunks, int dst_rows, uint4* __restrict__ dst) {
  const int n = min(max(*n_rows, 0), dst_rows);
  const int64_t total = (int64_t)n * chunks;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  // four independent 16-byte pieces per thread and trip: all loads are issued before
  // the first store, which keeps enough bytes in flight to cover the HBM latency
  for (int64_t i0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i0 < total; i0 += 4 * stride) {
    uint4 v[4];
#pragma unroll
    for (int u = 0; u < 4; u++) {
      const int64_t i = i0 + u * stride;
      v[u] = make_uint4(0u, 0u, 0u, 0u);
      if (i < total) {
        const int j = (int)(i / chunks), c = (int)(i - (int64_t)j * chunks);
        const int r = idx[j];
        if (r >= 0 && r < src_rows) v[u] = src[(int64_t)r * chunks + c];
      }
    }
#pragma unroll
    for (int u = 0; u < 4; u++) {
      const int64_t i = i0 + u * stride;
      if (i < total) dst[i] = v[u];
    }
  }
}

// dst row r <- src row inverse[r] if that is a valid packed row, else zeros; every
// one of the dst_rows rows is written exactly once.
__global__ __launch_bounds__(256) void scatter_rows_kernel(const uint4* __restrict__ src,
                                                           const int32_t* __restrict__ inverse,
                                                           const int32_t* __restrict__ n_rows, int src_rows,
                                                           int chunks, int dst_rows, uint4* __restrict__ dst) {
  const int n = min(max(*n_rows, 0), src_rows);
  const int64_t total = (int64_t)dst_rows * chunks;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i0 < total; i0 += 4 * stride) {
    uint4 v[4];
#pragma unroll
    for (int u = 0; u < 4; u++) {
      const int64_t i = i0 + u * stride;
      v[u] = make_uint4(0u, 0u, 0u, 0u);
      if (i < total) {
        const int r = (int)(i / chunks), c = (int)(i - (int64_t)r * chunks);
        const int j = inverse[r];
        if (j >= 0 && j < n) v[u] = src[(int64_t)j * chunks + c];
      }
    }
#pragma unroll
    for (int u = 0; u < 4; u++) {
      const int64_t i = i0 + u * stride;
      if (i < total) dst[i] = v[u];
    }
  }
}

}  // namespace fmha
