// Dropout + residual add + LayerNorm over the rows of the packed [T, N] hidden
// states: one forward kernel and two backward kernels, the split the paper
// describes for its Dropout_Add_LayerNorm fusion (Section IV-C-1).
//
//   forward   z = x o M c + r,  y = (z - mean z) rstd gamma + beta,  rstd = (var z + eps)^-1/2
//   backward  g = dy gamma, xh = (z - mu) rstd,
//             dz = rstd (g - mean g - xh mean(g xh)),  dr = dz,  dx = dz o M c,
//             dgamma = sum_rows dy xh,  dbeta = sum_rows dy
//
// All of it is bound by HBM traffic (about 8 bytes per element forward, 8 - 10
// backward), so the layout is what matters: one wavefront owns one row at a
// time, lane l holds columns 16(l + 64i) .. +15 (two 16-byte loads per tensor
// and trip), every statistic is a wavefront reduction, nothing goes through
// LDS except the once-per-kernel column sums of the backward.  Rows are taken
// grid-stride by persistent wavefronts so that the column sums live in
// registers for the whole kernel.
//
// The dropout mask is regenerated, not stored: element (row t, column c) reads
// byte c & 15 of the Philox4x32-10 call with counter (c >> 4, t, kLnTag, 0) and
// the seed as key - one call per lane and 16 columns.
#pragma once
#include "dropout.h"

namespace fmha {

constexpr uint32_t kLnTag = 0x4C4Eu;
constexpr int kLnFwdThreads = 256;   // 4 rows in flight per workgroup
constexpr int kLnBwdThreads = 1024;  // per workgroup at CPL = 1 (16 rows in flight); 1024 / CPL in general, so
                                     // that a wavefront's register budget grows with the columns it holds

struct LnArgs {
  const int32_t* n_rows;  // device, may be null: rows actually present (<= rows)
  int32_t rows, hidden;
  float eps;
  DropArgs drop;
};

template <typename T>
struct Cvt;
template <>
struct Cvt<_Float16> {
  static __device__ __forceinline__ float lo(uint32_t w) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(w & 0xffffu)); }
  static __device__ __forceinline__ float hi(uint32_t w) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16)); }
};
template <>
struct Cvt<__bf16> {
  static __device__ __forceinline__ float lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
  static __device__ __forceinline__ float hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); }
};

// 16 consecutive 16-bit elements at p (32-byte aligned piece of a row) as floats
template <typename T>
static __device__ __forceinline__ void load16(const uint16_t* p, float (&f)[16]) {
  const u32x4 a = *reinterpret_cast<const u32x4*>(p), b = *reinterpret_cast<const u32x4*>(p + 8);
#pragma unroll
  for (int e = 0; e < 4; e++) {
    f[2 * e] = Cvt<T>::lo(a[e]);
    f[2 * e + 1] = Cvt<T>::hi(a[e]);
    f[8 + 2 * e] = Cvt<T>::lo(b[e]);
    f[8 + 2 * e + 1] = Cvt<T>::hi(b[e]);
  }
}

// the same in two steps, so that the loads of the next row can be in flight while the
// current one is worked on
struct Raw16 {
  u32x4 a, b;
};
static __device__ __forceinline__ Raw16 load16_raw(const uint16_t* p) {
  return Raw16{*reinterpret_cast<const u32x4*>(p), *reinterpret_cast<const u32x4*>(p + 8)};
}
template <typename T>
static __device__ __forceinline__ void unpack16(const Raw16& w, float (&f)[16]) {
#pragma unroll
  for (int e = 0; e < 4; e++) {
    f[2 * e] = Cvt<T>::lo(w.a[e]);
    f[2 * e + 1] = Cvt<T>::hi(w.a[e]);
    f[8 + 2 * e] = Cvt<T>::lo(w.b[e]);
    f[8 + 2 * e + 1] = Cvt<T>::hi(w.b[e]);
  }
}

template <typename T>
static __device__ __forceinline__ void store16(uint16_t* p, const float (&f)[16]) {
  u32x4 a, b;
#pragma unroll
  for (int e = 0; e < 4; e++) {
    a[e] = Op<T>::pack2(f[2 * e], f[2 * e + 1]);
    b[e] = Op<T>::pack2(f[8 + 2 * e], f[8 + 2 * e + 1]);
  }
  *reinterpret_cast<u32x4*>(p) = a;
  *reinterpret_cast<u32x4*>(p + 8) = b;
}

static __device__ __forceinline__ void load16f(const float* p, float (&f)[16]) {
#pragma unroll
  for (int e = 0; e < 4; e++) {
    const float4 v = *reinterpret_cast<const float4*>(p + 4 * e);
    f[4 * e] = v.x, f[4 * e + 1] = v.y, f[4 * e + 2] = v.z, f[4 * e + 3] = v.w;
  }
}

static __device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
  return v;
}

// keep factors (0 or c) of the 16 columns of chunk ci in row `row`
static __device__ __forceinline__ void keep16(float (&m)[16], int ci, int row, const DropArgs& d) {
  const u32x4 w = philox4x32_10((uint32_t)ci, (uint32_t)row, kLnTag, 0u, d.k0, d.k1);
#pragma unroll
  for (int k = 0; k < 16; k++) m[k] = ((w[k >> 2] >> (8 * (k & 3))) & 0xffu) >= d.thr ? d.rp : 0.f;
}

static __device__ __forceinline__ int ln_rows(const LnArgs& a) {
  int n = a.rows;
  if (a.n_rows) n = min(max(*a.n_rows, 0), n);
  return n;
}

// CPL = 16-column chunks per lane: hidden <= 1024 * CPL.
template <typename T, int CPL, bool DROP>
__global__ __launch_bounds__(kLnFwdThreads) void ln_fwd_kernel(const LnArgs a, const uint16_t* __restrict__ x,
                                                               const uint16_t* __restrict__ r,
                                                               const float* __restrict__ gamma,
                                                               const float* __restrict__ beta,
                                                               uint16_t* __restrict__ y, uint16_t* __restrict__ z,
                                                               float* __restrict__ mu, float* __restrict__ rstd) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int n = a.hidden, rows = ln_rows(a);
  const float inv_n = 1.f / (float)n;
  const int per_grid = gridDim.x * (kLnFwdThreads / 64);
  // the next row's x and residual are requested before the current row is worked on
  Raw16 nx[CPL], nr[CPL];
  auto fetch = [&](int row) {
    const int64_t base = (int64_t)row * n;
#pragma unroll
    for (int i = 0; i < CPL; i++) {
      const int ci = lane + 64 * i;
      if (16 * ci < n) {
        nx[i] = load16_raw(x + base + 16 * ci);
        nr[i] = load16_raw(r + base + 16 * ci);
      }
    }
  };
  const int first = blockIdx.x * (kLnFwdThreads / 64) + wave;
  if (first < rows) fetch(first);
  for (int row = first; row < rows; row += per_grid) {
    const int64_t base = (int64_t)row * n;
    float zf[CPL][16];
    float sum = 0.f;
    Raw16 cx[CPL], cr[CPL];
#pragma unroll
    for (int i = 0; i < CPL; i++) {
      cx[i] = nx[i];
      cr[i] = nr[i];
    }
    if (row + per_grid < rows) fetch(row + per_grid);
#pragma unroll
    for (int i = 0; i < CPL; i++) {
      const int ci = lane + 64 * i;
      if (16 * ci < n) {
        float xf[16], rf[16];
        unpack16<T>(cx[i], xf);
        unpack16<T>(cr[i], rf);
        if (DROP) {
          float m[16];
          keep16(m, ci, row, a.drop);
#pragma unroll
          for (int k = 0; k < 16; k++) zf[i][k] = __builtin_fmaf(xf[k], m[k], rf[k]);
        } else {
#pragma unroll
          for (int k = 0; k < 16; k++) zf[i][k] = xf[k] + rf[k];
        }
#pragma unroll
        for (int k = 0; k < 16; k++) sum += zf[i][k];
      } else {
#pragma unroll
        for (int k = 0; k < 16; k++) zf[i][k] = 0.f;
      }
    }
    const float mean = wave_sum(sum) * inv_n;
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < CPL; i++)
      if (16 * (lane + 64 * i) < n) {
#pragma unroll
        for (int k = 0; k < 16; k++) {
          const float dlt = zf[i][k] - mean;
          sq = __builtin_fmaf(dlt, dlt, sq);
        }
      }
    const float rs = 1.f / __builtin_sqrtf(wave_sum(sq) * inv_n + a.eps);
    if (lane == 0) {
      mu[row] = mean;
      rstd[row] = rs;
    }
#pragma unroll
    for (int i = 0; i < CPL; i++) {
      const int ci = lane + 64 * i;
      if (16 * ci < n) {
        float gf[16], bf[16], yf[16];
        load16f(gamma + 16 * ci, gf);
        load16f(beta + 16 * ci, bf);
#pragma unroll
        for (int k = 0; k < 16; k++) yf[k] = __builtin_fmaf((zf[i][k] - mean) * rs, gf[k], bf[k]);
        store16<T>(y + base + 16 * ci, yf);
        store16<T>(z + base + 16 * ci, zf[i]);
      }
    }
  }
}

// Backward, kernel 1 of 2: dx, dr per row, and this workgroup's column sums of dy xh and dy
// into partial[blockIdx.x][0 | 1][hidden].
template <typename T, int CPL, bool DROP>
__global__ __launch_bounds__(kLnBwdThreads / CPL) void ln_bwd_rows_kernel(const LnArgs a, const uint16_t* __restrict__ dy,
                                                                    const uint16_t* __restrict__ z,
                                                                    const float* __restrict__ mu,
                                                                    const float* __restrict__ rstd,
                                                                    const float* __restrict__ gamma,
                                                                    uint16_t* __restrict__ dx, uint16_t* __restrict__ dr,
                                                                    float* __restrict__ partial) {
  __shared__ __align__(16) float colsum[(kLnBwdThreads / CPL / 64 / 2) * 1024 * CPL];  // 32 KB
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int n = a.hidden, rows = ln_rows(a);
  const float inv_n = 1.f / (float)n;
  constexpr int kThreadsHere = kLnBwdThreads / CPL, kWaves = kThreadsHere / 64;
  const int per_grid = gridDim.x * kWaves;
  float acc_g[CPL][16], acc_b[CPL][16];
#pragma unroll
  for (int i = 0; i < CPL; i++)
#pragma unroll
    for (int k = 0; k < 16; k++) acc_g[i][k] = acc_b[i][k] = 0.f;

  for (int row = blockIdx.x * kWaves + wave; row < rows; row += per_grid) {
    const int64_t base = (int64_t)row * n;
    const float mean = mu[row], rs = rstd[row];
    float g[CPL][16], xh[CPL][16];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < CPL; i++) {
      const int ci = lane + 64 * i;
      if (16 * ci < n) {
        float dyf[16], zf[16], gf[16];
        load16<T>(dy + base + 16 * ci, dyf);
        load16<T>(z + base + 16 * ci, zf);
        load16f(gamma + 16 * ci, gf);
#pragma unroll
        for (int k = 0; k < 16; k++) {
          xh[i][k] = (zf[k] - mean) * rs;
          g[i][k] = dyf[k] * gf[k];
          s1 += g[i][k];
          s2 = __builtin_fmaf(g[i][k], xh[i][k], s2);
          acc_g[i][k] = __builtin_fmaf(dyf[k], xh[i][k], acc_g[i][k]);
          acc_b[i][k] += dyf[k];
        }
      }
    }
    const float m1 = wave_sum(s1) * inv_n, m2 = wave_sum(s2) * inv_n;
#pragma unroll
    for (int i = 0; i < CPL; i++) {
      const int ci = lane + 64 * i;
      if (16 * ci < n) {
        float dz[16];
#pragma unroll
        for (int k = 0; k < 16; k++) dz[k] = rs * (g[i][k] - m1 - xh[i][k] * m2);
        if (dr) store16<T>(dr + base + 16 * ci, dz);
        if (DROP) {
          float m[16];
          keep16(m, ci, row, a.drop);
#pragma unroll
          for (int k = 0; k < 16; k++) dz[k] *= m[k];
        }
        store16<T>(dx + base + 16 * ci, dz);
      }
    }
  }

  // Column sums over the workgroup's wavefronts by halving: the upper half of the live
  // wavefronts hands its sums over through LDS, the lower half adds them, until wavefront 0
  // holds the total.  A fixed tree: results do not change from run to run.
#pragma unroll
  for (int which = 0; which < 2; which++) {
    float(&acc)[CPL][16] = which == 0 ? acc_g : acc_b;
    for (int half = kWaves / 2; half >= 1; half >>= 1) {
      if (wave >= half && wave < 2 * half) {
#pragma unroll
        for (int i = 0; i < CPL; i++) {
          const int ci = lane + 64 * i;
          if (16 * ci < n) {
            float* s = &colsum[(wave - half) * (1024 * CPL) + 16 * ci];
#pragma unroll
            for (int k4 = 0; k4 < 4; k4++)
              *reinterpret_cast<float4*>(s + 4 * k4) =
                  make_float4(acc[i][4 * k4], acc[i][4 * k4 + 1], acc[i][4 * k4 + 2], acc[i][4 * k4 + 3]);
          }
        }
      }
      __syncthreads();
      if (wave < half) {
#pragma unroll
        for (int i = 0; i < CPL; i++) {
          const int ci = lane + 64 * i;
          if (16 * ci < n) {
            const float* s = &colsum[wave * (1024 * CPL) + 16 * ci];
#pragma unroll
            for (int k4 = 0; k4 < 4; k4++) {
              const float4 v = *reinterpret_cast<const float4*>(s + 4 * k4);
              acc[i][4 * k4] += v.x, acc[i][4 * k4 + 1] += v.y, acc[i][4 * k4 + 2] += v.z, acc[i][4 * k4 + 3] += v.w;
            }
          }
        }
      }
      __syncthreads();
    }
    if (wave == 0) {
      float* out = partial + ((int64_t)blockIdx.x * 2 + which) * n;
#pragma unroll
      for (int i = 0; i < CPL; i++) {
        const int ci = lane + 64 * i;
        if (16 * ci < n) {
#pragma unroll
          for (int k4 = 0; k4 < 4; k4++)
            *reinterpret_cast<float4*>(out + 16 * ci + 4 * k4) =
                make_float4(acc[i][4 * k4], acc[i][4 * k4 + 1], acc[i][4 * k4 + 2], acc[i][4 * k4 + 3]);
        }
      }
    }
  }
}

// Backward, kernel 2 of 2: dgamma, dbeta <- sums of the workgroups' partial column sums.
// One workgroup per 64 columns and output; its 16 wavefronts split the partial rows (four
// independent running sums each, so that the loads overlap), then combine in a fixed order.
constexpr int kLnColsThreads = 1024;
__global__ __launch_bounds__(kLnColsThreads) void ln_bwd_cols_kernel(const float* __restrict__ partial, int n_partial,
                                                                     int n, float* __restrict__ dgamma,
                                                                     float* __restrict__ dbeta) {
  constexpr int kWaves = kLnColsThreads / 64;
  __shared__ float part[kWaves][64];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int which = blockIdx.y;
  const int c = blockIdx.x * 64 + lane;
  float s[4] = {0.f, 0.f, 0.f, 0.f};
  if (c < n) {
    const float* p = partial + (int64_t)which * n + c;
    const int64_t step = 2 * (int64_t)n;
    int b = wave;
    for (; b + 3 * kWaves < n_partial; b += 4 * kWaves) {
#pragma unroll
      for (int u = 0; u < 4; u++) s[u] += p[(int64_t)(b + u * kWaves) * step];
    }
    for (; b < n_partial; b += kWaves) s[0] += p[(int64_t)b * step];
  }
  part[wave][lane] = (s[0] + s[1]) + (s[2] + s[3]);
  __syncthreads();
  if (wave == 0 && c < n) {
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; w++) t += part[w][lane];
    (which == 0 ? dgamma : dbeta)[c] = t;
  }
}

}  // namespace fmha
