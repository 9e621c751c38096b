// Host side of the Dropout + Add + LayerNorm entry points declared in
// include/fmha_varlen.h: argument checks (host memory only) and launches on the
// caller's stream.  Nothing here allocates, copies to the host or waits.
#include <hip/hip_runtime.h>

#include "../../include/fmha_varlen.h"
#include "host_error.h"
#include "layernorm_kernels.h"

namespace {

using fmha_host::fail;

bool misaligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

int chunks_per_lane(int hidden) { return hidden <= 1024 ? 1 : (hidden <= 2048 ? 2 : 4); }

int bwd_waves(int hidden) { return fmha::kLnBwdThreads / chunks_per_lane(hidden) / 64; }

// Workgroups of the first backward kernel: one per compute unit's worth of registers
// (256 * CPL), fewer if the rows run out.
int bwd_grid(int rows, int hidden) {
  const int w = bwd_waves(hidden);
  int64_t g = ((int64_t)rows + w - 1) / w;
  const int64_t cap = 256 * chunks_per_lane(hidden);
  if (g > cap) g = cap;
  return (int)(g < 1 ? 1 : g);
}

int check(const fmha_ln_params_t* p, fmha::LnArgs* a) {
  if (!p) return fail(FMHA_ERR_INVALID_ARG, "params is null");
  if (p->dtype != FMHA_F16 && p->dtype != FMHA_BF16) return fail(FMHA_ERR_UNSUPPORTED, "dtype=%d is neither FMHA_F16 nor FMHA_BF16", p->dtype);
  if (p->rows < 0) return fail(FMHA_ERR_INVALID_ARG, "rows=%d is negative", p->rows);
  if (p->hidden <= 0 || (p->hidden & 15)) return fail(FMHA_ERR_INVALID_ARG, "hidden=%d must be a positive multiple of 16", p->hidden);
  if (p->hidden > 4096) return fail(FMHA_ERR_UNSUPPORTED, "hidden=%d, at most 4096 is supported", p->hidden);
  if (!(p->eps >= 0.f) || p->eps - p->eps != 0.f) return fail(FMHA_ERR_INVALID_ARG, "eps must be finite and not negative");
  if (!(p->dropout.p >= 0.f && p->dropout.p < 1.f)) return fail(FMHA_ERR_INVALID_ARG, "dropout p=%g is not in [0, 1)", (double)p->dropout.p);
  if (p->n_rows && misaligned(p->n_rows, 4)) return fail(FMHA_ERR_INVALID_ARG, "n_rows must be 4-byte aligned");
  int t = (int)(256.f * p->dropout.p + 0.5f);
  if (t > 255) t = 255;
  a->n_rows = p->n_rows;
  a->rows = p->rows;
  a->hidden = p->hidden;
  a->eps = p->eps;
  a->drop = fmha::DropArgs{(uint32_t)t, (uint32_t)(p->dropout.seed & 0xffffffffu), (uint32_t)(p->dropout.seed >> 32),
                           256.f / (float)(256 - t)};
  return FMHA_OK;
}

int check_ptr(const char* name, const void* ptr, size_t align) {
  if (!ptr) return fail(FMHA_ERR_INVALID_ARG, "%s is null", name);
  if (misaligned(ptr, align)) return fail(FMHA_ERR_INVALID_ARG, "%s is not %zu-byte aligned", name, align);
  return FMHA_OK;
}

template <typename T, int CPL>
void launch_fwd(const fmha::LnArgs& a, unsigned grid, hipStream_t st, const void* x, const void* r, const float* gamma,
                const float* beta, void* y, void* z, float* mu, float* rstd) {
  auto xs = static_cast<const uint16_t*>(x), rs = static_cast<const uint16_t*>(r);
  auto ys = static_cast<uint16_t*>(y), zs = static_cast<uint16_t*>(z);
  if (a.drop.thr)
    fmha::ln_fwd_kernel<T, CPL, true><<<grid, fmha::kLnFwdThreads, 0, st>>>(a, xs, rs, gamma, beta, ys, zs, mu, rstd);
  else
    fmha::ln_fwd_kernel<T, CPL, false><<<grid, fmha::kLnFwdThreads, 0, st>>>(a, xs, rs, gamma, beta, ys, zs, mu, rstd);
}

template <typename T, int CPL>
void launch_bwd(const fmha::LnArgs& a, unsigned grid, hipStream_t st, const void* dy, const void* z, const float* mu,
                const float* rstd, const float* gamma, void* dx, void* dr, float* partial) {
  auto dys = static_cast<const uint16_t*>(dy), zs = static_cast<const uint16_t*>(z);
  auto dxs = static_cast<uint16_t*>(dx), drs = static_cast<uint16_t*>(dr);
  constexpr int threads = fmha::kLnBwdThreads / CPL;
  if (a.drop.thr)
    fmha::ln_bwd_rows_kernel<T, CPL, true><<<grid, threads, 0, st>>>(a, dys, zs, mu, rstd, gamma, dxs, drs, partial);
  else
    fmha::ln_bwd_rows_kernel<T, CPL, false><<<grid, threads, 0, st>>>(a, dys, zs, mu, rstd, gamma, dxs, drs, partial);
}

}  // namespace

extern "C" {

size_t fmha_dropout_add_ln_bwd_workspace_size(int32_t rows, int32_t hidden) {
  if (rows < 0 || hidden <= 0 || (hidden & 15) || hidden > 4096) return 0;
  return (size_t)bwd_grid(rows, hidden) * 2 * (size_t)hidden * sizeof(float);
}

int fmha_dropout_add_ln_fwd(const fmha_ln_params_t* p, const void* x, const void* residual, const float* gamma,
                            const float* beta, void* y, void* z, float* mu, float* rstd, void* stream) {
  fmha::LnArgs a;
  int rc = check(p, &a);
  if (rc) return rc;
  fmha_host::g_err[0] = 0;
  if (a.rows == 0) return FMHA_OK;  // nothing to read or write: the row buffers may be null
  if ((rc = check_ptr("x", x, 16)) || (rc = check_ptr("residual", residual, 16)) || (rc = check_ptr("gamma", gamma, 16)) ||
      (rc = check_ptr("beta", beta, 16)) || (rc = check_ptr("y", y, 16)) || (rc = check_ptr("z", z, 16)) ||
      (rc = check_ptr("mu", mu, 4)) || (rc = check_ptr("rstd", rstd, 4)))
    return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int per = fmha::kLnFwdThreads / 64;
  int64_t g = ((int64_t)a.rows + per - 1) / per;
  if (g > 256 * 8) g = 256 * 8;  // 8 workgroups (32 rows) per compute unit in flight, the rest grid-stride
  const unsigned grid = (unsigned)g;
  const int cpl = chunks_per_lane(a.hidden);
  const bool f16 = p->dtype == FMHA_F16;
  if (cpl == 1)
    f16 ? launch_fwd<_Float16, 1>(a, grid, st, x, residual, gamma, beta, y, z, mu, rstd)
        : launch_fwd<__bf16, 1>(a, grid, st, x, residual, gamma, beta, y, z, mu, rstd);
  else if (cpl == 2)
    f16 ? launch_fwd<_Float16, 2>(a, grid, st, x, residual, gamma, beta, y, z, mu, rstd)
        : launch_fwd<__bf16, 2>(a, grid, st, x, residual, gamma, beta, y, z, mu, rstd);
  else
    f16 ? launch_fwd<_Float16, 4>(a, grid, st, x, residual, gamma, beta, y, z, mu, rstd)
        : launch_fwd<__bf16, 4>(a, grid, st, x, residual, gamma, beta, y, z, mu, rstd);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(FMHA_ERR_HIP, "LayerNorm forward launch failed: %s", hipGetErrorString(e));
  return FMHA_OK;
}

int fmha_dropout_add_ln_bwd(const fmha_ln_params_t* p, const void* dy, const void* z, const float* mu,
                            const float* rstd, const float* gamma, void* dx, void* dresidual, float* dgamma,
                            float* dbeta, void* workspace, size_t workspace_bytes, void* stream) {
  fmha::LnArgs a;
  int rc = check(p, &a);
  if (rc) return rc;
  // with no rows the row buffers may be null: the kernels never touch them, but dgamma and
  // dbeta are still written (zeros)
  if (a.rows > 0 &&
      ((rc = check_ptr("dy", dy, 16)) || (rc = check_ptr("z", z, 16)) || (rc = check_ptr("mu", mu, 4)) ||
       (rc = check_ptr("rstd", rstd, 4)) || (rc = check_ptr("dx", dx, 16))))
    return rc;
  if ((rc = check_ptr("gamma", gamma, 16)) || (rc = check_ptr("dgamma", dgamma, 4)) || (rc = check_ptr("dbeta", dbeta, 4)))
    return rc;
  if (dresidual && misaligned(dresidual, 16)) return fail(FMHA_ERR_INVALID_ARG, "dresidual is not 16-byte aligned");
  const size_t need = fmha_dropout_add_ln_bwd_workspace_size(a.rows, a.hidden);
  if (!workspace || misaligned(workspace, 16)) return fail(FMHA_ERR_WORKSPACE, "workspace is null or not 16-byte aligned (%zu bytes needed)", need);
  if (workspace_bytes < need) return fail(FMHA_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
  fmha_host::g_err[0] = 0;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const unsigned grid = (unsigned)bwd_grid(a.rows, a.hidden);
  float* partial = static_cast<float*>(workspace);
  const int cpl = chunks_per_lane(a.hidden);
  const bool f16 = p->dtype == FMHA_F16;
  // with no rows the first kernel still runs: it writes zero column sums
  if (cpl == 1)
    f16 ? launch_bwd<_Float16, 1>(a, grid, st, dy, z, mu, rstd, gamma, dx, dresidual, partial)
        : launch_bwd<__bf16, 1>(a, grid, st, dy, z, mu, rstd, gamma, dx, dresidual, partial);
  else if (cpl == 2)
    f16 ? launch_bwd<_Float16, 2>(a, grid, st, dy, z, mu, rstd, gamma, dx, dresidual, partial)
        : launch_bwd<__bf16, 2>(a, grid, st, dy, z, mu, rstd, gamma, dx, dresidual, partial);
  else
    f16 ? launch_bwd<_Float16, 4>(a, grid, st, dy, z, mu, rstd, gamma, dx, dresidual, partial)
        : launch_bwd<__bf16, 4>(a, grid, st, dy, z, mu, rstd, gamma, dx, dresidual, partial);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(FMHA_ERR_HIP, "LayerNorm backward launch failed: %s", hipGetErrorString(e));
  fmha::ln_bwd_cols_kernel<<<dim3((unsigned)((a.hidden + 63) / 64), 2), fmha::kLnColsThreads, 0, st>>>(partial, (int)grid, a.hidden, dgamma, dbeta);
  e = hipGetLastError();
  if (e != hipSuccess) return fail(FMHA_ERR_HIP, "LayerNorm column-sum launch failed: %s", hipGetErrorString(e));
  return FMHA_OK;
}

}  // extern "C"
