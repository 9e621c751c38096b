// Host side of the C ABI declared in include/fmha_varlen.h: argument checks
// (host memory only), workspace carving, and the launches.  One launch per
// direction and kernel on the caller's stream; nothing here allocates,
// copies to the host or waits for the device.
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>

#include "../../include/fmha_varlen.h"
#include "host_error.h"
#include "bwd_kernels.h"
#include "fwd64_kernel.h"
#include "fwd_kernel.h"
#include "keep_mask_kernel.h"
#include "schedule.h"

namespace fmha_host {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

}  // namespace fmha_host

namespace {

using fmha_host::fail;
using fmha_host::g_err;

constexpr size_t kAlign = 256;
size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Tiles of 128 rows: sum_i ceil(L_i/128) <= T/128 + B for any lengths.
int64_t tile_capacity(int64_t batch, int64_t total_tokens) {
  return total_tokens / fmha::kTileRows + batch;
}

struct Workspace {
  int32_t* count;
  uint32_t* feed;  // the item feed's counters (item_feed.h)
  fmha::TileItem* list;
  float* dsum;
  float* lse2;
  size_t count_off, feed_off, list_off, dsum_off, lse2_off, bytes_fwd, bytes_bwd;
};

Workspace carve(void* base, int64_t batch, int64_t total_tokens, int64_t heads) {
  Workspace w;
  w.count_off = 0;
  w.feed_off = kAlign;
  w.list_off = w.feed_off + sizeof(uint32_t) * fmha::kFeedWords;
  const size_t list_bytes = sizeof(fmha::TileItem) * (size_t)(tile_capacity(batch, total_tokens) + 1);
  w.dsum_off = round_up(w.list_off + list_bytes, kAlign);
  w.bytes_fwd = w.dsum_off;
  // one float per (token, head) plus one pad entry
  const size_t stat_bytes = round_up(sizeof(float) * ((size_t)total_tokens * (size_t)heads + 1), kAlign);
  w.lse2_off = w.dsum_off + stat_bytes;
  w.bytes_bwd = w.lse2_off + stat_bytes;
  // (base is null when only the sizes are wanted: no pointer arithmetic on it then)
  const uintptr_t b = reinterpret_cast<uintptr_t>(base);
  auto at = [b](size_t off) { return b ? reinterpret_cast<void*>(b + off) : nullptr; };
  w.count = static_cast<int32_t*>(at(w.count_off));
  w.feed = static_cast<uint32_t*>(at(w.feed_off));
  w.list = static_cast<fmha::TileItem*>(at(w.list_off));
  w.dsum = static_cast<float*>(at(w.dsum_off));
  w.lse2 = static_cast<float*>(at(w.lse2_off));
  return w;
}

bool misaligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

int check_stride(const char* name, int64_t s, int64_t dense, int64_t* out) {
  if (s == 0) s = dense;
  if (s < dense || (s & 7)) return fail(FMHA_ERR_INVALID_ARG, "%s_stride=%lld must be 0 or a multiple of 8 that is >= heads*64=%lld",
                                        name, (long long)s, (long long)dense);
  // the kernels address the 64 rows of a block with 32-bit byte offsets from a 64-bit base
  if (s > ((int64_t)1 << 24)) return fail(FMHA_ERR_INVALID_ARG, "%s_stride=%lld exceeds 2^24 elements", name, (long long)s);
  *out = s;
  return FMHA_OK;
}

int check_common(const fmha_varlen_params_t* p, bool bwd) {
  if (!p) return fail(FMHA_ERR_INVALID_ARG, "params is null");
  if (p->head_dim != fmha::kHeadDim) return fail(FMHA_ERR_UNSUPPORTED, "head_dim=%d, only 64 is supported", p->head_dim);
  if (p->dtype != FMHA_F16 && p->dtype != FMHA_BF16) return fail(FMHA_ERR_UNSUPPORTED, "dtype=%d is neither FMHA_F16 nor FMHA_BF16", p->dtype);
  if (p->batch < 0) return fail(FMHA_ERR_INVALID_ARG, "batch=%d is negative", p->batch);
  if (p->total_tokens < 0) return fail(FMHA_ERR_INVALID_ARG, "total_tokens=%d is negative", p->total_tokens);
  if (p->heads <= 0) return fail(FMHA_ERR_INVALID_ARG, "heads=%d must be positive", p->heads);
  if ((int64_t)p->total_tokens * p->heads > (int64_t)1 << 40) return fail(FMHA_ERR_INVALID_ARG, "total_tokens*heads too large");
  if (!(p->scale == p->scale) || p->scale - p->scale != 0.f) return fail(FMHA_ERR_INVALID_ARG, "scale is not finite");
  if (!p->cu_seqlens) return fail(FMHA_ERR_INVALID_ARG, "cu_seqlens is null");
  if (misaligned(p->cu_seqlens, 4) || (p->seqused && misaligned(p->seqused, 4)))
    return fail(FMHA_ERR_INVALID_ARG, "cu_seqlens/seqused must be 4-byte aligned");
  if (p->cu_seqlens_host) {
    const int32_t* cu = p->cu_seqlens_host;
    if (cu[0] != 0) return fail(FMHA_ERR_INVALID_ARG, "cu_seqlens_host[0]=%d, expected 0", cu[0]);
    for (int i = 0; i < p->batch; i++) {
      if (cu[i + 1] < cu[i]) return fail(FMHA_ERR_INVALID_ARG, "cu_seqlens_host decreases at %d (%d -> %d)", i, cu[i], cu[i + 1]);
      if (p->max_seqlen > 0 && cu[i + 1] - cu[i] > p->max_seqlen)
        return fail(FMHA_ERR_INVALID_ARG, "sequence %d has %d tokens, more than max_seqlen=%d", i, cu[i + 1] - cu[i], p->max_seqlen);
    }
    if (cu[p->batch] != p->total_tokens)
      return fail(FMHA_ERR_INVALID_ARG, "cu_seqlens_host[batch]=%d differs from total_tokens=%d", cu[p->batch], p->total_tokens);
  }
  const size_t need = fmha_varlen_workspace_size(p->batch, p->total_tokens, p->heads, bwd);
  if (!p->workspace) return fail(FMHA_ERR_WORKSPACE, "workspace is null (%zu bytes needed)", need);
  if (misaligned(p->workspace, kAlign)) return fail(FMHA_ERR_WORKSPACE, "workspace must be 256-byte aligned");
  if (p->workspace_bytes < need) return fail(FMHA_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", p->workspace_bytes, need);
  return FMHA_OK;
}

int check_ptr(const char* name, const void* ptr) {
  if (!ptr) return fail(FMHA_ERR_INVALID_ARG, "%s is null", name);
  if (misaligned(ptr, 16)) return fail(FMHA_ERR_INVALID_ARG, "%s is not 16-byte aligned", name);
  return FMHA_OK;
}

// Compute units of the current device (host query, cached per device).
int compute_units() {
  thread_local int cached_dev = -1, cached_cus = 0;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 256;
  if (dev != cached_dev) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    cached_dev = dev;
    cached_cus = n;
  }
  return cached_cus;
}

// Workgroups launched: persistent, `per_cu` per compute unit, but never more than
// the (tile, head) items that can exist.  max_seqlen, when given, tightens that
// bound; the kernels stride over the list, so a wrong bound costs time, never
// correctness.
unsigned grid_for(const fmha_varlen_params_t* p, int per_cu) {
  int64_t tiles = tile_capacity(p->batch, p->total_tokens);
  if (p->max_seqlen > 0) {
    const int64_t per_seq = (p->max_seqlen + fmha::kTileRows - 1) / fmha::kTileRows;
    if (per_seq * p->batch < tiles) tiles = per_seq * p->batch;
  }
  int64_t g = tiles * p->heads;
  const int64_t resident = (int64_t)compute_units() * per_cu;
  if (g > resident) g = resident;
  if (g < 1) g = 1;
  return (unsigned)g;
}

int launch_schedule(const fmha_varlen_params_t* p, const Workspace& w, hipStream_t st) {
  if (p->flags & FMHA_FLAG_REUSE_SCHEDULE) return FMHA_OK;
  const int cap = (int)tile_capacity(p->batch, p->total_tokens);
  fmha::schedule_kernel<<<1, fmha::kSchedThreads, 0, st>>>(p->cu_seqlens, p->seqused, p->batch, p->total_tokens, w.count,
                                                          w.list, cap, w.feed);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(FMHA_ERR_HIP, "schedule launch failed: %s", hipGetErrorString(e));
  return FMHA_OK;
}

fmha::Problem problem_of(const fmha_varlen_params_t* p, const Workspace& w) {
  fmha::Problem pb;
  pb.n_tiles = w.count;
  pb.tiles = w.list;
  pb.heads = p->heads;
  pb.total_tokens = p->total_tokens;
  pb.scale = p->scale;
  return pb;
}

// Upper bound on the number of (tile, head) items, from host-visible sizes only.
int64_t items_bound(const fmha_varlen_params_t* p) {
  int64_t tiles = tile_capacity(p->batch, p->total_tokens);
  if (p->max_seqlen > 0) {
    const int64_t per_seq = (p->max_seqlen + fmha::kTileRows - 1) / fmha::kTileRows;
    if (per_seq * p->batch < tiles) tiles = per_seq * p->batch;
  }
  return tiles * p->heads;
}

// Persistent grid of `per_cu` workgroups per compute unit (a multiple of 8, never more than
// there can be items), and the item feed's chunk size for it: about 24 chunks per workgroup
// on large batches, single items on small ones.
unsigned feed_grid(const fmha_varlen_params_t* p, int per_cu, const Workspace& w, fmha::FeedArgs* feed) {
  const int64_t items = items_bound(p);
  int64_t g = (int64_t)compute_units() * per_cu;
  if (g > items) g = items;
  g = (g + 7) / 8 * 8;
  if (g < 8) g = 8;
  int64_t chunk = items / (g * 24);
  if (chunk < 1) chunk = 1;
  if (chunk > 256) chunk = 256;
  feed->counters = w.feed;
  feed->chunk = (int32_t)chunk;
  return (unsigned)g;
}

// Dropout arguments for the kernels; d == nullptr means no dropout.
int drop_args(const fmha_dropout_t* d, bool required, fmha::DropArgs* out) {
  *out = fmha::DropArgs{0u, 0u, 0u, 1.f};
  if (!d) return required ? fail(FMHA_ERR_INVALID_ARG, "dropout is null") : FMHA_OK;
  if (!(d->p >= 0.f && d->p < 1.f)) return fail(FMHA_ERR_INVALID_ARG, "dropout p=%g is not in [0, 1)", (double)d->p);
  int t = (int)(256.f * d->p + 0.5f);  // p is exactly representable times 256: no double rounding
  if (t > 255) t = 255;
  out->thr = (uint32_t)t;
  out->k0 = (uint32_t)(d->seed & 0xffffffffu);
  out->k1 = (uint32_t)(d->seed >> 32);
  out->rp = 256.f / (float)(256 - t);
  return FMHA_OK;
}

// ---- the library's own scratch memory, for fmha_varlen_fwd_static -----------------
// `scratch` is a device array: in host code its name is only a handle for
// hipGetSymbolAddress, never an address to hand to a kernel.  Every GPU holds its own copy
// at its own address, looked up once per device (with that device current) and kept.
constexpr size_t kStaticScratchBytes = (size_t)1 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(FMHA_ERR_HIP, "hipGetDevice failed: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return fail(FMHA_ERR_HIP, "device index %d is outside [0, %d)", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr)
      return fail(FMHA_ERR_HIP, "hipGetSymbolAddress(scratch) failed on device %d: %s", dev, hipGetErrorString(e));
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return FMHA_OK;
}

int run_fwd(const fmha_varlen_params_t* p, const fmha_dropout_t* d, bool with_dropout, const void* q,
            const void* k, const void* v, void* o, float* lse, void* stream);
int run_bwd(const fmha_varlen_params_t* p, const fmha_dropout_t* d, bool with_dropout, const void* q,
            const void* k, const void* v, const void* o, const void* d_o, const float* lse, void* dq,
            void* dk, void* dv, void* stream);

}  // namespace

extern "C" {

const char* fmha_last_error(void) { return g_err; }

size_t fmha_varlen_workspace_size(int32_t batch, int32_t total_tokens, int32_t heads, int32_t need_bwd) {
  if (batch < 0 || total_tokens < 0 || heads <= 0) return 0;
  Workspace w = carve(nullptr, batch, total_tokens, heads);
  return need_bwd ? w.bytes_bwd : w.bytes_fwd;
}

int32_t fmha_varlen_schedule_info(int32_t batch, int32_t total_tokens, int32_t max_seqlen,
                                  size_t* count_offset, size_t* list_offset) {
  if (batch < 0 || total_tokens < 0) return -1;
  Workspace w = carve(nullptr, batch, total_tokens, 1);
  if (count_offset) *count_offset = w.count_off;
  if (list_offset) *list_offset = w.list_off;
  (void)max_seqlen;
  return (int32_t)tile_capacity(batch, total_tokens);
}

int fmha_varlen_fwd(const fmha_varlen_params_t* p, const void* q, const void* k, const void* v,
                    void* o, float* lse, void* stream) {
  return run_fwd(p, nullptr, false, q, k, v, o, lse, stream);
}

int fmha_varlen_fwd_dropout(const fmha_varlen_params_t* p, const fmha_dropout_t* dropout, const void* q,
                            const void* k, const void* v, void* o, float* lse, void* stream) {
  return run_fwd(p, dropout, true, q, k, v, o, lse, stream);
}

size_t fmha_varlen_static_scratch_bytes(void) { return kStaticScratchBytes; }

int fmha_varlen_fwd_static(const fmha_varlen_params_t* p, const void* q, const void* k, const void* v,
                           void* o, float* lse, void* stream) {
  if (!p) return fail(FMHA_ERR_INVALID_ARG, "params is null");
  if (p->batch < 0 || p->total_tokens < 0 || p->heads <= 0)
    return fail(FMHA_ERR_INVALID_ARG, "batch=%d, total_tokens=%d, heads=%d: invalid sizes", p->batch, p->total_tokens, p->heads);
  const size_t need = fmha_varlen_workspace_size(p->batch, p->total_tokens, p->heads, 0);
  if (need > kStaticScratchBytes)
    return fail(FMHA_ERR_WORKSPACE,
                "a batch of %d sequences and %d tokens needs %zu bytes for its tile list, the built-in scratch "
                "holds %zu: use fmha_varlen_fwd with a workspace",
                p->batch, p->total_tokens, need, kStaticScratchBytes);
  void* ptr = nullptr;
  int rc = static_scratch(&ptr);
  if (rc) return rc;
  fmha_varlen_params_t local = *p;
  local.workspace = ptr;
  local.workspace_bytes = kStaticScratchBytes;
  return run_fwd(&local, nullptr, false, q, k, v, o, lse, stream);
}

int fmha_varlen_bwd(const fmha_varlen_params_t* p, const void* q, const void* k, const void* v,
                    const void* o, const void* d_o, const float* lse, void* dq, void* dk,
                    void* dv, void* stream) {
  return run_bwd(p, nullptr, false, q, k, v, o, d_o, lse, dq, dk, dv, stream);
}

int fmha_varlen_bwd_dropout(const fmha_varlen_params_t* p, const fmha_dropout_t* dropout, const void* q,
                            const void* k, const void* v, const void* o, const void* d_o,
                            const float* lse, void* dq, void* dk, void* dv, void* stream) {
  return run_bwd(p, dropout, true, q, k, v, o, d_o, lse, dq, dk, dv, stream);
}

int fmha_dropout_keep_mask(const fmha_varlen_params_t* p, const fmha_dropout_t* dropout, int32_t orientation,
                           int32_t row_bytes, uint8_t* mask, void* stream) {
  int rc = check_common(p, false);
  if (rc) return rc;
  fmha::DropArgs da;
  if ((rc = drop_args(dropout, true, &da))) return rc;
  if (!mask) return fail(FMHA_ERR_INVALID_ARG, "mask is null");
  if (orientation != 0 && orientation != 1) return fail(FMHA_ERR_INVALID_ARG, "orientation=%d is neither 0 nor 1", orientation);
  if (row_bytes <= 0) return fail(FMHA_ERR_INVALID_ARG, "row_bytes=%d must be positive", row_bytes);
  if (p->max_seqlen > row_bytes) return fail(FMHA_ERR_INVALID_ARG, "row_bytes=%d is smaller than max_seqlen=%d", row_bytes, p->max_seqlen);
  g_err[0] = 0;
  if (p->batch == 0 || p->total_tokens == 0) return FMHA_OK;
  hipStream_t st = static_cast<hipStream_t>(stream);
  Workspace w = carve(p->workspace, p->batch, p->total_tokens, p->heads);
  if ((rc = launch_schedule(p, w, st))) return rc;
  const fmha::Problem pb = problem_of(p, w);
  const unsigned grid = grid_for(p, 4);
  if (orientation == 0)
    fmha::keep_mask_kernel<false><<<grid, fmha::kThreads, 0, st>>>(pb, da, mask, row_bytes);
  else
    fmha::keep_mask_kernel<true><<<grid, fmha::kThreads, 0, st>>>(pb, da, mask, row_bytes);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(FMHA_ERR_HIP, "keep-mask launch failed: %s", hipGetErrorString(e));
  return FMHA_OK;
}

}  // extern "C"

namespace {

int run_fwd(const fmha_varlen_params_t* p, const fmha_dropout_t* d, bool with_dropout, const void* q,
            const void* k, const void* v, void* o, float* lse, void* stream) {
  int rc = check_common(p, false);
  if (rc) return rc;
  fmha::DropArgs da;
  if ((rc = drop_args(d, with_dropout, &da))) return rc;
  if ((rc = check_ptr("q", q)) || (rc = check_ptr("k", k)) || (rc = check_ptr("v", v)) ||
      (rc = check_ptr("o", o)) || (rc = check_ptr("lse", lse)))
    return rc;
  const int64_t dense = (int64_t)p->heads * fmha::kHeadDim;
  fmha::FwdArgs a;
  if ((rc = check_stride("q", p->q_stride, dense, &a.q_stride)) ||
      (rc = check_stride("k", p->k_stride, dense, &a.k_stride)) ||
      (rc = check_stride("v", p->v_stride, dense, &a.v_stride)) ||
      (rc = check_stride("o", p->o_stride, dense, &a.o_stride)))
    return rc;
  g_err[0] = 0;
  if (p->batch == 0 || p->total_tokens == 0) return FMHA_OK;
  hipStream_t st = static_cast<hipStream_t>(stream);
  Workspace w = carve(p->workspace, p->batch, p->total_tokens, p->heads);
  if ((rc = launch_schedule(p, w, st))) return rc;
  a.pb = problem_of(p, w);
  a.feed = fmha::FeedArgs{w.feed, 1};
  a.q = static_cast<const uint16_t*>(q);
  a.k = static_cast<const uint16_t*>(k);
  a.v = static_cast<const uint16_t*>(v);
  a.o = static_cast<uint16_t*>(o);
  a.lse = lse;
  const unsigned grid = grid_for(p, 3);
  a.drop = da;
  // p = 0 (threshold 0) keeps everything: the plain kernels serve it
  if (da.thr == 0) {
    // persistent: 4 workgroups of 2 wavefronts per compute unit
    const unsigned grid64 = feed_grid(p, 4, w, &a.feed);
    if (p->dtype == FMHA_F16)
      fmha::fmha_fwd64_kernel<_Float16><<<grid64, fmha::kF64Threads, 0, st>>>(a);
    else
      fmha::fmha_fwd64_kernel<__bf16><<<grid64, fmha::kF64Threads, 0, st>>>(a);
  } else {
    if (p->dtype == FMHA_F16)
      fmha::fmha_fwd_kernel<_Float16, true><<<grid, fmha::kThreads, 0, st>>>(a);
    else
      fmha::fmha_fwd_kernel<__bf16, true><<<grid, fmha::kThreads, 0, st>>>(a);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(FMHA_ERR_HIP, "forward launch failed: %s", hipGetErrorString(e));
  return FMHA_OK;
}

int run_bwd(const fmha_varlen_params_t* p, const fmha_dropout_t* d, bool with_dropout, const void* q,
            const void* k, const void* v, const void* o, const void* d_o, const float* lse, void* dq,
            void* dk, void* dv, void* stream) {
  int rc = check_common(p, true);
  if (rc) return rc;
  fmha::DropArgs da;
  if ((rc = drop_args(d, with_dropout, &da))) return rc;
  if ((p->flags & FMHA_FLAG_BWD_ONLY_DQ) && (p->flags & FMHA_FLAG_BWD_ONLY_DKV))
    return fail(FMHA_ERR_INVALID_ARG, "FMHA_FLAG_BWD_ONLY_DQ and FMHA_FLAG_BWD_ONLY_DKV exclude each other");
  if ((rc = check_ptr("q", q)) || (rc = check_ptr("k", k)) || (rc = check_ptr("v", v)) ||
      (rc = check_ptr("o", o)) || (rc = check_ptr("d_o", d_o)) || (rc = check_ptr("lse", lse)) ||
      (rc = check_ptr("dq", dq)) || (rc = check_ptr("dk", dk)) || (rc = check_ptr("dv", dv)))
    return rc;
  const int64_t dense = (int64_t)p->heads * fmha::kHeadDim;
  fmha::BwdArgs a;
  if ((rc = check_stride("q", p->q_stride, dense, &a.q_stride)) ||
      (rc = check_stride("k", p->k_stride, dense, &a.k_stride)) ||
      (rc = check_stride("v", p->v_stride, dense, &a.v_stride)) ||
      (rc = check_stride("o", p->o_stride, dense, &a.o_stride)) ||
      (rc = check_stride("do", p->do_stride, dense, &a.do_stride)) ||
      (rc = check_stride("dq", p->dq_stride, dense, &a.dq_stride)) ||
      (rc = check_stride("dk", p->dk_stride, dense, &a.dk_stride)) ||
      (rc = check_stride("dv", p->dv_stride, dense, &a.dv_stride)))
    return rc;
  g_err[0] = 0;
  if (p->batch == 0 || p->total_tokens == 0) return FMHA_OK;
  hipStream_t st = static_cast<hipStream_t>(stream);
  Workspace w = carve(p->workspace, p->batch, p->total_tokens, p->heads);
  if ((rc = launch_schedule(p, w, st))) return rc;
  a.pb = problem_of(p, w);
  a.feed = fmha::FeedArgs{w.feed, 1};
  a.drop = da;
  a.q = static_cast<const uint16_t*>(q);
  a.k = static_cast<const uint16_t*>(k);
  a.v = static_cast<const uint16_t*>(v);
  a.o = static_cast<const uint16_t*>(o);
  a.d_o = static_cast<const uint16_t*>(d_o);
  a.lse = lse;
  a.dsum = w.dsum;
  a.lse2 = w.lse2;
  a.dq = static_cast<uint16_t*>(dq);
  a.dk = static_cast<uint16_t*>(dk);
  a.dv = static_cast<uint16_t*>(dv);
  // persistent grids with their own hand-out chunk sizes: 3 workgroups per compute unit for
  // the dQ pass (2 with dropout), 2 for the dK/dV pass
  fmha::BwdArgs a_dq = a, a_dkv = a;
  const unsigned grid_dq = feed_grid(p, da.thr == 0 ? 3 : 2, w, &a_dq.feed);
  const unsigned grid_dkv = feed_grid(p, 2, w, &a_dkv.feed);
  const bool run_dq = !(p->flags & FMHA_FLAG_BWD_ONLY_DKV);
  const bool run_dkv = !(p->flags & FMHA_FLAG_BWD_ONLY_DQ);
  if (da.thr == 0) {
    if (p->dtype == FMHA_F16) {
      if (run_dq) fmha::bwd_dq_kernel<_Float16, false><<<grid_dq, fmha::kThreads, 0, st>>>(a_dq);
      if (run_dkv) fmha::bwd_dkv_kernel<_Float16, false><<<grid_dkv, fmha::kThreads, 0, st>>>(a_dkv);
    } else {
      if (run_dq) fmha::bwd_dq_kernel<__bf16, false><<<grid_dq, fmha::kThreads, 0, st>>>(a_dq);
      if (run_dkv) fmha::bwd_dkv_kernel<__bf16, false><<<grid_dkv, fmha::kThreads, 0, st>>>(a_dkv);
    }
  } else {
    if (p->dtype == FMHA_F16) {
      if (run_dq) fmha::bwd_dq_kernel<_Float16, true><<<grid_dq, fmha::kThreads, 0, st>>>(a_dq);
      if (run_dkv) fmha::bwd_dkv_kernel<_Float16, true><<<grid_dkv, fmha::kThreads, 0, st>>>(a_dkv);
    } else {
      if (run_dq) fmha::bwd_dq_kernel<__bf16, true><<<grid_dq, fmha::kThreads, 0, st>>>(a_dq);
      if (run_dkv) fmha::bwd_dkv_kernel<__bf16, true><<<grid_dkv, fmha::kThreads, 0, st>>>(a_dkv);
    }
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(FMHA_ERR_HIP, "backward launch failed: %s", hipGetErrorString(e));
  return FMHA_OK;
}

}  // namespace
