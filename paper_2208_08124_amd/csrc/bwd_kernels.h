// Backward of Eq. 1 by recomputation, in two passes that need no atomics and
// give run-to-run identical results:
//
//   pass 1 (bwd_dq_kernel)  - per tile of 128 query rows: D = rowsum(dO o O),
//       then for every block of keys  S^T = K Q^T,  dP^T = V dO^T,
//       P^T = exp(S^T - LSE),  dS^T = P^T o (dP^T - D),  dQ^T += K^T dS^T.
//   pass 2 (bwd_dkv_kernel) - per tile of 128 key rows, for every block of
//       queries  S = Q K^T,  dP = dO V^T,  P, dS as above,
//       dV^T += dO^T P,  dK^T += Q^T dS.
//
// With dropout (DROP) the mask M is regenerated from the seed (dropout.h):
// dP = (dO V^T) o M / (1-p) in both passes and dV^T += dO^T (P o M) with the
// factor 1/(1-p) applied to the finished rows; D = rowsum(dO o O) as before.
//
// Both orientations are chosen so that the MFMA result tile of the first two
// products has, in every lane, the reduction index of the following product
// spread over its registers; P and dS then go back in as B operands without
// passing through LDS, and the per-row statistics (LSE, D) are per-lane
// scalars in pass 1 and broadcast LDS reads in pass 2.
//
// The streamed operand (K and V in pass 1; Q, dO and the row statistics in
// pass 2) moves from HBM straight into a ring of swizzled LDS stages, two
// blocks ahead of its use, one barrier per block.
#pragma once
#include "dropout.h"
#include "kernel_args.h"
#include "mfma_tiles.h"

namespace fmha {

constexpr int kBwdStages = 3;

// registers 8*t2 .. 8*t2+7 of a result tile as one B operand
template <typename T>
static __device__ __forceinline__ u32x4 pack8(const float (&x)[16], int t2) {
  return u32x4{Op<T>::pack2(x[8 * t2 + 0], x[8 * t2 + 1]), Op<T>::pack2(x[8 * t2 + 2], x[8 * t2 + 3]),
               Op<T>::pack2(x[8 * t2 + 4], x[8 * t2 + 5]), Op<T>::pack2(x[8 * t2 + 6], x[8 * t2 + 7])};
}

// ---------------------------------------------------------------- pass 1: dQ
// One block of 64 keys for one wavefront (32 queries), done as two halves of 32 keys
// so that only one half's scores and operands are live at a time.
template <typename T, bool RAGGED, bool DROP>
__device__ __forceinline__ void dq_block(f32x16 (&dq)[2], const uint16_t* sK, const uint16_t* sV,
                                         const u32x4 (&qb)[4], const u32x4 (&gb)[4], float c2,
                                         float lse2, float dsum, int key_base, int nk, int g,
                                         const RowRead& rr, const ColRead& cr, int q4, int ln, int r0,
                                         int head, const DropArgs& drop) {
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int kb = 0; kb < 2; kb++) {
    if (RAGGED && key_base + 32 * kb >= nk) break;
    __builtin_amdgcn_sched_barrier(0);
    u32x4 ka[4], va[4];
#pragma unroll
    for (int t = 0; t < 4; t++) {
      ka[t] = rr.read(sK, kb, t);
      va[t] = rr.read(sV, kb, t);
    }
    __builtin_amdgcn_sched_barrier(0);
    f32x16 s, dp;
#pragma unroll
    for (int t = 0; t < 4; t++) {
      s = Op<T>::mfma(ka[t], qb[t], t == 0 ? zero : s);
      dp = Op<T>::mfma(va[t], gb[t], t == 0 ? zero : dp);
    }
    uint32_t kb8[4];  // mask bytes: independent of the products just issued
    if (DROP) keep_bytes<false>(kb8, q4, ((key_base + 32 * kb) >> 2) + g, ln, r0, head, drop);
    __builtin_amdgcn_sched_barrier(0);
    u32x4 kT[2][2];
#pragma unroll
    for (int t2 = 0; t2 < 2; t2++)
#pragma unroll
      for (int cb = 0; cb < 2; cb++) kT[t2][cb] = cr.read(sK, 2 * kb + t2, cb);
    __builtin_amdgcn_sched_barrier(0);
    const int key0 = key_base + 32 * kb + 4 * g;
    float ds[16];
#pragma unroll
    for (int r = 0; r < 16; r++) {
      float p = fast_exp2(__builtin_fmaf(s[r], c2, -lse2));
      if (RAGGED && key0 + 8 * (r >> 2) + (r & 3) >= nk) p = 0.f;
      const float dpr = DROP ? (kept(kb8, r, drop.thr) ? dp[r] * drop.rp : 0.f) : dp[r];
      ds[r] = p * (dpr - dsum);
    }
    u32x4 dsb[2];
#pragma unroll
    for (int t2 = 0; t2 < 2; t2++) dsb[t2] = pack8<T>(ds, t2);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int t2 = 0; t2 < 2; t2++)
#pragma unroll
      for (int cb = 0; cb < 2; cb++) dq[cb] = Op<T>::mfma(kT[t2][cb], dsb[t2], dq[cb]);
  }
}

template <typename T, bool DROP>
__global__ __launch_bounds__(kThreads, DROP ? 2 : 3) void bwd_dq_kernel(const BwdArgs a) {
  constexpr int kPerCu = DROP ? 2 : 3;  // workgroups per compute unit (the launcher's grid assumes it)
  __shared__ __align__(1024) uint16_t ring[kBwdStages][2][kTileElems];  // [stage][K|V]

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int g = lane >> 5, ln = lane & 31;
  const int heads = a.pb.heads;
  const int n_items = tile_count(a.pb) * heads;
  const float c2 = a.pb.scale * kLog2e;
  const int slot = blockIdx.x / max(gridDim.x / (unsigned)kPerCu, 1u);  // which of the workgroups of its compute unit
  const DmaLane dl(wave, lane);
  const RowRead rr(ln, g);
  const ColRead cr(lane);
  const uint32_t ring_addr = lds_addr(&ring[0][0][0]);
  constexpr uint32_t kTileBytes = kTileElems * 2;
  // this lane's piece within a 64-row block (rows dl.row and dl.row + 32), in elements
  const uint32_t k_lane = (dl.row * (uint32_t)a.k_stride + dl.chunk * 8) * 2u;  // bytes
  const uint32_t v_lane = (dl.row * (uint32_t)a.v_stride + dl.chunk * 8) * 2u;

  // one entry behind each statistics array stands for "row past the end" in pass 2:
  // LSE = +inf makes its probabilities vanish
  if (blockIdx.x == 0 && tid == 0) {
    a.lse2[(int64_t)heads * a.pb.total_tokens] = INFINITY;
    a.dsum[(int64_t)heads * a.pb.total_tokens] = 0.f;
  }

  // Persistent workgroups that draw their items from the feed (item_feed.h); the record of
  // the next item is fetched while the current one is computed.
  __shared__ uint32_t mailbox;
  ItemFeed feed;
  int item = feed.init(a.feed, blockIdx.x, gridDim.x);
  int item1 = feed.next();
  TileItem ti_next = load_tile(a.pb, (item < n_items ? item : 0) / heads);
  while (item < n_items) {
    const int head = item % heads;
    const TileItem ti = ti_next;
    ti_next = load_tile(a.pb, (item1 < n_items ? item1 : item) / heads);
    const int r0 = ti.r0, len = ti.len, nk = ti.nk;
    const int qrow = ti.row0 + 32 * wave + ln;
    const bool wave_on = ti.row0 + 32 * wave < len;
    const bool row_on = qrow < len;
    const uint16_t* kbase = a.k + (int64_t)r0 * a.k_stride + head * kHeadDim;
    const uint16_t* vbase = a.v + (int64_t)r0 * a.v_stride + head * kHeadDim;
    const int n = (nk + kBlockKeys - 1) / kBlockKeys;

    // (the empty asm keeps the lane offsets from being combined with anything ahead of the
    // item loop and held in registers through it)
    uint32_t kl = k_lane, vl = v_lane;
    asm volatile("" : "+v"(kl), "+v"(vl));
    auto start_block = [&](int kt, int stage) {  // 4 pieces per thread
      const uint32_t st_addr = ring_addr + stage * (2 * kTileBytes);
      if ((kt + 1) * kBlockKeys <= nk) {
        dma_tile_full(kbase + (int64_t)kt * kBlockKeys * a.k_stride, kl, a.k_stride, wave, st_addr);
        dma_tile_full(vbase + (int64_t)kt * kBlockKeys * a.v_stride, vl, a.v_stride, wave, st_addr + kTileBytes);
      } else {
        dma_tile(kbase, a.k_stride, kt * kBlockKeys, nk - 1, dl, wave, st_addr);
        dma_tile(vbase, a.v_stride, kt * kBlockKeys, nk - 1, dl, wave, st_addr + kTileBytes);
      }
    };
    // Everything the tile needs first is requested in one batch, so that one memory
    // round trip covers it: the wavefront's 32 query rows (into its private rows of
    // the last ring stage, see own_piece), the first two key blocks, then dO, O and
    // LSE of this lane's query as ordinary loads.
    {
      const uint32_t own_addr = ring_addr + (kBwdStages - 1) * (2 * kTileBytes) + 1024u * wave;
      // rows relative to the wavefront's first row, clamped into the sequence
      const int w0 = min(ti.row0 + 32 * wave, len - 1);
      const uint16_t* qrows = a.q + uniform_i64((int64_t)(r0 + w0) * a.q_stride + head * kHeadDim);
      const int le = lane_id();
      const int room = len - 1 - w0;
#pragma unroll
      for (int i = 0; i < 4; i++) {
        const int r = 8 * i + (le >> 3);  // row within the wavefront's 32
        const uint32_t off = ((uint32_t)min(r, room) * (uint32_t)a.q_stride + ((le & 7) ^ swz(r)) * 8) * 2u;
        dma16s(qrows, off, __builtin_amdgcn_readfirstlane(own_addr + own_piece(i)));
      }
    }
    if (n > 0) start_block(0, 0);
    if (n > 1) start_block(1, 1);

    // dO^T as B operand (column = query ln, slots = channels 16t+8g..+7), and
    // D = sum_c dO*O over this lane's 32 channels, completed with the other half.
    u32x4 qb[4], gb[4];
    float dsum = 0.f, lse2 = 0.f;
    {
      const int qr = row_on ? qrow : len - 1;
      const int64_t tok = r0 + qr;
      const uint16_t* gp = a.d_o + tok * a.do_stride + head * kHeadDim + 8 * g;
      const uint16_t* op = a.o + tok * a.o_stride + head * kHeadDim + 8 * g;
#pragma unroll
      for (int t = 0; t < 4; t++) {
        gb[t] = *reinterpret_cast<const u32x4*>(gp + 16 * t);
        const u32x4 ov = *reinterpret_cast<const u32x4*>(op + 16 * t);
#pragma unroll
        for (int e = 0; e < 4; e++) dsum = Op<T>::dot2(gb[t][e], ov[e], dsum);
      }
      dsum += other_half(dsum);
      const int64_t si = (int64_t)head * a.pb.total_tokens + tok;
      lse2 = a.lse[si] * kLog2e;
    }
    // Q^T as B operand, from the private rows.  The query rows were requested before
    // the loads just consumed, so they have landed (vector memory loads complete in
    // issue order); the explicit wait keeps the LDS reads below it.
    wait_vmem<0>();
    {
      const uint16_t* sq = &ring[kBwdStages - 1][0][0] + 512 * wave + own_piece(ln >> 3) / 2 + (ln & 7) * 64;
      const int sw = swz(ln);
#pragma unroll
      for (int t = 0; t < 4; t++) qb[t] = *reinterpret_cast<const u32x4*>(sq + (((2 * t + g) ^ sw) << 3));
    }

    f32x16 dq[2];  // dQ^T: column = query ln, rows = channels
#pragma unroll
    for (int cb = 0; cb < 2; cb++)
#pragma unroll
      for (int r = 0; r < 16; r++) dq[cb][r] = 0.f;

    int stage = 0;
    for (int kt = 0; kt < n; kt++) {
      // block kt has landed once at most block kt+1's 4 pieces are outstanding
      if (kt + 1 < n)
        wait_vmem<4>();
      else
        wait_vmem<0>();
      __syncthreads();  // everyone's pieces; and everyone is done with block kt-1's stage
      rotate_priority(kt, slot, kPerCu);
      const int ahead = stage == 0 ? kBwdStages - 1 : stage - 1;  // (kt + 2) % 3
      if (kt + 2 < n) start_block(kt + 2, ahead);
      if (wave_on) {
        const uint16_t* sK = &ring[0][0][0] + stage * (2 * kTileElems);
        const uint16_t* sV = sK + kTileElems;
        const int q4 = qrow >> 2;
        if ((kt + 1) * kBlockKeys > nk)
          dq_block<T, true, DROP>(dq, sK, sV, qb, gb, c2, lse2, dsum, kt * kBlockKeys, nk, g, rr, cr, q4, ln, r0, head, a.drop);
        else
          dq_block<T, false, DROP>(dq, sK, sV, qb, gb, c2, lse2, dsum, kt * kBlockKeys, nk, g, rr, cr, q4, ln, r0, head, a.drop);
      }
      stage = stage == kBwdStages - 1 ? 0 : stage + 1;
    }
    feed.publish(&mailbox);
    __syncthreads();  // the ring is free for the next item
    feed.receive(&mailbox);
    const int item2 = feed.next();
    feed.request(a.feed);

    // The row statistics for pass 2 are stored here rather than where they are
    // computed: a store issued ahead of the key loop would have to be acknowledged
    // before the loop's first wait on the fetch counter lets go.
    {
      const int le = lane_id();
      const int row = ti.row0 + 32 * wave + (le & 31);
      if (row < len && le < 32) {
        const int64_t si = (int64_t)head * a.pb.total_tokens + r0 + row;
        a.dsum[si] = dsum;
        a.lse2[si] = lse2;
      }
    }
    // dQ leaves as whole rows, turned around in the wavefront's private rows of
    // the last ring stage (see store_rows).
    if (wave_on)
      store_rows<T>(dq, a.pb.scale, &ring[kBwdStages - 1][0][0], wave, a.dq,
                    (int64_t)(r0 + ti.row0 + 32 * wave) * a.dq_stride + head * kHeadDim, a.dq_stride,
                    len - (ti.row0 + 32 * wave));
    item = item1;
    item1 = item2;
  }
  feed.finish(a.feed, gridDim.x);
}

// ------------------------------------------------------------ pass 2: dK, dV
struct DkvStage {
  uint16_t q[kTileElems];   // 64 queries x 64 channels, swizzled
  uint16_t g[kTileElems];   // dO, same
  float stat[4][64];        // [0] = LSE*log2(e), [1] = D of the 64 queries; [2], [3] unused
};

// One block of 32 queries (rows 32*qb.. of the stage) for one wavefront (32 keys).
// No masking is needed here: query rows past the end of the sequence carry
// LSE = +inf in the stage (so P = 0), and the columns of keys that are masked
// or past the end are independent of all others and are simply not stored.
template <typename T, bool DROP>
__device__ __forceinline__ void dkv_block(f32x16 (&dk)[2], f32x16 (&dv)[2], const DkvStage* st,
                                          int qb, const u32x4 (&kb4)[4], const u32x4 (&vb4)[4],
                                          float c2, int g, const RowRead& rr, const ColRead& cr,
                                          int k4, int q_base, int ln, int r0, int head,
                                          const DropArgs& drop) {
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  u32x4 qa[4], ga[4];
#pragma unroll
  for (int t = 0; t < 4; t++) {
    qa[t] = rr.read(st->q, qb, t);
    ga[t] = rr.read(st->g, qb, t);
  }
  __builtin_amdgcn_sched_barrier(0);
  // S = Q K^T, dP = dO V^T : rows = queries (32), column = key ln
  f32x16 s, dp;
#pragma unroll
  for (int t = 0; t < 4; t++) {
    s = Op<T>::mfma(qa[t], kb4[t], t == 0 ? zero : s);
    dp = Op<T>::mfma(ga[t], vb4[t], t == 0 ? zero : dp);
  }
  uint32_t kb8[4];  // mask bytes: independent of the products just issued
  if (DROP) keep_bytes<true>(kb8, k4, ((q_base + 32 * qb) >> 2) + g, ln, r0, head, drop);
  __builtin_amdgcn_sched_barrier(0);
  // rows 32qb + 8j + 4g + {0..3}: their statistics sit side by side
  float4 l4[4], d4[4];
#pragma unroll
  for (int j = 0; j < 4; j++) {
    l4[j] = *reinterpret_cast<const float4*>(&st->stat[0][32 * qb + 8 * j + 4 * g]);
    d4[j] = *reinterpret_cast<const float4*>(&st->stat[1][32 * qb + 8 * j + 4 * g]);
  }
  u32x4 gT[2][2];  // dO^T operands: [16-query step][channel block]
#pragma unroll
  for (int t2 = 0; t2 < 2; t2++)
#pragma unroll
    for (int cb = 0; cb < 2; cb++) gT[t2][cb] = cr.read(st->g, 2 * qb + t2, cb);
  __builtin_amdgcn_sched_barrier(0);
  float p[16], ds[16];
#pragma unroll
  for (int j = 0; j < 4; j++) {
    const float lv[4] = {l4[j].x, l4[j].y, l4[j].z, l4[j].w};
    const float dvv[4] = {d4[j].x, d4[j].y, d4[j].z, d4[j].w};
#pragma unroll
    for (int e = 0; e < 4; e++) {
      const float pe = fast_exp2(__builtin_fmaf(s[4 * j + e], c2, -lv[e]));
      if (DROP) {
        const bool on = kept(kb8, 4 * j + e, drop.thr);
        p[4 * j + e] = on ? pe : 0.f;
        ds[4 * j + e] = pe * ((on ? dp[4 * j + e] * drop.rp : 0.f) - dvv[e]);
      } else {
        p[4 * j + e] = pe;
        ds[4 * j + e] = pe * (dp[4 * j + e] - dvv[e]);
      }
    }
  }
  u32x4 pb[2], dsb[2];
#pragma unroll
  for (int t2 = 0; t2 < 2; t2++) {
    pb[t2] = pack8<T>(p, t2);
    dsb[t2] = pack8<T>(ds, t2);
  }
  __builtin_amdgcn_sched_barrier(0);
  // Q^T operands are requested now and arrive under the dV MFMAs
  u32x4 qT[2][2];
#pragma unroll
  for (int t2 = 0; t2 < 2; t2++)
#pragma unroll
    for (int cb = 0; cb < 2; cb++) qT[t2][cb] = cr.read(st->q, 2 * qb + t2, cb);
  // dV^T += dO^T P, dK^T += Q^T dS : rows = channels, contraction over queries
#pragma unroll
  for (int t2 = 0; t2 < 2; t2++)
#pragma unroll
    for (int cb = 0; cb < 2; cb++) dv[cb] = Op<T>::mfma(gT[t2][cb], pb[t2], dv[cb]);
#pragma unroll
  for (int t2 = 0; t2 < 2; t2++)
#pragma unroll
    for (int cb = 0; cb < 2; cb++) dk[cb] = Op<T>::mfma(qT[t2][cb], dsb[t2], dk[cb]);
}

template <typename T, bool DROP>
__global__ __launch_bounds__(kThreads, 2) void bwd_dkv_kernel(const BwdArgs a) {
  __shared__ __align__(1024) DkvStage ring[kBwdStages];

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int g = lane >> 5, ln = lane & 31;
  const int heads = a.pb.heads;
  const int n_items = tile_count(a.pb) * heads;
  const float c2 = a.pb.scale * kLog2e;
  const int slot = blockIdx.x / max(gridDim.x / 2u, 1u);  // which of the 2 workgroups per compute unit
  const DmaLane dl(wave, lane);
  const RowRead rr(ln, g);
  const ColRead cr(lane);
  const uint32_t ring_addr = lds_addr(&ring[0]);
  constexpr uint32_t kStageBytes = sizeof(DkvStage), kTileBytes = kTileElems * 2;
  // this lane's piece within a 64-row block (rows dl.row and dl.row + 32), in elements
  const uint32_t q_lane = (dl.row * (uint32_t)a.q_stride + dl.chunk * 8) * 2u;  // bytes
  const uint32_t g_lane = (dl.row * (uint32_t)a.do_stride + dl.chunk * 8) * 2u;

  // Persistent workgroups that draw their items from the feed (item_feed.h); the record of
  // the next item is fetched while the current one is computed.
  __shared__ uint32_t mailbox;
  ItemFeed feed;
  int item = feed.init(a.feed, blockIdx.x, gridDim.x);
  int item1 = feed.next();
  TileItem ti_next = load_tile(a.pb, (item < n_items ? item : 0) / heads);
  while (item < n_items) {
    const int head = item % heads;
    const TileItem ti = ti_next;
    ti_next = load_tile(a.pb, (item1 < n_items ? item1 : item) / heads);
    const int r0 = ti.r0, len = ti.len, nk = ti.nk;
    const int krow = ti.row0 + 32 * wave + ln;      // this lane's key, within the sequence
    const bool wave_on = ti.row0 + 32 * wave < nk;  // wavefront owns at least one live key
    const bool tile_on = ti.row0 < nk;              // uniform over the workgroup
    const bool key_on = krow < nk;
    const uint16_t* qbase = a.q + (int64_t)r0 * a.q_stride + head * kHeadDim;
    const uint16_t* gbase = a.d_o + (int64_t)r0 * a.do_stride + head * kHeadDim;
    // statistics: wavefront 0 moves LSE*log2e, wavefront 1 moves D (2 and 3 repeat them
    // into the unused quarter of the stage so that every thread has the same piece count).
    // Rows past the end of the sequence read the +inf / 0 that pass 1 left behind the arrays.
    const float* stat_arr = (wave & 1) ? a.dsum : a.lse2;
    const float* stat_src = stat_arr + (int64_t)head * a.pb.total_tokens + r0;
    const float* stat_pad = stat_arr + (int64_t)heads * a.pb.total_tokens;
    const int n = tile_on ? (len + kBlockKeys - 1) / kBlockKeys : 0;  // query blocks

    // (the empty asm keeps the lane offsets from being combined with anything ahead of the
    // item loop and held in registers through it)
    uint32_t ql = q_lane, gl = g_lane;
    asm volatile("" : "+v"(ql), "+v"(gl));
    auto start_block = [&](int qt, int stage) {  // 5 pieces per thread
      const uint32_t st_addr = ring_addr + stage * kStageBytes;
      if ((qt + 1) * kBlockKeys <= len) {
        dma_tile_full(qbase + (int64_t)qt * kBlockKeys * a.q_stride, ql, a.q_stride, wave, st_addr);
        dma_tile_full(gbase + (int64_t)qt * kBlockKeys * a.do_stride, gl, a.do_stride, wave, st_addr + kTileBytes);
      } else {
        dma_tile(qbase, a.q_stride, qt * kBlockKeys, len - 1, dl, wave, st_addr);
        dma_tile(gbase, a.do_stride, qt * kBlockKeys, len - 1, dl, wave, st_addr + kTileBytes);
      }
      const uint32_t m0 = __builtin_amdgcn_readfirstlane(st_addr + 2 * kTileBytes + 256u * wave);
      const int srow = qt * kBlockKeys + lane;
      dma4(srow < len ? stat_src + srow : stat_pad, m0);
    };
    if (n > 0) start_block(0, 0);
    if (n > 1) start_block(1, 1);

    // K^T and V^T as B operands: column = key ln, slots = channels 16t+8g..+7
    u32x4 kb4[4], vb4[4];
    {
      const int kr = krow < len ? krow : len - 1;
      const uint16_t* kp = a.k + (int64_t)(r0 + kr) * a.k_stride + head * kHeadDim + 8 * g;
      const uint16_t* vp = a.v + (int64_t)(r0 + kr) * a.v_stride + head * kHeadDim + 8 * g;
#pragma unroll
      for (int t = 0; t < 4; t++) {
        kb4[t] = *reinterpret_cast<const u32x4*>(kp + 16 * t);
        vb4[t] = *reinterpret_cast<const u32x4*>(vp + 16 * t);
      }
      // Consume them here: the compiler then waits for these loads now, together
      // with the first blocks, instead of in front of their first use inside the
      // query loop - where the wait would also cover the block just requested and
      // so expose a full memory round trip in every iteration.
#pragma unroll
      for (int t = 0; t < 4; t++) asm volatile("" ::"v"(kb4[t]), "v"(vb4[t]));
    }

    f32x16 dk[2], dv[2];  // dK^T, dV^T: column = key ln, rows = channels
#pragma unroll
    for (int cb = 0; cb < 2; cb++)
#pragma unroll
      for (int r = 0; r < 16; r++) dk[cb][r] = dv[cb][r] = 0.f;

    int stage = 0;
    for (int qt = 0; qt < n; qt++) {
      if (qt + 1 < n)
        wait_vmem<5>();
      else
        wait_vmem<0>();
      __syncthreads();
      rotate_priority(qt, slot, 2);
      const int ahead = stage == 0 ? kBwdStages - 1 : stage - 1;
      if (qt + 2 < n) start_block(qt + 2, ahead);
      if (wave_on) {
        const DkvStage* st = &ring[stage];
        const int k4 = krow >> 2;
        dkv_block<T, DROP>(dk, dv, st, 0, kb4, vb4, c2, g, rr, cr, k4, qt * kBlockKeys, ln, r0, head, a.drop);
        if (qt * kBlockKeys + 32 < len)
          dkv_block<T, DROP>(dk, dv, st, 1, kb4, vb4, c2, g, rr, cr, k4, qt * kBlockKeys, ln, r0, head, a.drop);
      }
      stage = stage == kBwdStages - 1 ? 0 : stage + 1;
    }
    feed.publish(&mailbox);
    __syncthreads();
    feed.receive(&mailbox);
    const int item2 = feed.next();
    feed.request(a.feed);

    // every row of the tile is written: live keys get their gradients, keys
    // masked by seqused get zeros.  dK and dV leave as whole rows, turned around in
    // the wavefront's private rows of the last two ring stages (see store_rows).
    if (ti.row0 + 32 * wave < len) {
      if (!key_on) {
#pragma unroll
        for (int cb = 0; cb < 2; cb++)
#pragma unroll
          for (int r = 0; r < 16; r++) dv[cb][r] = dk[cb][r] = 0.f;
      }
      const int64_t tok = r0 + ti.row0 + 32 * wave;
      const int n_rows = len - (ti.row0 + 32 * wave);
      store_rows<T>(dk, a.pb.scale, ring[kBwdStages - 1].q, wave, a.dk, tok * a.dk_stride + head * kHeadDim,
                    a.dk_stride, n_rows);
      store_rows<T>(dv, DROP ? a.drop.rp : 1.f, ring[kBwdStages - 2].q, wave, a.dv, tok * a.dv_stride + head * kHeadDim,
                    a.dv_stride, n_rows);
    }
    item = item1;
    item1 = item2;
  }
  feed.finish(a.feed, gridDim.x);
}

}  // namespace fmha
