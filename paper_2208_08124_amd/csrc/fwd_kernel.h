// Forward kernel: O = softmax(scale Q K^T) V on packed rows (Eq. 1 of the
// paper, one sequence and head at a time), fused in one pass over the keys
// with a running row maximum and row sum.
//
// One workgroup (4 wavefronts) takes one tile of 128 query rows of one
// (sequence, head); wavefront w owns rows 32w..32w+31.  Keys and values move
// 64 rows at a time from HBM straight into a ring of four LDS stages, up to
// three blocks ahead of the one being soft-maxed, with one barrier per step.
//
// The scores are produced TRANSPOSED, S^T = K Q^T, so that in the MFMA result
// layout every lane holds 16 keys of ONE query: the row maximum and row sum
// are then per-lane reductions plus a single exchange with the lane 32 away,
// and the probabilities are already in the operand layout of the second
// product O^T = V^T P^T.
//
// The softmax competes with the matrix cores for issue slots (a v_exp_f32
// costs a quarter of the MFMA time a score needs), and two wavefronts sharing
// a SIMD fall into lock step rather than filling each other's gaps.  So each
// wavefront overlaps the two units itself: the MFMAs that compute the scores of
// block i+1 are woven through the exponentials of block i.  The vector work per
// score is one fused multiply-add, one exp2, half a max3, half a pack and half
// a dot2 (row sum).
//
// The running maximum is only raised when a block exceeds it by more than
// kRescaleStep (log2 units); until then probabilities may exceed 1 (by at most
// 2^kRescaleStep: harmless in fp16/bf16 and fp32) and the accumulators are not
// rescaled.  The result is the same softmax: the maximum cancels between
// numerator and row sum.
#pragma once
#include "kernel_args.h"
#include "mfma_tiles.h"

namespace fmha {

constexpr float kRescaleStep = 8.f;
constexpr int kRing = 4;  // LDS ring: one K and one V tile per stage (16 KB)

struct FwdAcc {
  f32x16 o[2];  // O^T: column = query ln; o[cb][r] is channel 32cb + 8(r/4) + 4g + r%4
  float m_run;  // running maximum, log2 domain (scaled by |scale|*log2 e)
  float l_run;  // this lane's share of the running row sum
};

// S^T = K Q^T for one block of 64 keys: rows = keys (two blocks of 32), column = query ln
template <typename T>
__device__ __forceinline__ void fwd_scores(f32x16 (&s)[2], const uint16_t* sK, const u32x4 (&qb)[4],
                                           const RowRead& rr) {
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  u32x4 ka[4][2];
#pragma unroll
  for (int t = 0; t < 4; t++)
#pragma unroll
    for (int kb = 0; kb < 2; kb++) ka[t][kb] = rr.read(sK, kb, t);
#pragma unroll
  for (int t = 0; t < 4; t++)
#pragma unroll
    for (int kb = 0; kb < 2; kb++) s[kb] = Op<T>::mfma(ka[t][kb], qb[t], t == 0 ? zero : s[kb]);
}

// One pipeline step of one wavefront over a block of 64 keys:
//   vector ALU  : soft-max block i, whose scores are in s_cur
//   matrix core : (HAS_NEXT) scores of block i+1 (keys in sK_next) -> s_next, the MFMAs
//                 woven through the exponentials; then O^T += V_i^T P_i^T (keys in sV).
// RAGGED: keys at or beyond nk (only in a sequence's last block) are excluded.
// Apart from the rare rescale branch after the maximum, the step is
// straight-line code.
template <typename T, bool RAGGED, bool HAS_NEXT>
__device__ __forceinline__ void fwd_step(FwdAcc& acc, const f32x16 (&s_cur)[2], f32x16 (&s_next)[2],
                                         const uint16_t* sK_next, const uint16_t* sV,
                                         const u32x4 (&qb)[4], float c2, int key_base, int nk, int g,
                                         const RowRead& rr, const ColRead& cr) {
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  // operands of the score product are requested first; they arrive under the maximum
  u32x4 ka[4][2];
  if (HAS_NEXT) {
#pragma unroll
    for (int t = 0; t < 4; t++)
#pragma unroll
      for (int kb = 0; kb < 2; kb++) ka[t][kb] = rr.read(sK_next, kb, t);
  }
  const int key0 = key_base + 4 * g;      // key of s_cur[0][0]
  float mxs[2] = {-INFINITY, -INFINITY};  // two independent chains
#pragma unroll
  for (int kb = 0; kb < 2; kb++)
#pragma unroll
    for (int r = 0; r < 16; r++) {
      float x = s_cur[kb][r];
      if (RAGGED && key0 + 32 * kb + 8 * (r >> 2) + (r & 3) >= nk) x = -INFINITY;
      mxs[kb] = fmaxf(mxs[kb], x);
    }
  float mx = fmaxf(mxs[0], mxs[1]);
  mx = fmaxf(mx, other_half(mx));
  const float m_blk = mx * c2;  // c2 >= 0: the sign of the scale was folded into Q
  // first block: m_run = -inf, so alpha = 0 and the (zero) accumulators stay zero
  if (__any(m_blk > acc.m_run + kRescaleStep)) {
    const float m_new = m_blk > acc.m_run + kRescaleStep ? m_blk : acc.m_run;
    const float alpha = fast_exp2(acc.m_run - m_new);
    acc.m_run = m_new;
    acc.l_run *= alpha;
#pragma unroll
    for (int cb = 0; cb < 2; cb++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc.o[cb][r] *= alpha;
  }
  __builtin_amdgcn_sched_barrier(0);

  // V^T operands: [key block][16-key step][channel block]; they arrive under the exponentials
  u32x4 va[2][2][2];
#pragma unroll
  for (int kb = 0; kb < 2; kb++)
#pragma unroll
    for (int t2 = 0; t2 < 2; t2++)
#pragma unroll
      for (int cb = 0; cb < 2; cb++) va[kb][t2][cb] = cr.read(sV, 2 * kb + t2, cb);
  if (HAS_NEXT) {
#pragma unroll
    for (int t = 0; t < 4; t++)
#pragma unroll
      for (int kb = 0; kb < 2; kb++)
        s_next[kb] = Op<T>::mfma(ka[t][kb], qb[t], t == 0 ? zero : s_next[kb]);
  }
  const float neg_m = -acc.m_run;
  float psum = 0.f;
  u32x4 pb[2][2];  // P^T as B operands: [key block][16-key step]
#pragma unroll
  for (int kb = 0; kb < 2; kb++) {
    float p[16];
#pragma unroll
    for (int r = 0; r < 16; r++) {
      p[r] = fast_exp2(__builtin_fmaf(s_cur[kb][r], c2, neg_m));
      if (RAGGED && key0 + 32 * kb + 8 * (r >> 2) + (r & 3) >= nk) p[r] = 0.f;
    }
#pragma unroll
    for (int t2 = 0; t2 < 2; t2++) {
      u32x4 w;
#pragma unroll
      for (int e = 0; e < 4; e++) {
        w[e] = Op<T>::pack2(p[8 * t2 + 2 * e], p[8 * t2 + 2 * e + 1]);
        psum = Op<T>::add_pair(w[e], psum);  // sums what actually multiplies V
      }
      pb[kb][t2] = w;
    }
  }
  acc.l_run += psum;
  if (HAS_NEXT) {
    // two transpose reads, one MFMA, a dozen vector instructions, eight times over
#pragma unroll
    for (int i = 0; i < 8; i++) {
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, 13, 0);
    }
  }
  __builtin_amdgcn_sched_barrier(0);
  // O^T += V^T P^T : rows = channels (two blocks of 32), contraction over keys
#pragma unroll
  for (int kb = 0; kb < 2; kb++)
#pragma unroll
    for (int t2 = 0; t2 < 2; t2++)
#pragma unroll
      for (int cb = 0; cb < 2; cb++)
        acc.o[cb] = Op<T>::mfma(va[kb][t2][cb], pb[kb][t2], acc.o[cb]);
}

template <typename T>
__global__ __launch_bounds__(kThreads, 2) void fmha_fwd_kernel(const FwdArgs a) {
  __shared__ __align__(1024) uint16_t ring[kRing][2][kTileElems];  // [stage][K|V]
  // The item's 128 query rows (two swizzled tiles): they arrive as whole 128-byte rows.
  __shared__ __align__(1024) uint16_t xbuf[2][kTileElems];

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int g = lane >> 5, ln = lane & 31;
  const int heads = a.pb.heads;
  const int n_items = *a.pb.n_tiles * heads;
  const float c2 = fabsf(a.pb.scale) * kLog2e;  // scores are kept in the log2 domain
  const uint32_t qflip = a.pb.scale < 0.f ? 0x80008000u : 0u;
  const DmaLane dl(wave, lane);
  const RowRead rr(ln, g);
  const ColRead cr(lane);
  const uint32_t ring_addr = lds_addr(&ring[0][0][0]);
  const uint32_t xbuf_addr = lds_addr(&xbuf[0][0]);
  constexpr uint32_t kTileBytes = kTileElems * 2;

  // Start moving key block kt of a (sequence, head) into ring stage `stage`: 4 pieces per thread.
  auto start_block = [&](const TileItem& t, int head, int kt, int stage) {
    const uint16_t* kbase = a.k + (int64_t)t.r0 * a.k_stride + head * kHeadDim;
    const uint16_t* vbase = a.v + (int64_t)t.r0 * a.v_stride + head * kHeadDim;
    const uint32_t st_addr = ring_addr + stage * (2 * kTileBytes);
    if ((kt + 1) * kBlockKeys <= t.nk) {
      const uint16_t* pk = kbase + (kt * kBlockKeys + dl.row) * a.k_stride + dl.chunk * 8;
      const uint16_t* pv = vbase + (kt * kBlockKeys + dl.row) * a.v_stride + dl.chunk * 8;
      dma_tile_full(pk, pk + 32 * a.k_stride, wave, st_addr);
      dma_tile_full(pv, pv + 32 * a.v_stride, wave, st_addr + kTileBytes);
    } else {
      dma_tile(kbase, a.k_stride, kt * kBlockKeys, t.nk - 1, dl, wave, st_addr);
      dma_tile(vbase, a.v_stride, kt * kBlockKeys, t.nk - 1, dl, wave, st_addr + kTileBytes);
    }
  };
  // The first (up to) three key blocks of an item and its 128 query rows (clamped to the
  // sequence; 4 pieces per thread, into xbuf); issued as soon as stages 0..2 and xbuf are
  // free, i.e. before the previous item's outputs are written.
  auto start_item = [&](const TileItem& t, int head) {
    const int n = (t.nk + kBlockKeys - 1) / kBlockKeys;
#pragma unroll
    for (int kt = 0; kt < kRing - 1; kt++)
      if (kt < n) start_block(t, head, kt, kt);
    const uint16_t* qbase = a.q + (int64_t)t.r0 * a.q_stride + head * kHeadDim;
    dma_tile(qbase, a.q_stride, t.row0, t.len - 1, dl, wave, xbuf_addr);
    dma_tile(qbase, a.q_stride, t.row0 + 64, t.len - 1, dl, wave, xbuf_addr + kTileBytes);
  };

  // Persistent workgroups: workgroup b takes items b, b + grid, ...; the record of the
  // next item is fetched while the current one is computed.
  TileItem ti_next = a.pb.tiles[(blockIdx.x < n_items ? blockIdx.x : 0) / heads];
  if (blockIdx.x < n_items) start_item(ti_next, blockIdx.x % heads);
  for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
    const int head = item % heads;
    const TileItem ti = ti_next;
    const int item_next = item + gridDim.x;
    ti_next = a.pb.tiles[(item_next < n_items ? item_next : item) / heads];
    const int r0 = ti.r0, len = ti.len, nk = ti.nk;
    const int qrow = ti.row0 + 32 * wave + ln;       // this lane's query, within the sequence
    const bool wave_on = ti.row0 + 32 * wave < len;  // wavefront has at least one valid row
    const int n = (nk + kBlockKeys - 1) / kBlockKeys;  // blocks of 64 keys

    FwdAcc acc;
#pragma unroll
    for (int cb = 0; cb < 2; cb++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc.o[cb][r] = 0.f;
    acc.m_run = -INFINITY;
    acc.l_run = 0.f;

    // Pipeline: block kt's scores are computed one step early, under block kt-1's
    // exponentials.  At the top of step kt the pieces of blocks kt and kt+1 must have
    // landed (kt+1's keys are read in this step); block kt+3 is started into the stage
    // that block kt-1 occupied.  Each thread has 4 pieces per block in flight.
    static_assert(kRing == 4, "the waits below are written for a ring of four stages");
    // everything in flight is this item's: first key blocks, queries (and the previous
    // item's output rows on their way out)
    wait_vmem<0>();
    __syncthreads();
    // Q^T as the B operand: column = query ln, slots = channels 16t + 8g .. +7.
    // A negative scale is applied as a sign flip of Q so that the row maximum
    // can be taken on the raw scores.
    u32x4 qb[4];
#pragma unroll
    for (int t = 0; t < 4; t++) {
      qb[t] = rr.read(xbuf[wave >> 1], wave & 1, t);
#pragma unroll
      for (int e = 0; e < 4; e++) qb[t][e] ^= qflip;
    }
    if (n > 0) {
      f32x16 sA[2], sB[2];  // scores of even / odd blocks
      if (wave_on) fwd_scores<T>(sA, &ring[0][0][0], qb, rr);
      auto step = [&](int kt, const f32x16 (&s_cur)[2], f32x16 (&s_next)[2]) {
        const int left = n - kt;  // blocks not yet soft-maxed, this one included
        if (left >= 2 && kt > 0) {  // block kt+1 has to be complete (at kt = 0 it already is)
          if (left >= 3)
            wait_vmem<4>();
          else
            wait_vmem<0>();
          __syncthreads();  // also: everyone is done reading block kt-1's stage
        }
        const int stage = kt & 3;
        if (kt + 3 < n) start_block(ti, head, kt + 3, (stage + 3) & 3);
        if (wave_on) {
          const uint16_t* sV = &ring[0][0][0] + stage * (2 * kTileElems) + kTileElems;
          const uint16_t* sKn = &ring[0][0][0] + ((stage + 1) & 3) * (2 * kTileElems);
          if (left >= 2)
            fwd_step<T, false, true>(acc, s_cur, s_next, sKn, sV, qb, c2, kt * kBlockKeys, nk, g, rr, cr);
          else if ((kt + 1) * kBlockKeys > nk)
            fwd_step<T, true, false>(acc, s_cur, s_next, sKn, sV, qb, c2, kt * kBlockKeys, nk, g, rr, cr);
          else
            fwd_step<T, false, false>(acc, s_cur, s_next, sKn, sV, qb, c2, kt * kBlockKeys, nk, g, rr, cr);
        }
      };
      for (int kt = 0; kt < n; kt += 2) {
        step(kt, sA, sB);
        if (kt + 1 < n) step(kt + 1, sB, sA);
      }
    }
    __syncthreads();  // the ring and the query tiles are free
    if (item_next < n_items) start_item(ti_next, item_next % heads);

    // epilogue: combine the two half-rows' sums, normalise; the output rows go through
    // this wavefront's quarter of ring stage 3 (which the next item does not fill before
    // its first barrier) so that they leave as whole 128-byte rows
    if (wave_on) {
      const float l_tot = acc.l_run + other_half(acc.l_run);
      const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
      uint16_t* stage_o = &ring[kRing - 1][0][0] + wave * (32 * 64);
#pragma unroll
      for (int cb = 0; cb < 2; cb++)
#pragma unroll
        for (int j = 0; j < 4; j++) {
          u32x2 w = {Op<T>::pack2(acc.o[cb][4 * j] * inv, acc.o[cb][4 * j + 1] * inv),
                     Op<T>::pack2(acc.o[cb][4 * j + 2] * inv, acc.o[cb][4 * j + 3] * inv)};
          *reinterpret_cast<u32x2*>(stage_o + tile_off(ln, 32 * cb + 8 * j + 4 * g)) = w;
        }
      if (qrow < len && g == 0)
        a.lse[(int64_t)head * a.pb.total_tokens + r0 + qrow] =
            l_tot > 0.f ? (acc.m_run + __builtin_amdgcn_logf(l_tot)) * kLn2 : -INFINITY;
      const int orow0 = ti.row0 + 32 * wave;  // first row of this wavefront's piece
#pragma unroll
      for (int k4 = 0; k4 < 4; k4++) {
        const int row = 8 * k4 + (lane >> 3);
        const u32x4 w = *reinterpret_cast<const u32x4*>(stage_o + tile_off(row, 8 * (lane & 7)));
        if (orow0 + row < len)
          *reinterpret_cast<u32x4*>(a.o + (int64_t)(r0 + orow0 + row) * a.o_stride + head * kHeadDim +
                                    8 * (lane & 7)) = w;
      }
    }
  }
}

}  // namespace fmha
