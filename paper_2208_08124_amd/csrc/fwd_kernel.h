// Forward kernel: O = softmax(scale Q K^T) V on packed rows (Eq. 1 of the
// paper, one sequence and head at a time), fused in one pass over the keys
// with a running row maximum and row sum.
//
// One workgroup (4 wavefronts) takes one tile of 128 query rows of one
// (sequence, head); wavefront w owns rows 32w..32w+31.  Keys and values move
// 64 rows at a time from HBM straight into a ring of three LDS stages, two
// blocks ahead of the one being computed, with one barrier per block.  A
// wavefront's 32 query rows arrive the same way, into rows of the ring that
// only its own transfers write, together with the first key blocks; its 32
// output rows leave through the same rows as whole 128-byte rows.
//
// The scores are produced TRANSPOSED, S^T = K Q^T, so that in the MFMA result
// layout every lane holds 16 keys of ONE query: the row maximum and row sum
// are then per-lane reductions plus a single exchange with the lane 32 away,
// and the probabilities are already in the operand layout of the second
// product O^T = V^T P^T.
//
// The softmax competes with the matrix cores for issue slots (a v_exp_f32
// costs a quarter of the MFMA time a score needs), so the vector work per score
// is kept to one fused multiply-add, one exp2, half a max3, half a pack and
// half a dot2 (row sum).  The kernel is kept lean in registers (three
// wavefronts per SIMD): measured on MI355X, that occupancy hides the LDS and
// MFMA latencies at least as well as software-pipelining two blocks inside a
// wavefront, which costs the third wavefront.
//
// The running maximum is only raised when a block exceeds it by more than
// kRescaleStep (log2 units); until then probabilities may exceed 1 (by at most
// 2^kRescaleStep: harmless in fp16/bf16 and fp32) and the accumulators are not
// rescaled.  The result is the same softmax: the maximum cancels between
// numerator and row sum.
#pragma once
#include "dropout.h"
#include "kernel_args.h"
#include "mfma_tiles.h"

namespace fmha {

constexpr float kRescaleStep = 8.f;
constexpr int kFwdStages = 3;  // LDS ring: one K and one V tile per stage (16 KB)

struct FwdAcc {
  f32x16 o[2];  // O^T: column = query ln; o[cb][r] is channel 32cb + 8(r/4) + 4g + r%4
  float m_run;  // running maximum, log2 domain (scaled by |scale|*log2 e)
  float l_run;  // this lane's share of the running row sum
};

// One block of 64 keys for one wavefront.  RAGGED: keys at or beyond nk (only
// possible in a sequence's last block) are excluded.  The LDS reads of each
// product are issued together ahead of its MFMAs (the sched_barrier keeps the
// compiler from sinking each read next to its use, which would serialise LDS
// latency with every MFMA); the transpose reads of V fly during the
// exponentials.
// DROP: dropout on the probabilities.  q4 = (this lane's query) >> 2; the running row sum
// then takes the probabilities before the mask, the second product those that are kept
// (their common factor 1/(1-p) is applied once, to the finished rows).
template <typename T, bool RAGGED, bool DROP>
__device__ __forceinline__ void fwd_block(FwdAcc& acc, const uint16_t* sK, const uint16_t* sV,
                                          const u32x4 (&qb)[4], float c2, int key_base, int nk,
                                          int g, const RowRead& rr, const ColRead& cr, int q4,
                                          int ln, int r0, int head, const DropArgs& drop) {
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  // S^T = K Q^T : rows = keys (two blocks of 32), column = query ln
  f32x16 s[2];
  const bool one_half = RAGGED && key_base + 32 >= nk;  // uniform: no key in the second 32
  {
    u32x4 ka[4][2];
#pragma unroll
    for (int t = 0; t < 4; t++)
#pragma unroll
      for (int kb = 0; kb < 2; kb++)
        if (kb == 0 || !one_half) ka[t][kb] = rr.read(sK, kb, t);
    __builtin_amdgcn_sched_barrier(0);
    if (one_half) {
#pragma unroll
      for (int t = 0; t < 4; t++) s[0] = Op<T>::mfma(ka[t][0], qb[t], t == 0 ? zero : s[0]);
    } else {
#pragma unroll
      for (int t = 0; t < 4; t++)
#pragma unroll
        for (int kb = 0; kb < 2; kb++) s[kb] = Op<T>::mfma(ka[t][kb], qb[t], t == 0 ? zero : s[kb]);
    }
  }
  // the mask bytes do not depend on the scores: their arithmetic fills the time the
  // matrix cores need for the products just issued
  uint32_t kb8[2][4];
  if (DROP) {
    keep_bytes<false>(kb8[0], q4, (key_base >> 2) + g, ln, r0, head, drop);
    if (!one_half) keep_bytes<false>(kb8[1], q4, ((key_base + 32) >> 2) + g, ln, r0, head, drop);
  }
  __builtin_amdgcn_sched_barrier(0);
  const int key0 = key_base + 4 * g;      // key of s[0][0]
  float mxs[2] = {-INFINITY, -INFINITY};  // two independent chains
#pragma unroll
  for (int kb = 0; kb < 2; kb++) {
    if (kb == 1 && one_half) break;
#pragma unroll
    for (int r = 0; r < 16; r++) {
      // no mask needed here: the rows of a ragged block past the last key repeat
      // that key (the fetch clamps the row index), so they cannot raise the maximum
      mxs[kb] = fmaxf(mxs[kb], s[kb][r]);
    }
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
  const float neg_m = -acc.m_run;
  float psum = 0.f;
#pragma unroll
  for (int kb = 0; kb < 2; kb++) {
    if (kb == 1 && one_half) break;
    u32x4 va[2][2];  // V^T operands of this half: [16-key step][channel block]
#pragma unroll
    for (int t2 = 0; t2 < 2; t2++)
#pragma unroll
      for (int cb = 0; cb < 2; cb++) va[t2][cb] = cr.read(sV, 2 * kb + t2, cb);
    float p[16];
#pragma unroll
    for (int r = 0; r < 16; r++) {
      p[r] = fast_exp2(__builtin_fmaf(s[kb][r], c2, neg_m));
      if (RAGGED && key0 + 32 * kb + 8 * (r >> 2) + (r & 3) >= nk) p[r] = 0.f;
      if (DROP) {
        psum += p[r];
        if (!kept(kb8[kb], r, drop.thr)) p[r] = 0.f;
      }
    }
    u32x4 pb[2];  // P^T as B operands, one per 16-key step
#pragma unroll
    for (int t2 = 0; t2 < 2; t2++) {
      u32x4 w;
#pragma unroll
      for (int e = 0; e < 4; e++) {
        w[e] = Op<T>::pack2(p[8 * t2 + 2 * e], p[8 * t2 + 2 * e + 1]);
        if (!DROP) psum = Op<T>::add_pair(w[e], psum);  // sums what actually multiplies V
      }
      pb[t2] = w;
    }
    // O^T += V^T P^T : rows = channels (two blocks of 32), contraction over keys
#pragma unroll
    for (int t2 = 0; t2 < 2; t2++)
#pragma unroll
      for (int cb = 0; cb < 2; cb++) acc.o[cb] = Op<T>::mfma(va[t2][cb], pb[t2], acc.o[cb]);
  }
  acc.l_run += psum;
}

template <typename T, bool DROP>
__global__ __launch_bounds__(kThreads, 3) void fmha_fwd_kernel(const FwdArgs a) {
  constexpr int kPerCu = 3;  // workgroups per compute unit (the launcher's grid assumes it)
  __shared__ __align__(1024) uint16_t ring[kFwdStages][2][kTileElems];  // [stage][K|V]

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int g = lane >> 5, ln = lane & 31;
  const int heads = a.pb.heads;
  const int n_items = tile_count(a.pb) * heads;
  const float c2 = fabsf(a.pb.scale) * kLog2e;  // scores are kept in the log2 domain
  const uint32_t qflip = a.pb.scale < 0.f ? 0x80008000u : 0u;
  const int slot = blockIdx.x / max(gridDim.x / (unsigned)kPerCu, 1u);  // which of the workgroups of its compute unit
  const DmaLane dl(wave, lane);
  const RowRead rr(ln, g);
  const ColRead cr(lane);
  const uint32_t ring_addr = lds_addr(&ring[0][0][0]);
  constexpr uint32_t kTileBytes = kTileElems * 2;
  // this lane's piece within a 64-row block (rows dl.row and dl.row + 32), in elements
  const uint32_t k_lane = (dl.row * (uint32_t)a.k_stride + dl.chunk * 8) * 2u;  // bytes
  const uint32_t v_lane = (dl.row * (uint32_t)a.v_stride + dl.chunk * 8) * 2u;

  // Persistent workgroups: workgroup b takes items b, b + grid, ...; the record of the
  // next item is fetched while the current one is computed.
  TileItem ti_next = load_tile(a.pb, ((int)blockIdx.x < n_items ? (int)blockIdx.x : 0) / heads);
  for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
    const int head = item % heads;
    const TileItem ti = ti_next;
    {
      const int nxt = item + gridDim.x;
      ti_next = load_tile(a.pb, (nxt < n_items ? nxt : item) / heads);
    }
    const int r0 = ti.r0, len = ti.len, nk = ti.nk;
    const bool wave_on = ti.row0 + 32 * wave < len;  // wavefront has at least one valid row
    const uint16_t* kbase = a.k + (int64_t)r0 * a.k_stride + head * kHeadDim;
    const uint16_t* vbase = a.v + (int64_t)r0 * a.v_stride + head * kHeadDim;
    const int n = (nk + kBlockKeys - 1) / kBlockKeys;  // blocks of 64 keys

    // Start moving key block kt into ring stage `stage`: 4 pieces per thread.
    // (the empty asm keeps the lane offsets from being combined with anything ahead of the
    // item loop and held in registers through it)
    uint32_t kl = k_lane, vl = v_lane;
    asm volatile("" : "+v"(kl), "+v"(vl));
    auto start_block = [&](int kt, int stage) {
      const uint32_t st_addr = ring_addr + stage * (2 * kTileBytes);
      if ((kt + 1) * kBlockKeys <= nk) {
        dma_tile_full(kbase + (int64_t)kt * kBlockKeys * a.k_stride, kl, a.k_stride, wave, st_addr);
        dma_tile_full(vbase + (int64_t)kt * kBlockKeys * a.v_stride, vl, a.v_stride, wave, st_addr + kTileBytes);
      } else {
        dma_tile(kbase, a.k_stride, kt * kBlockKeys, nk - 1, dl, wave, st_addr);
        dma_tile(vbase, a.v_stride, kt * kBlockKeys, nk - 1, dl, wave, st_addr + kTileBytes);
      }
    };
    // Q first: each wavefront moves its own 32 query rows (four pieces of eight
    // rows) into its private 4 KB of the last ring stage - the rows of that stage
    // which only this wavefront's own fetches write, so no barrier is involved -
    // ahead of the first two key blocks; they are awaited together with block 0.
    const uint32_t own_addr = ring_addr + (kFwdStages - 1) * (2 * kTileBytes) + 1024u * wave;
    {
      // rows relative to the wavefront's first row (clamped into the sequence, so that the
      // offsets of a wavefront that lies entirely past the end stay non-negative)
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

    FwdAcc acc;
#pragma unroll
    for (int cb = 0; cb < 2; cb++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc.o[cb][r] = 0.f;
    acc.m_run = -INFINITY;
    acc.l_run = 0.f;

    // Q and block 0 have landed once at most the 4 pieces of block 1 are outstanding
    // (vector memory loads complete in issue order).
    if (n > 1)
      wait_vmem<4>();
    else
      wait_vmem<0>();
    // Q^T as the B operand: column = query ln, slots = channels 16t + 8g .. +7.  A
    // negative scale is applied as a sign flip of Q so that the row maximum can be
    // taken on the raw scores.
    u32x4 qb[4];
    {
      const uint16_t* sq = &ring[kFwdStages - 1][0][0] + 512 * wave + own_piece(ln >> 3) / 2 + (ln & 7) * 64;
      const int sw = swz(ln);
#pragma unroll
      for (int t = 0; t < 4; t++) {
        qb[t] = *reinterpret_cast<const u32x4*>(sq + (((2 * t + g) ^ sw) << 3));
#pragma unroll
        for (int e = 0; e < 4; e++) qb[t][e] ^= qflip;
      }
    }

    int stage = 0;  // kt % 3
    for (int kt = 0; kt < n; kt++) {
      // this thread's pieces of block kt have landed once at most the 4 pieces of
      // block kt+1 are outstanding (vector memory loads complete in issue order)
      if (kt + 1 < n)
        wait_vmem<4>();
      else
        wait_vmem<0>();
      __syncthreads();  // everyone's pieces landed; everyone is done with block kt-1's stage
      rotate_priority(kt, slot, kPerCu);
      const int ahead = stage == 0 ? kFwdStages - 1 : stage - 1;  // (kt + 2) % 3
      if (kt + 2 < n) start_block(kt + 2, ahead);
      if (wave_on) {
        const uint16_t* sK = &ring[0][0][0] + stage * (2 * kTileElems);
        const uint16_t* sV = sK + kTileElems;
        const int q4 = (ti.row0 + 32 * wave + ln) >> 2;
        if ((kt + 1) * kBlockKeys > nk)
          fwd_block<T, true, DROP>(acc, sK, sV, qb, c2, kt * kBlockKeys, nk, g, rr, cr, q4, ln, r0, head, a.drop);
        else
          fwd_block<T, false, DROP>(acc, sK, sV, qb, c2, kt * kBlockKeys, nk, g, rr, cr, q4, ln, r0, head, a.drop);
      }
      stage = stage == kFwdStages - 1 ? 0 : stage + 1;
    }
    __syncthreads();  // the ring is free for the next item

    // epilogue: combine the two half-rows' sums, normalise, store LSE and O (as
    // whole rows, turned around in the wavefront's private rows of the last stage)
    if (wave_on) {
      const float l_tot = acc.l_run + other_half(acc.l_run);
      const float inv = l_tot > 0.f ? (DROP ? a.drop.rp : 1.f) / l_tot : 0.f;
      const int le = lane_id();
      const int qrow = ti.row0 + 32 * wave + (le & 31);  // this lane's query, within the sequence
      if (qrow < len && le < 32) {
        float* lrow = a.lse + uniform_i64((int64_t)head * a.pb.total_tokens + r0 + ti.row0 + 32 * wave);
        lrow[le & 31] = l_tot > 0.f ? (acc.m_run + __builtin_amdgcn_logf(l_tot)) * kLn2 : -INFINITY;
      }
      store_rows<T>(acc.o, inv, &ring[kFwdStages - 1][0][0], wave, a.o,
                    (int64_t)(r0 + ti.row0 + 32 * wave) * a.o_stride + head * kHeadDim, a.o_stride,
                    len - (ti.row0 + 32 * wave));
    }
  }
}

}  // namespace fmha
