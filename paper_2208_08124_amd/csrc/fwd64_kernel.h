// Forward kernel, 64 query rows per wavefront: O = softmax(scale Q K^T) V on packed
// rows (Eq. 1 of the paper, one sequence and head at a time), one pass over the keys.
//
// Why this shape.  Measured on MI355X, a wavefront's MFMAs and vector instructions
// overlap when they alternate in program order: an 8-pass MFMA (32 cycles of the matrix
// pipe) keeps the vector ALU from issuing for about 11 cycles, everything else runs
// under it, except v_dot2c, which does not overlap at all.  At head size 64 a score costs 8
// MFMA cycles forward, and the plain recipe (row maximum, fused multiply-add, exp2, add,
// convert) about 20 vector cycles: the forward is bound by the vector ALU, each SIMD by
// itself (measured: redistributing work between workgroups changes nothing).  So the kernel
// is built around the vector instruction count:
//   * one workgroup = 2 wavefronts x 64 query rows = one 128-row tile; the two 32-query
//     blocks (a, b) of a wavefront are independent instruction streams, and every K / V
//     operand read from LDS feeds two MFMAs;
//   * keys move in steps of 32.  Step j is spread over two half-steps, each a single basic
//     block in which the MFMAs do not depend on the vector work beside them:
//       half 1:  softmax of S(j, a)   next to   S(j, b),  O += V(j-1)^T P(j-1),  row sums of P(j-1)
//       half 2:  softmax of S(j, b)   next to   S(j+1, a)
//   * no row maximum per step and no rescaling: the exponent is taken against the maximum m
//     of the first 32 keys.  A later score may exceed m; the probabilities then exceed 1,
//     which is the same softmax (m cancels between numerator and row sum) as long as nothing
//     overflows, and that is checked once per item on the finished row sums: only if a sum
//     is not finite is the item computed again the classic way (running maximum and
//     rescaling in every step; CLASSIC below);
//   * the row sums are formed on the matrix core from the rounded probabilities
//     (Op<T>::sum4), not by vector adds;
//   * per probability that leaves one fused multiply-add, one exp2 and half a convert.
// K and V tiles (32 rows, 4 KB, swizzled as in mfma_tiles.h) move from HBM straight into
// two rings of three LDS slots, K three steps and V two steps ahead of their use, one
// barrier per step between the two wavefronts.  Workgroups are persistent; the item feed
// (item_feed.h) hands them (tile, head) items, and the first transfers of the next item
// (known two items ahead) go out before the current item's results are stored.
#pragma once
#include <type_traits>

#include "item_feed.h"
#include "kernel_args.h"
#include "mfma_tiles.h"

namespace fmha {

constexpr int kF64Threads = 128;  // 2 wavefronts; each owns 64 query rows of the tile
constexpr int kStepKeys = 32;     // keys per step
constexpr int kRing = 3;          // LDS slots per ring
constexpr int kTile32 = 32 * 64;  // elements of a 32-row tile (4 KB)

struct Fwd64Lds {
  uint16_t k[kRing][kTile32];
  uint16_t v[kRing][kTile32];
  uint16_t out[2][kTile32];  // per wavefront: output rows on their way out
  uint32_t mailbox[2];       // first lane to everybody: the item feed's claim (used in turn)
  uint32_t redo[2];          // per wavefront: some row sum of the item was not finite
};

// slot + d in a ring of three (0 <= d <= 3)
__device__ __forceinline__ int ring_add(int slot, int d) {
  const int s = slot + d;
  return s >= kRing ? s - kRing : s;
}

// Pieces a lane moves per 32-row tile: wavefront w fills rows 8w..8w+7 and 16+8w..16+8w+7.
struct DmaLane32 {
  int row;    // first row (second is row + 16)
  int chunk;  // global 16-byte chunk (same for both rows: swz(row) == swz(row + 16))
  __device__ __forceinline__ DmaLane32(int wave, int lane) {
    row = 8 * wave + (lane >> 3);
    chunk = (lane & 7) ^ swz(row);
  }
};

// 32 full rows starting at `rows` (wave-uniform); lane_bytes = (row * stride + chunk * 8) * 2.
static __device__ __forceinline__ void dma_tile32_full(const uint16_t* rows, uint32_t lane_bytes, int64_t stride,
                                                       int wave, uint32_t tile_addr) {
  const uint32_t m0 = __builtin_amdgcn_readfirstlane(tile_addr + 1024u * wave);
  dma16s(rows, lane_bytes, m0);
  dma16s(rows + 16 * stride, lane_bytes, m0 + 2048u);
}

// Rows [row0, row0 + 32) clamped to last_row (the tail of a sequence repeats its last row).
static __device__ __forceinline__ void dma_tile32(const uint16_t* base, int64_t stride, int row0, int last_row,
                                                  const DmaLane32& dl, int wave, uint32_t tile_addr) {
  const int ra = min(dl.row, last_row - row0), rb = min(dl.row + 16, last_row - row0);
  const uint32_t m0 = __builtin_amdgcn_readfirstlane(tile_addr + 1024u * wave);
  const uint16_t* rows = base + uniform_i64((int64_t)row0 * stride);
  const uint32_t st = (uint32_t)stride;
  dma16s(rows, (ra * st + dl.chunk * 8) * 2u, m0);
  dma16s(rows, (rb * st + dl.chunk * 8) * 2u, m0 + 2048u);
}

// Wait for this wavefront's LDS reads, then meet the other wavefront.  (Inline assembly so
// that no fence comes with it: the waits on the transfer counter are the explicit ones.)
static __device__ __forceinline__ void pair_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <typename T>
struct Fwd64State {
  f32x16 o[2][2];  // O^T [channel block][query block]: column = query ln, rows = channels
  f32x16 s[2];     // S^T of the current step, per query block: column = query ln, rows = keys
  f32x4 l[2];      // every element: this lane's share of the running row sum, per query block
  float m[2];      // maximum the exponents are taken against, per query block (log2 domain)
  u32x4 p[2][2];   // P^T of the previous step as B operands [query block][16-key half]
  u32x4 ka[4];     // K operands of the tile from which S(., b) is still to be formed
  u32x4 q[2][4];   // Q^T as B operands [query block][16-channel step]
};

// Two probabilities (registers r, r + 1 of a 32-key x 32-query block) against the maximum m
// (neg_m = -m), packed as one dword of the B operand of the second product.  MASK: register r
// is masked iff 8 (r / 4) + r % 4 >= lim.
template <typename T, bool MASK>
static __device__ __forceinline__ uint32_t softmax_pair(const f32x16& s, int r, float c2, float neg_m, int lim) {
  float p0 = fast_exp2(__builtin_fmaf(s[r], c2, neg_m));
  float p1 = fast_exp2(__builtin_fmaf(s[r + 1], c2, neg_m));
  if (MASK && 8 * (r >> 2) + (r & 3) >= lim) p0 = 0.f;
  if (MASK && 8 * ((r + 1) >> 2) + ((r + 1) & 3) >= lim) p1 = 0.f;
  return Op<T>::pack2(p0, p1);
}

// CLASSIC only: raise the maximum of query block qb to that of its current scores and rescale
// what has been accumulated.
template <typename T>
static __device__ __forceinline__ void raise_maximum(Fwd64State<T>& st, int qb, float c2) {
  float mx = st.s[qb][0];
#pragma unroll
  for (int r = 1; r < 16; r++) mx = fmaxf(mx, st.s[qb][r]);  // rows past the last key repeat it
  mx = fmaxf(mx, other_half(mx));
  const float m_new = fmaxf(st.m[qb], mx * c2);
  const float alpha = fast_exp2(st.m[qb] - m_new);
  st.m[qb] = m_new;
#pragma unroll
  for (int i = 0; i < 4; i++) st.l[qb][i] *= alpha;
#pragma unroll
  for (int cb = 0; cb < 2; cb++)
#pragma unroll
    for (int r = 0; r < 16; r++) st.o[cb][qb][r] *= alpha;
}

// One step of 32 keys for one wavefront.  vt = V tile of the previous step, kt = K tile of
// the next step.  FIRST: there is no previous step (and S(0, b) is already formed);
// LAST: there is no next step, and keys at or beyond nk are masked.
//
// All LDS reads of the step are issued at its start.  Both half-steps then carry the same
// load: 12 MFMAs (8 large, 4 small) beside 40 vector instructions, in eight groups of one
// or two MFMAs followed by the vector work for two probabilities.  The two wavefronts of a
// SIMD issue in order, so whenever both stand at an MFMA, or both at vector work, one of the
// two pipes idles (measured with an MFMA-heavy first and a vector-heavy second half: the
// pipes overlapped a quarter of the time); the fences between the groups keep the
// compiler's scheduler from regrouping them.
template <typename T, bool FIRST, bool LAST, bool CLASSIC>
static __device__ __forceinline__ void fwd64_step(Fwd64State<T>& st, const uint16_t* vt, const uint16_t* kt,
                                                  float c2, int lim, const RowRead& rr, const ColRead& cr) {
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  u32x4 va[2][2], kn[4];
  if (!FIRST) {
#pragma unroll
    for (int t2 = 0; t2 < 2; t2++)
#pragma unroll
      for (int cb = 0; cb < 2; cb++) va[t2][cb] = cr.read(vt, t2, cb);
  }
  if (!LAST) {
#pragma unroll
    for (int t = 0; t < 4; t++) kn[t] = rr.read(kt, 0, t);
  }
  __builtin_amdgcn_sched_barrier(0);
  // MFMA number i (0..11) of the first / second half-step
  auto mfma_first = [&](int i) {
    if (FIRST) return;
    if (i < 4) {
      st.s[1] = Op<T>::mfma(st.ka[i], st.q[1][i], i == 0 ? zero : st.s[1]);  // S(j, b)
    } else if (i < 8) {
      const int cb = (i - 4) >> 1, qb = (i - 4) & 1;
      st.o[cb][qb] = Op<T>::mfma(va[0][cb], st.p[qb][0], st.o[cb][qb]);
    } else {
      const int qb = (i - 8) >> 1, h = (i - 8) & 1;
      st.l[qb] = Op<T>::sum4(u32x2{st.p[qb][0][2 * h], st.p[qb][0][2 * h + 1]}, st.l[qb]);
    }
  };
  auto mfma_second = [&](int i) {
    if (i < 4) {
      if (FIRST) return;
      const int cb = i >> 1, qb = i & 1;
      st.o[cb][qb] = Op<T>::mfma(va[1][cb], st.p[qb][1], st.o[cb][qb]);
    } else if (i < 8) {
      if (FIRST) return;
      const int qb = (i - 4) >> 1, h = (i - 4) & 1;
      st.l[qb] = Op<T>::sum4(u32x2{st.p[qb][1][2 * h], st.p[qb][1][2 * h + 1]}, st.l[qb]);
    } else {
      if (LAST) return;
      st.s[0] = Op<T>::mfma(kn[i - 8], st.q[0][i - 8], i == 8 ? zero : st.s[0]);  // S(j+1, a)
    }
  };
  u32x4 pa[2], pb[2];
  if (CLASSIC) {
    // everything of P(j-1) has to be in before the accumulators are rescaled
#pragma unroll
    for (int i = 0; i < 12; i++) mfma_first(i);
#pragma unroll
    for (int i = 0; i < 8; i++) mfma_second(i);
    raise_maximum<T>(st, 0, c2);
    raise_maximum<T>(st, 1, c2);
#pragma unroll
    for (int e = 0; e < 8; e++) {
      pa[e >> 2][e & 3] = softmax_pair<T, LAST>(st.s[0], 2 * e, c2, -st.m[0], lim);
      pb[e >> 2][e & 3] = softmax_pair<T, LAST>(st.s[1], 2 * e, c2, -st.m[1], lim);
    }
#pragma unroll
    for (int i = 8; i < 12; i++) mfma_second(i);
  } else {
    // Sixteen groups (eight per half-step: first S(j, a) -> P(j, a) beside S(j, b) and the
    // first half of O += V(j-1)^T P(j-1), then S(j, b) -> P(j, b) beside the second half of
    // that and S(j+1, a)).  The vector work is staggered over three groups - multiply-add for
    // pair g, exp2 for pair g-1, convert for pair g-2 - so that no instruction waits for the
    // one just ahead of it.
    float t[2] = {0.f, 0.f}, e2[2] = {0.f, 0.f};
#pragma unroll
    for (int g = 0; g < 18; g++) {
      if (g < 8) {
        mfma_first(3 * g / 2);
        if (g & 1) mfma_first(3 * g / 2 + 1);
      } else if (g < 16) {
        mfma_second(3 * (g - 8) / 2);
        if (g & 1) mfma_second(3 * (g - 8) / 2 + 1);
      }
      // convert pair g-2 (its exponentials were taken in the previous group)
      if (g >= 2) {
        const int e = g - 2, r = 2 * (e & 7);
        float p0 = e2[0], p1 = e2[1];
        if (LAST && 8 * (r >> 2) + (r & 3) >= lim) p0 = 0.f;
        if (LAST && 8 * ((r + 1) >> 2) + ((r + 1) & 3) >= lim) p1 = 0.f;
        uint32_t w = Op<T>::pack2(p0, p1);
        asm volatile("" : "+v"(w));  // (keeps the vector work between the fences)
        if (e < 8)
          pa[e >> 2][e & 3] = w;
        else
          pb[(e - 8) >> 2][e & 3] = w;
      }
      // exp2 for pair g-1
      if (g >= 1 && g < 17) {
        e2[0] = fast_exp2(t[0]);
        e2[1] = fast_exp2(t[1]);
        asm volatile("" : "+v"(e2[0]), "+v"(e2[1]));
      }
      // multiply-add for pair g
      if (g < 16) {
        const int qb = g >> 3, r = 2 * (g & 7);
        t[0] = __builtin_fmaf(st.s[qb][r], c2, -st.m[qb]);
        t[1] = __builtin_fmaf(st.s[qb][r + 1], c2, -st.m[qb]);
        asm volatile("" : "+v"(t[0]), "+v"(t[1]));
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  if (!LAST) {
#pragma unroll
    for (int t = 0; t < 4; t++) st.ka[t] = kn[t];
  }
  st.p[0][0] = pa[0];
  st.p[0][1] = pa[1];
  st.p[1][0] = pb[0];
  st.p[1][1] = pb[1];
}

struct Fwd64Item {
  int r0, len, nk, row0, head;
  int n, n_full;  // steps of 32 keys; complete tiles
};

template <typename T>
__global__ __launch_bounds__(kF64Threads, 2) void fmha_fwd64_kernel(const FwdArgs a) {
  __shared__ __align__(1024) Fwd64Lds lds;

  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // (tells the compiler it is uniform)
  const int heads = a.pb.heads;
  const int n_items = tile_count(a.pb) * heads;
  const float c2 = fabsf(a.pb.scale) * kLog2e;  // scores are kept in the log2 domain
  const uint32_t k_addr = lds_addr(&lds.k[0][0]), v_addr = lds_addr(&lds.v[0][0]);
  constexpr uint32_t kTileBytes = kTile32 * 2;

  auto decode = [&](const TileItem& ti, int item) {
    Fwd64Item x;
    x.r0 = ti.r0;
    x.len = ti.len;
    x.nk = ti.nk;
    x.row0 = ti.row0;
    x.head = item % heads;
    x.n = (ti.nk + kStepKeys - 1) / kStepKeys;
    x.n_full = ti.nk / kStepKeys;
    return x;
  };
  // Transfers of K tile kt / V tile kt of item x (2 per wavefront each) into ring slot `slot`.
  // (lane_bytes = this lane's byte offset within a complete tile, see dma_tile32_full; a
  // partial tile - only ever the last one - forms its clamped offsets on the spot)
  auto start_k = [&](const Fwd64Item& x, int kt, int slot, uint32_t lane_bytes) {
    const uint16_t* kbase = a.k + (int64_t)x.r0 * a.k_stride + x.head * kHeadDim;
    const uint32_t dst = k_addr + slot * kTileBytes;
    if (kt < x.n_full)
      dma_tile32_full(kbase + (int64_t)kt * kStepKeys * a.k_stride, lane_bytes, a.k_stride, wave, dst);
    else
      dma_tile32(kbase, a.k_stride, kt * kStepKeys, x.nk - 1, DmaLane32(wave, lane_id()), wave, dst);
  };
  auto start_v = [&](const Fwd64Item& x, int kt, int slot, uint32_t lane_bytes) {
    const uint16_t* vbase = a.v + (int64_t)x.r0 * a.v_stride + x.head * kHeadDim;
    const uint32_t dst = v_addr + slot * kTileBytes;
    if (kt < x.n_full)
      dma_tile32_full(vbase + (int64_t)kt * kStepKeys * a.v_stride, lane_bytes, a.v_stride, wave, dst);
    else
      dma_tile32(vbase, a.v_stride, kt * kStepKeys, x.nk - 1, DmaLane32(wave, lane_id()), wave, dst);
  };
  auto k_lane_bytes = [&]() {
    const DmaLane32 dl(wave, lane_id());
    return (dl.row * (uint32_t)a.k_stride + dl.chunk * 8) * 2u;
  };
  auto v_lane_bytes = [&]() {
    const DmaLane32 dl(wave, lane_id());
    return (dl.row * (uint32_t)a.v_stride + dl.chunk * 8) * 2u;
  };
  // The first transfers of an item: K(0), K(1), K(2) into slots 0, 1, 2 and V(0) into slot vb
  // (V tile kt lives in slot (kt + vb) % 3: the numbering runs on from item to item).
  auto request_kv = [&](const Fwd64Item& x, int vb) {
    if (x.n == 0) return;
    const uint32_t kl = k_lane_bytes();
    start_k(x, 0, 0, kl);
    if (x.n > 1) start_k(x, 1, 1, kl);
    if (x.n > 2) start_k(x, 2, 2, kl);
    start_v(x, 0, vb, v_lane_bytes());
  };
  // This wavefront's 64 query rows, straight into the operand registers (Q^T as B operands:
  // column = query ln, slots = channels 16t + 8g .. +7; rows past the end of the sequence
  // repeat its last row).
  auto request_q = [&](const Fwd64Item& x, u32x4 (&q)[2][4]) {
    if (x.n == 0) return;
    const int lane = lane_id();
    const int g = lane >> 5, ln = lane & 31;
    const int w0 = min(x.row0 + 64 * wave, x.len - 1);
    const char* qrows =
        reinterpret_cast<const char*>(a.q + uniform_i64((int64_t)(x.r0 + w0) * a.q_stride + x.head * kHeadDim));
    const int room = x.len - 1 - w0;
#pragma unroll
    for (int qb = 0; qb < 2; qb++) {
      const uint32_t off = ((uint32_t)min(32 * qb + ln, room) * (uint32_t)a.q_stride + 8 * g) * 2u;
#pragma unroll
      for (int t = 0; t < 4; t++) q[qb][t] = *reinterpret_cast<const u32x4*>(qrows + off + 32 * t);
    }
  };

  Fwd64State<T> st;

  // All keys of item x for this wavefront's rows: from "K(0) is on its way" to the finished
  // accumulators and row sums.  Returns whether every row sum is finite.
  auto attend = [&](const Fwd64Item& x, int vb, auto classic) -> bool {
    constexpr bool CLASSIC = decltype(classic)::value;
    const int nk = x.nk, n = x.n;
    const bool wave_on = x.row0 + 64 * wave < x.len;
    // Lane-derived values are formed from lane_id() (which the compiler cannot move) inside
    // the item loop: formed ahead of it they would be held in registers through all of it.
    const int lane = lane_id();
    const int g = lane >> 5, ln = lane & 31;
    const RowRead rr(ln, g);
    const ColRead cr(lane);
#pragma unroll
    for (int qb = 0; qb < 2; qb++) {
      st.m[qb] = 0.f;
      st.l[qb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int cb = 0; cb < 2; cb++)
#pragma unroll
        for (int r = 0; r < 16; r++) st.o[cb][qb][r] = 0.f;
    }
    // K(0) has landed once only the later transfers are outstanding (transfers complete in
    // issue order; stores of the previous item that are still on their way only make the
    // wait longer)
    if (n > 2)
      wait_vmem<6>();
    else if (n > 1)
      wait_vmem<4>();
    else
      wait_vmem<2>();
    pair_barrier();
    if (n > 0) {
      if (!CLASSIC) {
        // The query rows were requested ahead of K(0), so they are in as well.  The compiler
        // tracks those loads but not the transfers issued after them, so its own wait could
        // fall short; routing the registers through this statement keeps every use of them
        // below the wait above.
#pragma unroll
        for (int qb = 0; qb < 2; qb++)
#pragma unroll
          for (int t = 0; t < 4; t++) asm volatile("" : "+v"(st.q[qb][t]));
        // A negative scale is applied as a sign flip of Q, so that c2 >= 0 and the maximum of
        // the raw scores is the maximum of the scaled ones.
        if (a.pb.scale < 0.f) {
#pragma unroll
          for (int qb = 0; qb < 2; qb++)
#pragma unroll
            for (int t = 0; t < 4; t++)
#pragma unroll
              for (int e = 0; e < 4; e++) st.q[qb][t][e] ^= 0x80008000u;
        }
      }
      // S(0) for both query blocks, and its exact row maximum
      {
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int t = 0; t < 4; t++) st.ka[t] = rr.read(&lds.k[0][0], 0, t);
#pragma unroll
        for (int t = 0; t < 4; t++) {
          st.s[0] = Op<T>::mfma(st.ka[t], st.q[0][t], t == 0 ? zero : st.s[0]);
          st.s[1] = Op<T>::mfma(st.ka[t], st.q[1][t], t == 0 ? zero : st.s[1]);
        }
#pragma unroll
        for (int qb = 0; qb < 2; qb++) {
          float mx = st.s[qb][0];
#pragma unroll
          for (int r = 1; r < 16; r++) mx = fmaxf(mx, st.s[qb][r]);  // rows past the last key repeat it
          mx = fmaxf(mx, other_half(mx));
          st.m[qb] = mx * c2;
        }
      }
      // the last tile masks keys at or beyond nk: register r is masked iff 8 (r / 4) + r % 4 >= lim
      const int lim = nk - (n - 1) * kStepKeys - 4 * g;

      // Step j needs K(j+1) and V(j-1), requested two steps earlier, and requests K(j+3)
      // (into the slot of K(j)) and V(j+1) (into the slot of V(j-2)).  Transfers complete in
      // issue order: once K(j+1) and V(j-1) are in, only step j-1's requests K(j+2), V(j)
      // (at step 0: K(2), V(0)) can still be on their way.
      // ks / vs: ring slots of K(j+1) / V(j-1), kept as running scalars.
      int ks = 1, vs = ring_add(vb, 2);
      const uint32_t kl = k_lane_bytes(), vl = v_lane_bytes();
      auto open_step = [&](int j) {
        if (j + 2 < n)
          wait_vmem<4>();
        else
          wait_vmem<2>();
        pair_barrier();
        if (j + 3 < n) start_k(x, j + 3, ring_add(ks, 2), kl);
        if (j + 1 < n) start_v(x, j + 1, ring_add(vs, 2), vl);
      };
      auto close_step = [&]() {
        ks = ring_add(ks, 1);
        vs = ring_add(vs, 1);
      };
      open_step(0);
      if (wave_on) {
        if (n == 1)
          fwd64_step<T, true, true, CLASSIC>(st, &lds.v[0][0], &lds.k[0][0], c2, lim, rr, cr);
        else
          fwd64_step<T, true, false, CLASSIC>(st, &lds.v[0][0], &lds.k[1][0], c2, lim, rr, cr);
      }
      close_step();
      // The steps in the middle of a long sequence run without a single branch besides the
      // loop's own (a wavefront alone on its SIMD was measured at 9 cycles per instruction
      // with the ten or so branches per step the general form below has): all of K(j+3),
      // V(j+1) are complete tiles there.
      int j = 1;
      if (wave_on) {
        const uint16_t* kbase = a.k + uniform_i64((int64_t)x.r0 * a.k_stride + x.head * kHeadDim);
        const uint16_t* vbase = a.v + uniform_i64((int64_t)x.r0 * a.v_stride + x.head * kHeadDim);
        for (; j + 3 < x.n_full; j++) {
          wait_vmem<4>();
          pair_barrier();
          dma_tile32_full(kbase + uniform_i64((int64_t)(j + 3) * kStepKeys * a.k_stride), kl, a.k_stride, wave,
                          k_addr + ring_add(ks, 2) * kTileBytes);
          dma_tile32_full(vbase + uniform_i64((int64_t)(j + 1) * kStepKeys * a.v_stride), vl, a.v_stride, wave,
                          v_addr + ring_add(vs, 2) * kTileBytes);
          fwd64_step<T, false, false, CLASSIC>(st, &lds.v[0][0] + vs * kTile32, &lds.k[0][0] + ks * kTile32, c2,
                                               lim, rr, cr);
          close_step();
        }
      }
      for (; j + 1 < n; j++) {
        open_step(j);
        if (wave_on)
          fwd64_step<T, false, false, CLASSIC>(st, &lds.v[0][0] + vs * kTile32, &lds.k[0][0] + ks * kTile32, c2,
                                               lim, rr, cr);
        close_step();
      }
      if (n > 1) {
        open_step(n - 1);
        if (wave_on)
          fwd64_step<T, false, true, CLASSIC>(st, &lds.v[0][0] + vs * kTile32, &lds.k[0][0], c2, lim, rr, cr);
        close_step();
      }
      // all transfers of this item are in
      wait_vmem<0>();
      pair_barrier();
      // O += V(n-1)^T P(n-1), and the last row sums
      if (wave_on) {
        const uint16_t* vt = &lds.v[0][0] + vs * kTile32;
#pragma unroll
        for (int t2 = 0; t2 < 2; t2++) {
          const u32x4 va[2] = {cr.read(vt, t2, 0), cr.read(vt, t2, 1)};
#pragma unroll
          for (int cb = 0; cb < 2; cb++)
#pragma unroll
            for (int qb = 0; qb < 2; qb++) st.o[cb][qb] = Op<T>::mfma(va[cb], st.p[qb][t2], st.o[cb][qb]);
#pragma unroll
          for (int qb = 0; qb < 2; qb++) {
            st.l[qb] = Op<T>::sum4(u32x2{st.p[qb][t2][0], st.p[qb][t2][1]}, st.l[qb]);
            st.l[qb] = Op<T>::sum4(u32x2{st.p[qb][t2][2], st.p[qb][t2][3]}, st.l[qb]);
          }
        }
      }
    }
    const float lsum = st.l[0][0] + st.l[1][0];
    return __builtin_amdgcn_ballot_w64(!(fabsf(lsum) < 3.0e38f)) == 0;
  };

  // persistent workgroups; the item feed hands out the (tile, head) items, two ahead
  ItemFeed feed;
  int item = feed.init(a.feed, blockIdx.x, gridDim.x);
  if (item >= n_items) {
    feed.finish(a.feed, gridDim.x);
    return;
  }
  int item1 = feed.next();
  Fwd64Item cur = decode(load_tile(a.pb, item / heads), item);
  TileItem ti1 = load_tile(a.pb, (item1 < n_items ? item1 : item) / heads);
  int vb = 0, parity = 0;
  request_q(cur, st.q);
  request_kv(cur, vb);

  while (true) {
    const bool has_next = item1 < n_items;
    const int n = cur.n;
    const bool fine = attend(cur, vb, std::false_type{});
    int vb_next = (vb + n) % kRing;

    // One more barrier at the item's end: it tells both wavefronts whether either one saw a
    // row sum that is not finite, and carries the item feed's claim from the first lane to
    // everybody.  (The words are rewritten an item later at the earliest, with other
    // barriers in between; the mailbox words are used in turn on top of that.)
    if ((threadIdx.x & 63) == 0) lds.redo[wave] = fine ? 0u : 1u;
    feed.publish(&lds.mailbox[parity]);
    pair_barrier();
    const bool redo = __builtin_amdgcn_readfirstlane((int)(lds.redo[0] | lds.redo[1])) != 0;
    feed.receive(&lds.mailbox[parity]);
    parity ^= 1;
    if (redo) {
      request_kv(cur, vb_next);
      attend(cur, vb_next, std::true_type{});
      vb_next = (vb_next + n) % kRing;
    }

    // the item after the next one: its record is fetched now and used an item later
    const int item2 = feed.next();
    feed.request(a.feed);  // answered long before the end of the next item
    const TileItem ti2 = load_tile(a.pb, (item2 < n_items ? item2 : item) / heads);

    // The next item's first transfers go out before this item's results are stored.  Both
    // wavefronts are past the barriers above, so all K slots are free; V(0) of the next item
    // takes the slot after this item's last V tile, which the other wavefront may still be
    // reading.
    const Fwd64Item done = cur;
    if (has_next) {
      cur = decode(ti1, item1);
      request_q(cur, st.q);
      request_kv(cur, vb_next);
    }

    // epilogue: combine the two half-rows' sums, normalise, store LSE and O (as whole rows,
    // turned around in the wavefront's output scratch, one 32-row block at a time)
    const int len = done.len;
    const int qrow0 = done.row0 + 64 * wave;  // first query row of this wavefront, within the sequence
    if (qrow0 < len) {
#pragma unroll
      for (int qb = 0; qb < 2; qb++) {
        const int row = qrow0 + 32 * qb;  // first row of the block, within the sequence
        if (row < len) {
          const float l_tot = st.l[qb][0] + other_half(st.l[qb][0]);
          const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
          const int le = lane_id();
          if (row + (le & 31) < len && le < 32) {
            float* lrow = a.lse + uniform_i64((int64_t)done.head * a.pb.total_tokens + done.r0 + row);
            lrow[le & 31] = l_tot > 0.f ? (st.m[qb] + __builtin_amdgcn_logf(l_tot)) * kLn2 : -INFINITY;
          }
          const f32x16 ot[2] = {st.o[0][qb], st.o[1][qb]};
          store_rows32<T>(ot, inv, &lds.out[wave][0], a.o,
                          (int64_t)(done.r0 + row) * a.o_stride + done.head * kHeadDim, a.o_stride, len - row);
        }
      }
    }
    if (!has_next) break;
    vb = vb_next;
    item = item1;
    item1 = item2;
    ti1 = ti2;
  }
  feed.finish(a.feed, gridDim.x);
}

}  // namespace fmha
