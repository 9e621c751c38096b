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
// Both orientations are chosen so that the MFMA result tile of the first two
// products has, in every lane, the reduction index of the following product
// spread over its registers; P and dS then go back in as B operands without
// passing through LDS, and the per-row statistics (LSE, D) are per-lane
// scalars in pass 1 and broadcast LDS reads in pass 2.
#pragma once
#include "fwd_kernel.h"

namespace fmha {

// Register-staged, padded LDS tiles (row stride 64 + 8 elements).
constexpr int kLdsRow = 72;

__device__ __forceinline__ void load_tile_regs(const uint16_t* __restrict__ base, int64_t stride,
                                               int row0, int nrows, int tid, u32x4 (&r)[2]) {
#pragma unroll
  for (int i = 0; i < 2; i++) {
    const int c = tid + kThreads * i;
    const int row = row0 + (c >> 3);
    r[i] = u32x4{0, 0, 0, 0};
    if (row < nrows) r[i] = *reinterpret_cast<const u32x4*>(base + row * stride + (c & 7) * 8);
  }
}

__device__ __forceinline__ void store_tile_lds(uint16_t* tile, int tid, const u32x4 (&r)[2]) {
#pragma unroll
  for (int i = 0; i < 2; i++) {
    const int c = tid + kThreads * i;
    *reinterpret_cast<u32x4*>(tile + (c >> 3) * kLdsRow + (c & 7) * 8) = r[i];
  }
}

static __device__ __forceinline__ u32x4 pad_read_row8(const uint16_t* tile, int row, int col) {
  return *reinterpret_cast<const u32x4*>(tile + row * kLdsRow + col);
}

static __device__ __forceinline__ u32x4 pad_read_col8(const uint16_t* tile, int base, int col16,
                                                      int lane16) {
  const uint16_t* p = tile + (base + (lane16 >> 2)) * kLdsRow + col16 + 4 * (lane16 & 3);
  u32x2 a = lds_read_tr16(p);
  u32x2 b = lds_read_tr16(p + 8 * kLdsRow);
  return u32x4{a[0], a[1], b[0], b[1]};
}

// ---------------------------------------------------------------- pass 1: dQ
template <typename T>
__global__ __launch_bounds__(kThreads, 2) void bwd_dq_kernel(const BwdArgs a) {
  __shared__ __align__(16) uint16_t sK[kBlockKeys * kLdsRow];
  __shared__ __align__(16) uint16_t sV[kBlockKeys * kLdsRow];

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int g = lane >> 5, ln = lane & 31, lane16 = lane & 15, half16 = (lane >> 4) & 1;
  const int heads = a.pb.heads;
  const int n_items = *a.pb.n_tiles * heads;
  const float c2 = a.pb.scale * kLog2e;

  for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
    const int head = item % heads;
    const TileItem ti = a.pb.tiles[item / heads];
    const int r0 = a.pb.cu[ti.seq];
    const int len = a.pb.cu[ti.seq + 1] - r0;
    int nk = a.pb.seqused ? min(a.pb.seqused[ti.seq], len) : len;
    nk = nk < 0 ? 0 : nk;
    const int qrow = ti.row0 + 32 * wave + ln;
    const bool wave_on = ti.row0 + 32 * wave < len;
    const bool row_on = qrow < len;
    const uint16_t* kbase = a.k + (int64_t)r0 * a.k_stride + head * kHeadDim;
    const uint16_t* vbase = a.v + (int64_t)r0 * a.v_stride + head * kHeadDim;

    // Q^T and dO^T as B operands (column = query ln, slots = channels 16t+8g..+7),
    // and D = sum_c dO*O over this lane's 32 channels, completed with the other half.
    u32x4 qb[4], gb[4];
    float dsum = 0.f, lse2 = 0.f;
    {
      const int qr = row_on ? qrow : len - 1;
      const int64_t tok = r0 + qr;
      const uint16_t* qp = a.q + tok * a.q_stride + head * kHeadDim + 8 * g;
      const uint16_t* gp = a.d_o + tok * a.do_stride + head * kHeadDim + 8 * g;
      const uint16_t* op = a.o + tok * a.o_stride + head * kHeadDim + 8 * g;
#pragma unroll
      for (int t = 0; t < 4; t++) {
        qb[t] = *reinterpret_cast<const u32x4*>(qp + 16 * t);
        gb[t] = *reinterpret_cast<const u32x4*>(gp + 16 * t);
        const u32x4 ov = *reinterpret_cast<const u32x4*>(op + 16 * t);
#pragma unroll
        for (int e = 0; e < 4; e++)
          dsum += Op<T>::lo(gb[t][e]) * Op<T>::lo(ov[e]) + Op<T>::hi(gb[t][e]) * Op<T>::hi(ov[e]);
      }
      dsum += other_half(dsum);
      const int64_t si = (int64_t)head * a.pb.total_tokens + tok;
      lse2 = a.lse[si] * kLog2e;
      if (row_on && g == 0) a.dsum[si] = dsum;
    }

    f32x16 dq[2];  // dQ^T: column = query ln, rows = channels
#pragma unroll
    for (int cb = 0; cb < 2; cb++)
#pragma unroll
      for (int r = 0; r < 16; r++) dq[cb][r] = 0.f;

    const int n_kt = (nk + kBlockKeys - 1) / kBlockKeys;
    u32x4 kreg[2], vreg[2];
    if (n_kt > 0) {
      load_tile_regs(kbase, a.k_stride, 0, nk, tid, kreg);
      load_tile_regs(vbase, a.v_stride, 0, nk, tid, vreg);
      store_tile_lds(sK, tid, kreg);
      store_tile_lds(sV, tid, vreg);
    }
    __syncthreads();

    for (int kt = 0; kt < n_kt; kt++) {
      const bool more = kt + 1 < n_kt;
      if (more) {
        load_tile_regs(kbase, a.k_stride, (kt + 1) * kBlockKeys, nk, tid, kreg);
        load_tile_regs(vbase, a.v_stride, (kt + 1) * kBlockKeys, nk, tid, vreg);
      }
      if (wave_on) {
        const int key0 = kt * kBlockKeys + 4 * g;
        const bool ragged = key0 - 4 * g + kBlockKeys > nk;
        u32x4 dsb[2][2];  // dS^T as B operands
#pragma unroll
        for (int kb = 0; kb < 2; kb++) {
          f32x16 s, dp;
#pragma unroll
          for (int r = 0; r < 16; r++) s[r] = dp[r] = 0.f;
#pragma unroll
          for (int t = 0; t < 4; t++) {
            s = Op<T>::mfma(pad_read_row8(sK, 32 * kb + ln, 16 * t + 8 * g), qb[t], s);
            dp = Op<T>::mfma(pad_read_row8(sV, 32 * kb + ln, 16 * t + 8 * g), gb[t], dp);
          }
          float ds[16];
#pragma unroll
          for (int r = 0; r < 16; r++) {
            float p = fast_exp2(s[r] * c2 - lse2);
            if (ragged && key0 + 32 * kb + 8 * (r >> 2) + (r & 3) >= nk) p = 0.f;
            ds[r] = p * (dp[r] - dsum);
          }
#pragma unroll
          for (int t2 = 0; t2 < 2; t2++)
            dsb[kb][t2] = u32x4{Op<T>::pack2(ds[8 * t2 + 0], ds[8 * t2 + 1]),
                                Op<T>::pack2(ds[8 * t2 + 2], ds[8 * t2 + 3]),
                                Op<T>::pack2(ds[8 * t2 + 4], ds[8 * t2 + 5]),
                                Op<T>::pack2(ds[8 * t2 + 6], ds[8 * t2 + 7])};
        }
        // dQ^T += K^T dS^T : rows = channels, contraction over keys
#pragma unroll
        for (int cb = 0; cb < 2; cb++)
#pragma unroll
          for (int kb = 0; kb < 2; kb++)
#pragma unroll
            for (int t2 = 0; t2 < 2; t2++)
              dq[cb] = Op<T>::mfma(
                  pad_read_col8(sK, 32 * kb + 16 * t2 + 4 * g, 32 * cb + 16 * half16, lane16),
                  dsb[kb][t2], dq[cb]);
      }
      __syncthreads();
      if (more) {
        store_tile_lds(sK, tid, kreg);
        store_tile_lds(sV, tid, vreg);
      }
      __syncthreads();
    }

    if (row_on) {
      const float sc = a.pb.scale;
      uint16_t* op = a.dq + (int64_t)(r0 + qrow) * a.dq_stride + head * kHeadDim + 4 * g;
#pragma unroll
      for (int cb = 0; cb < 2; cb++)
#pragma unroll
        for (int j = 0; j < 4; j++) {
          u32x2 w = {Op<T>::pack2(dq[cb][4 * j] * sc, dq[cb][4 * j + 1] * sc),
                     Op<T>::pack2(dq[cb][4 * j + 2] * sc, dq[cb][4 * j + 3] * sc)};
          *reinterpret_cast<u32x2*>(op + 32 * cb + 8 * j) = w;
        }
    }
  }
}

// ------------------------------------------------------------ pass 2: dK, dV
template <typename T>
__global__ __launch_bounds__(kThreads, 2) void bwd_dkv_kernel(const BwdArgs a) {
  __shared__ __align__(16) uint16_t sQ[kBlockKeys * kLdsRow];
  __shared__ __align__(16) uint16_t sG[kBlockKeys * kLdsRow];  // dO
  __shared__ __align__(16) float sLse[kBlockKeys];             // LSE * log2(e); +inf on pad rows
  __shared__ __align__(16) float sD[kBlockKeys];

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int g = lane >> 5, ln = lane & 31, lane16 = lane & 15, half16 = (lane >> 4) & 1;
  const int heads = a.pb.heads;
  const int n_items = *a.pb.n_tiles * heads;
  const float c2 = a.pb.scale * kLog2e;

  for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
    const int head = item % heads;
    const TileItem ti = a.pb.tiles[item / heads];
    const int r0 = a.pb.cu[ti.seq];
    const int len = a.pb.cu[ti.seq + 1] - r0;
    int nk = a.pb.seqused ? min(a.pb.seqused[ti.seq], len) : len;
    nk = nk < 0 ? 0 : nk;
    const int krow = ti.row0 + 32 * wave + ln;       // this lane's key, within the sequence
    const bool wave_on = ti.row0 + 32 * wave < nk;   // wavefront owns at least one live key
    const bool tile_on = ti.row0 < nk;               // uniform over the workgroup
    const bool key_on = krow < nk;
    const uint16_t* qbase = a.q + (int64_t)r0 * a.q_stride + head * kHeadDim;
    const uint16_t* gbase = a.d_o + (int64_t)r0 * a.do_stride + head * kHeadDim;
    const float* lsebase = a.lse + (int64_t)head * a.pb.total_tokens + r0;
    const float* dbase = a.dsum + (int64_t)head * a.pb.total_tokens + r0;

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
    }

    f32x16 dk[2], dv[2];  // dK^T, dV^T: column = key ln, rows = channels
#pragma unroll
    for (int cb = 0; cb < 2; cb++)
#pragma unroll
      for (int r = 0; r < 16; r++) dk[cb][r] = dv[cb][r] = 0.f;

    const int n_qt = tile_on ? (len + kBlockKeys - 1) / kBlockKeys : 0;
    u32x4 qreg[2], greg[2];
    float lreg = 0.f, dreg = 0.f;
    auto load_stats = [&](int q0) {
      if (tid < kBlockKeys) {
        const int r = q0 + tid;
        lreg = r < len ? lsebase[r] * kLog2e : INFINITY;
        dreg = r < len ? dbase[r] : 0.f;
      }
    };
    auto store_stats = [&]() {
      if (tid < kBlockKeys) {
        sLse[tid] = lreg;
        sD[tid] = dreg;
      }
    };
    if (n_qt > 0) {
      load_tile_regs(qbase, a.q_stride, 0, len, tid, qreg);
      load_tile_regs(gbase, a.do_stride, 0, len, tid, greg);
      load_stats(0);
      store_tile_lds(sQ, tid, qreg);
      store_tile_lds(sG, tid, greg);
      store_stats();
    }
    __syncthreads();

    for (int qt = 0; qt < n_qt; qt++) {
      const bool more = qt + 1 < n_qt;
      if (more) {
        load_tile_regs(qbase, a.q_stride, (qt + 1) * kBlockKeys, len, tid, qreg);
        load_tile_regs(gbase, a.do_stride, (qt + 1) * kBlockKeys, len, tid, greg);
        load_stats((qt + 1) * kBlockKeys);
      }
      if (wave_on) {
#pragma unroll
        for (int qb = 0; qb < 2; qb++) {
          // S = Q K^T, dP = dO V^T : rows = queries (32), column = key ln
          f32x16 s, dp;
#pragma unroll
          for (int r = 0; r < 16; r++) s[r] = dp[r] = 0.f;
#pragma unroll
          for (int t = 0; t < 4; t++) {
            s = Op<T>::mfma(pad_read_row8(sQ, 32 * qb + ln, 16 * t + 8 * g), kb4[t], s);
            dp = Op<T>::mfma(pad_read_row8(sG, 32 * qb + ln, 16 * t + 8 * g), vb4[t], dp);
          }
          float p[16], ds[16];
#pragma unroll
          for (int j = 0; j < 4; j++) {
            // rows 32qb + 8j + 4g + {0..3}: their statistics sit side by side in LDS
            const float4 l4 = *reinterpret_cast<const float4*>(&sLse[32 * qb + 8 * j + 4 * g]);
            const float4 d4 = *reinterpret_cast<const float4*>(&sD[32 * qb + 8 * j + 4 * g]);
            const float lv[4] = {l4.x, l4.y, l4.z, l4.w};
            const float dvv[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
            for (int e = 0; e < 4; e++) {
              float pe = fast_exp2(s[4 * j + e] * c2 - lv[e]);  // pad rows: exp2(-inf) = 0
              pe = key_on ? pe : 0.f;
              p[4 * j + e] = pe;
              ds[4 * j + e] = pe * (dp[4 * j + e] - dvv[e]);
            }
          }
          // dV^T += dO^T P, dK^T += Q^T dS : rows = channels, contraction over queries
#pragma unroll
          for (int t2 = 0; t2 < 2; t2++) {
            const u32x4 pb = {Op<T>::pack2(p[8 * t2 + 0], p[8 * t2 + 1]),
                              Op<T>::pack2(p[8 * t2 + 2], p[8 * t2 + 3]),
                              Op<T>::pack2(p[8 * t2 + 4], p[8 * t2 + 5]),
                              Op<T>::pack2(p[8 * t2 + 6], p[8 * t2 + 7])};
            const u32x4 dsb = {Op<T>::pack2(ds[8 * t2 + 0], ds[8 * t2 + 1]),
                               Op<T>::pack2(ds[8 * t2 + 2], ds[8 * t2 + 3]),
                               Op<T>::pack2(ds[8 * t2 + 4], ds[8 * t2 + 5]),
                               Op<T>::pack2(ds[8 * t2 + 6], ds[8 * t2 + 7])};
#pragma unroll
            for (int cb = 0; cb < 2; cb++) {
              const int base = 32 * qb + 16 * t2 + 4 * g, col = 32 * cb + 16 * half16;
              dv[cb] = Op<T>::mfma(pad_read_col8(sG, base, col, lane16), pb, dv[cb]);
              dk[cb] = Op<T>::mfma(pad_read_col8(sQ, base, col, lane16), dsb, dk[cb]);
            }
          }
        }
      }
      __syncthreads();
      if (more) {
        store_tile_lds(sQ, tid, qreg);
        store_tile_lds(sG, tid, greg);
        store_stats();
      }
      __syncthreads();
    }

    // every row of the tile is written: live keys get their gradients, keys
    // masked by seqused get zeros (their accumulators never left zero)
    if (krow < len) {
      const float sc = a.pb.scale;
      const int64_t tok = r0 + krow;
      uint16_t* kp = a.dk + tok * a.dk_stride + head * kHeadDim + 4 * g;
      uint16_t* vp = a.dv + tok * a.dv_stride + head * kHeadDim + 4 * g;
#pragma unroll
      for (int cb = 0; cb < 2; cb++)
#pragma unroll
        for (int j = 0; j < 4; j++) {
          u32x2 wk = {Op<T>::pack2(dk[cb][4 * j] * sc, dk[cb][4 * j + 1] * sc),
                      Op<T>::pack2(dk[cb][4 * j + 2] * sc, dk[cb][4 * j + 3] * sc)};
          u32x2 wv = {Op<T>::pack2(dv[cb][4 * j], dv[cb][4 * j + 1]),
                      Op<T>::pack2(dv[cb][4 * j + 2], dv[cb][4 * j + 3])};
          *reinterpret_cast<u32x2*>(kp + 32 * cb + 8 * j) = wk;
          *reinterpret_cast<u32x2*>(vp + 32 * cb + 8 * j) = wv;
        }
    }
  }
}

}  // namespace fmha
