// Forward kernel: O = softmax(scale Q K^T) V on packed rows (Eq. 1 of the
// paper, one sequence and head at a time), fused in one pass over the keys
// with a running row maximum and row sum.
//
// One workgroup (4 wavefronts) takes one tile of 128 query rows of one
// (sequence, head); wavefront w owns rows 32w..32w+31.  Keys and values are
// staged 64 rows at a time in LDS.  The scores are produced TRANSPOSED,
// S^T = K Q^T, so that in the MFMA result layout every lane holds 16 keys of
// ONE query: the row maximum and row sum are then plain per-lane reductions
// plus a single exchange with the lane 32 away, and the probabilities are
// already in the operand layout of the second product O^T = V^T P^T.
#pragma once
#include "kernel_args.h"
#include "mfma_tiles.h"

namespace fmha {

// Stage rows [row0, row0+64) x 64 columns of a packed tensor into registers:
// thread t carries 16-byte chunks t and t+256 (chunk c = row c/8, columns
// 8*(c%8)..+7).  Rows at or beyond `nrows` come back as zeros.
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

template <typename T>
__global__ __launch_bounds__(kThreads, 2) void fmha_fwd_kernel(const FwdArgs a) {
  __shared__ __align__(16) uint16_t sK[kBlockKeys * kLdsRow];
  __shared__ __align__(16) uint16_t sV[kBlockKeys * kLdsRow];

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int g = lane >> 5, ln = lane & 31, lane16 = lane & 15, half16 = (lane >> 4) & 1;
  const int heads = a.pb.heads;
  const int n_items = *a.pb.n_tiles * heads;
  const float c2 = a.pb.scale * kLog2e;  // scores are kept in the log2 domain

  for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
    const int head = item % heads;
    const TileItem ti = a.pb.tiles[item / heads];
    const int r0 = a.pb.cu[ti.seq];
    const int len = a.pb.cu[ti.seq + 1] - r0;
    int nk = a.pb.seqused ? min(a.pb.seqused[ti.seq], len) : len;
    nk = nk < 0 ? 0 : nk;
    const int qrow = ti.row0 + 32 * wave + ln;        // this lane's query, within the sequence
    const bool wave_on = ti.row0 + 32 * wave < len;   // wavefront has at least one valid row
    const uint16_t* kbase = a.k + (int64_t)r0 * a.k_stride + head * kHeadDim;
    const uint16_t* vbase = a.v + (int64_t)r0 * a.v_stride + head * kHeadDim;

    // Q^T as the B operand: column = query ln, slots = channels 16t + 8g .. +7
    u32x4 qb[4];
    {
      const int qr = qrow < len ? qrow : len - 1;
      const uint16_t* qp = a.q + (int64_t)(r0 + qr) * a.q_stride + head * kHeadDim + 8 * g;
#pragma unroll
      for (int t = 0; t < 4; t++) qb[t] = *reinterpret_cast<const u32x4*>(qp + 16 * t);
    }

    f32x16 oacc[2];  // O^T: column = query ln; oacc[cb][r] is channel 32cb + 8(r/4) + 4g + r%4
#pragma unroll
    for (int cb = 0; cb < 2; cb++)
#pragma unroll
      for (int r = 0; r < 16; r++) oacc[cb][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

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
      if (more) {  // next tile's global loads fly while this one is computed
        load_tile_regs(kbase, a.k_stride, (kt + 1) * kBlockKeys, nk, tid, kreg);
        load_tile_regs(vbase, a.v_stride, (kt + 1) * kBlockKeys, nk, tid, vreg);
      }
      if (wave_on) {
        // S^T = K Q^T : rows = keys (two blocks of 32), column = query ln
        f32x16 s[2];
#pragma unroll
        for (int kb = 0; kb < 2; kb++) {
#pragma unroll
          for (int r = 0; r < 16; r++) s[kb][r] = 0.f;
#pragma unroll
          for (int t = 0; t < 4; t++)
            s[kb] = Op<T>::mfma(lds_read_row8(sK, 32 * kb + ln, 16 * t + 8 * g), qb[t], s[kb]);
        }
        // scale into the log2 domain, mask keys past the end (last tile only)
        const int key0 = kt * kBlockKeys + 4 * g;
        const bool ragged = key0 - 4 * g + kBlockKeys > nk;
        float mx = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < 2; kb++)
#pragma unroll
          for (int r = 0; r < 16; r++) {
            float x = s[kb][r] * c2;
            if (ragged && key0 + 32 * kb + 8 * (r >> 2) + (r & 3) >= nk) x = -INFINITY;
            s[kb][r] = x;
            mx = fmaxf(mx, x);
          }
        mx = fmaxf(mx, other_half(mx));
        const float m_new = fmaxf(m_run, mx);  // finite: every staged tile has a valid key
        const float alpha = fast_exp2(m_run - m_new);
        m_run = m_new;
        float psum = 0.f;
        u32x4 pb[2][2];  // P^T as B operands: [key block][16-key step]
#pragma unroll
        for (int kb = 0; kb < 2; kb++) {
          float p[16];
#pragma unroll
          for (int r = 0; r < 16; r++) {
            p[r] = fast_exp2(s[kb][r] - m_new);
            psum += p[r];
          }
#pragma unroll
          for (int t2 = 0; t2 < 2; t2++)
            pb[kb][t2] = u32x4{Op<T>::pack2(p[8 * t2 + 0], p[8 * t2 + 1]),
                               Op<T>::pack2(p[8 * t2 + 2], p[8 * t2 + 3]),
                               Op<T>::pack2(p[8 * t2 + 4], p[8 * t2 + 5]),
                               Op<T>::pack2(p[8 * t2 + 6], p[8 * t2 + 7])};
        }
        l_run = l_run * alpha + psum;
#pragma unroll
        for (int cb = 0; cb < 2; cb++)
#pragma unroll
          for (int r = 0; r < 16; r++) oacc[cb][r] *= alpha;
        // O^T += V^T P^T : rows = channels (two blocks of 32), contraction over keys
#pragma unroll
        for (int cb = 0; cb < 2; cb++)
#pragma unroll
          for (int kb = 0; kb < 2; kb++)
#pragma unroll
            for (int t2 = 0; t2 < 2; t2++)
              oacc[cb] = Op<T>::mfma(
                  lds_read_col8(sV, 32 * kb + 16 * t2 + 4 * g, 32 * cb + 16 * half16, lane16),
                  pb[kb][t2], oacc[cb]);
      }
      __syncthreads();
      if (more) {
        store_tile_lds(sK, tid, kreg);
        store_tile_lds(sV, tid, vreg);
      }
      __syncthreads();
    }

    // epilogue: combine the two half-rows' sums, normalise, store O and LSE
    if (wave_on) {
      const float l_tot = l_run + other_half(l_run);
      const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
      if (qrow < len) {
        uint16_t* op = a.o + (int64_t)(r0 + qrow) * a.o_stride + head * kHeadDim + 4 * g;
#pragma unroll
        for (int cb = 0; cb < 2; cb++)
#pragma unroll
          for (int j = 0; j < 4; j++) {
            u32x2 w = {Op<T>::pack2(oacc[cb][4 * j] * inv, oacc[cb][4 * j + 1] * inv),
                       Op<T>::pack2(oacc[cb][4 * j + 2] * inv, oacc[cb][4 * j + 3] * inv)};
            *reinterpret_cast<u32x2*>(op + 32 * cb + 8 * j) = w;
          }
        if (g == 0)
          a.lse[(int64_t)head * a.pb.total_tokens + r0 + qrow] =
              l_tot > 0.f ? (m_run + __builtin_amdgcn_logf(l_tot)) * kLn2 : -INFINITY;
      }
    }
  }
}

}  // namespace fmha
