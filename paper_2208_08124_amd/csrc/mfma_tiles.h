// Device-side building blocks for gfx950 (CDNA4): 16-bit operand types, the
// 32x32x16 MFMA, LDS transpose reads, wave-half exchange, packing.
//
// Register layouts of v_mfma_f32_32x32x16_{f16,bf16} used throughout
// (lane = 0..63, ln = lane % 32, g = lane / 32):
//   A (32 x 16): lane holds row ln,    contraction slots 8g .. 8g+7
//   B (16 x 32): lane holds column ln, contraction slots 8g .. 8g+7
//   C (32 x 32): lane holds column ln; register r (0..15) is row
//                8*(r/4) + 4g + (r%4)
// The contraction index may be permuted freely as long as A and B agree, which
// is what lets a C tile be fed straight back in as a B operand: registers
// 8t..8t+7 of a C tile are "rows" 16t + {4g..4g+3, 8+4g..8+4g+3}, so the
// matching A operand has to carry those same rows in its eight slots.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fmha {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((__vector_size__(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

template <typename T>
struct Op;

template <>
struct Op<_Float16> {
  static __device__ __forceinline__ f32x16 mfma(u32x4 a, u32x4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a),
                                                  __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  }
  // two fp32 -> two halves in one dword, round to nearest even
  static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    h2 v = {(_Float16)lo, (_Float16)hi};
    return __builtin_bit_cast(uint32_t, v);
  }
  static __device__ __forceinline__ float lo(uint32_t w) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    return (float)__builtin_bit_cast(h2, w)[0];
  }
  static __device__ __forceinline__ float hi(uint32_t w) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    return (float)__builtin_bit_cast(h2, w)[1];
  }
};

template <>
struct Op<__bf16> {
  static __device__ __forceinline__ f32x16 mfma(u32x4 a, u32x4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    typedef __bf16 b2 __attribute__((ext_vector_type(2)));
    b2 v = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(uint32_t, v);
  }
  static __device__ __forceinline__ float lo(uint32_t w) {
    return __builtin_bit_cast(float, w << 16);
  }
  static __device__ __forceinline__ float hi(uint32_t w) {
    return __builtin_bit_cast(float, w & 0xffff0000u);
  }
};

// LDS transpose read (ds_read_b64_tr_b16).  Within each group of 16 lanes,
// lane i supplies the address of four consecutive 16-bit elements; seen as a
// 4 x 16 matrix M whose row e is supplied by lanes 4e..4e+3 (four elements
// each), lane j receives column j: M[0][j], M[1][j], M[2][j], M[3][j].
static __device__ __forceinline__ u32x2 lds_read_tr16(const uint16_t* p) {
  s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (s16x4 __attribute__((address_space(3)))*)(p));
  return __builtin_bit_cast(u32x2, v);
}

// Value held by the lane 32 away (v_permlane32_swap).
static __device__ __forceinline__ float other_half(float x) {
  uint32_t u = __builtin_bit_cast(uint32_t, x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  // lanes 0..31 see (own, partner); lanes 32..63 see (partner, own)
  uint32_t partner = (threadIdx.x & 32) ? r[0] : r[1];
  return __builtin_bit_cast(float, partner);
}

static __device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Row stride (in 16-bit elements) of a 64-wide tile in LDS: 64 + 8 keeps both
// the 16-byte row reads of 32 consecutive rows and the transpose reads spread
// over the banks.
constexpr int kLdsRow = 72;

// A operand from a row-major LDS tile: row `row`, elements col .. col+7.
static __device__ __forceinline__ u32x4 lds_read_row8(const uint16_t* tile, int row, int col) {
  return *reinterpret_cast<const u32x4*>(tile + row * kLdsRow + col);
}

// A operand for a contraction over the tile's ROWS: the lane gets, for column
// `col`, rows base+{0..3} and base+8+{0..3}.  `lane16 = lane % 16` picks the
// address this lane contributes; `col16` is the first of the 16 columns its
// 16-lane group covers.
static __device__ __forceinline__ u32x4 lds_read_col8(const uint16_t* tile, int base, int col16,
                                                      int lane16) {
  const uint16_t* p = tile + (base + (lane16 >> 2)) * kLdsRow + col16 + 4 * (lane16 & 3);
  u32x2 a = lds_read_tr16(p);
  u32x2 b = lds_read_tr16(p + 8 * kLdsRow);
  return u32x4{a[0], a[1], b[0], b[1]};
}

}  // namespace fmha
