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
typedef float f32x4 __attribute__((ext_vector_type(4)));
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
  // acc + (both halves of w), accumulated in fp32 (v_dot2c_f32_f16 with a vector of ones)
  static __device__ __forceinline__ float add_pair(uint32_t w, float acc) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(h2, w), h2{(_Float16)1.f, (_Float16)1.f}, acc,
                                  false);
  }
  // acc + a.lo * b.lo + a.hi * b.hi in fp32 (v_dot2c_f32_f16)
  static __device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float acc) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(h2, a), __builtin_bit_cast(h2, b), acc, false);
  }
  // Every element of acc + the sum of this lane's four 16-bit values in w, on the matrix core:
  // v_mfma_f32_4x4x4_16b with an A operand of ones gives D[i][j] = C[i][j] + sum_k B[k][j],
  // and a lane holds all four k of its column j whatever the block arrangement.  (Row sums
  // this way cost 8 cycles of the matrix pipe per four values and none of the vector ALU.)
  static __device__ __forceinline__ f32x4 sum4(u32x2 w, f32x4 acc) {
    typedef _Float16 h4 __attribute__((ext_vector_type(4)));
    const u32x2 ones = {0x3c003c00u, 0x3c003c00u};
    return __builtin_amdgcn_mfma_f32_4x4x4f16(__builtin_bit_cast(h4, ones), __builtin_bit_cast(h4, w), acc, 0, 0, 0);
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
  static __device__ __forceinline__ float add_pair(uint32_t w, float acc) {
    typedef __bf16 b2 __attribute__((ext_vector_type(2)));
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(b2, w), b2{(__bf16)1.f, (__bf16)1.f},
                                           acc, false);
  }
  static __device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float acc) {
    typedef __bf16 b2 __attribute__((ext_vector_type(2)));
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(b2, a), __builtin_bit_cast(b2, b), acc, false);
  }
  static __device__ __forceinline__ f32x4 sum4(u32x2 w, f32x4 acc) {
    typedef short s4 __attribute__((ext_vector_type(4)));
    const u32x2 ones = {0x3f803f80u, 0x3f803f80u};
    return __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(__builtin_bit_cast(s4, ones), __builtin_bit_cast(s4, w), acc, 0, 0, 0);
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

// ---------------------------------------------------------------------------
// 64 x 64 tiles of 16-bit elements in LDS: 8 KB, rows of 128 bytes, no padding.
// The 16-byte chunk c (0..7) of row r is stored at chunk position c ^ swz(r).
// With 64 four-byte banks a row covers half of them (which half = parity of
// r), so the swizzle is a bijection of (r/2) mod 8 - sixteen consecutive rows
// read at one column hit every bank once - and it moves bit 0 of r/2 to bit 2,
// so that the four consecutive rows of a transpose read, each reading four
// neighbouring chunks, land in different chunk groups.  Measured on MI355X:
// ~226 B/clk/CU for the 16-byte row reads and ~200 B/clk/CU for the transpose
// reads below, against 32 and 117 without a swizzle.
// ---------------------------------------------------------------------------
constexpr int kTileElems = 64 * 64;

static __device__ __forceinline__ int swz(int r) {
  const int x = (r >> 1) & 7;
  return ((x & 1) << 2) | (x >> 1);
}

// element offset of (row, col) inside a tile
static __device__ __forceinline__ int tile_off(int row, int col) {
  return row * 64 + ((((col >> 3) ^ swz(row)) << 3) | (col & 7));
}

// Per-lane offsets of the operand reads, computed once per kernel.  Moving by
// a multiple of 16 rows leaves swz() unchanged, so stepping through a tile only
// adds constants (which the LDS instructions carry as immediates).
//
// RowRead: A (or B) operand whose contraction runs along the tile's COLUMNS:
// the lane reads row ln (+32 per row block), columns 16t + 8g .. +7.
struct RowRead {
  int off[4];
  __device__ __forceinline__ RowRead(int ln, int g) {
#pragma unroll
    for (int t = 0; t < 4; t++) off[t] = tile_off(ln, 16 * t + 8 * g);
  }
  // rows 32*rb + ln, columns 16t + 8g .. +7
  __device__ __forceinline__ u32x4 read(const uint16_t* tile, int rb, int t) const {
    return *reinterpret_cast<const u32x4*>(tile + off[t] + 2048 * rb);
  }
};

// ColRead: A operand whose contraction runs along the tile's ROWS (transpose
// reads): for column 32cb + (lane % 32) the lane gets rows
// 16*step + {4g..4g+3, 8+4g..8+4g+3} - exactly the rows whose values sit in
// registers 8t..8t+7 of a C tile (see the layout note at the top).
struct ColRead {
  int off[2][2];  // [column block][second half of the eight rows]
  __device__ __forceinline__ ColRead(int lane) {
    const int g = lane >> 5, half16 = (lane >> 4) & 1, lane16 = lane & 15;
#pragma unroll
    for (int cb = 0; cb < 2; cb++)
#pragma unroll
      for (int hh = 0; hh < 2; hh++)
        off[cb][hh] = tile_off(4 * g + (lane16 >> 2) + 8 * hh, 32 * cb + 16 * half16 + 4 * (lane16 & 3));
  }
  // rows 16*step + ..., column block cb
  __device__ __forceinline__ u32x4 read(const uint16_t* tile, int step, int cb) const {
    u32x2 a = lds_read_tr16(tile + off[cb][0] + 1024 * step);
    u32x2 b = lds_read_tr16(tile + off[cb][1] + 1024 * step);
    return u32x4{a[0], a[1], b[0], b[1]};
  }
};

// ---------------------------------------------------------------------------
// Global -> LDS without passing through registers (global_load_lds_dwordx4):
// every lane names its own 16 global bytes; the wavefront's 64 pieces land at
// LDS address m0 + 16*lane, i.e. one instruction fills eight tile rows, and the
// swizzle is applied by choosing WHICH global chunk each lane fetches.
// The instruction is issued from inline assembly so that the compiler does
// not serialise every later LDS read behind it; completion is awaited with
// explicit s_waitcnt vmcnt(n) (vector memory loads complete in issue order).
// m0 is not named as a clobber: it is a reserved register to the compiler (which rejects
// it in clobber lists with a warning) - the compiler never keeps a value of its own in m0
// across other instructions, it writes m0 directly ahead of each instruction of its own
// that reads it.
// ---------------------------------------------------------------------------
static __device__ __forceinline__ uint32_t lds_addr(const void* p) {
  return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)p;
}

static __device__ __forceinline__ void dma16(const void* gptr, uint32_t lds_byte_addr) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off"
               :
               : "s"(lds_byte_addr), "v"(gptr)
               : "memory");
}

// Same for 4 bytes per lane: the wavefront's 64 dwords land at m0 + 4*lane.
static __device__ __forceinline__ void dma4(const void* gptr, uint32_t lds_byte_addr) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dword %1, off"
               :
               : "s"(lds_byte_addr), "v"(gptr)
               : "memory");
}

// The same with the address split into a wave-uniform base (scalar registers) and a
// 32-bit byte offset per lane: no 64-bit vector arithmetic per transfer.
static __device__ __forceinline__ void dma16s(const void* sbase, uint32_t voff, uint32_t lds_byte_addr) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_byte_addr), "v"(voff), "s"(sbase)
               : "memory");
}

// An offset the compiler may keep in scalar registers: the value is the same in every lane
// (it depends on the wavefront index at most), which the compiler cannot always see.  Added
// to a kernel-argument pointer it gives a wave-uniform base that still carries the pointer's
// address space (a pointer rebuilt from integers would be accessed with flat instructions).
static __device__ __forceinline__ int64_t uniform_i64(int64_t v) {
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)(uint64_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)v >> 32));
  return (int64_t)(((uint64_t)hi << 32) | lo);
}

template <int N>
static __device__ __forceinline__ void wait_vmem() {
  asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

// Rows and chunk of the two 1 KB pieces a lane moves per 64-row tile: wavefront
// w fills rows 8w..8w+7 and 32+8w..32+8w+7.
struct DmaLane {
  int row;    // first row (second is row + 32)
  int chunk;  // global 16-byte chunk (same for both rows: swz(row) == swz(row + 32))
  __device__ __forceinline__ DmaLane(int wave, int lane) {
    row = 8 * wave + (lane >> 3);
    chunk = (lane & 7) ^ swz(row);
  }
};

// Start moving 64 full rows that begin at `rows` (wave-uniform: first row, this head);
// lane_bytes = byte offset of this lane's chunk within its first row (DmaLane: row * stride +
// chunk * 8 elements), stride in elements.
static __device__ __forceinline__ void dma_tile_full(const uint16_t* rows, uint32_t lane_bytes, int64_t stride,
                                                     int wave, uint32_t tile_addr) {
  const uint32_t m0 = __builtin_amdgcn_readfirstlane(tile_addr + 1024u * wave);
  dma16s(rows, lane_bytes, m0);
  dma16s(rows + 32 * stride, lane_bytes, m0 + 4096u);
}

// Start moving rows [row0, row0 + 64) of a packed tensor (rows clamped to
// last_row, so the tail of a short sequence repeats its last valid row instead
// of reading past it) into the tile at LDS byte address `tile_addr`.
// (row0 <= last_row; the lane offsets are relative to row0, so they fit 32 bits)
static __device__ __forceinline__ void dma_tile(const uint16_t* base, int64_t stride, int row0,
                                                int last_row, const DmaLane& dl, int wave,
                                                uint32_t tile_addr) {
  const int ra = min(dl.row, last_row - row0), rb = min(dl.row + 32, last_row - row0);
  const uint32_t m0 = __builtin_amdgcn_readfirstlane(tile_addr + 1024u * wave);
  const uint16_t* rows = base + uniform_i64(row0 * stride);
  const uint32_t st = (uint32_t)stride;
  dma16s(rows, (ra * st + dl.chunk * 8) * 2u, m0);
  dma16s(rows, (rb * st + dl.chunk * 8) * 2u, m0 + 4096u);
}

// ---------------------------------------------------------------------------
// Rows of a ring stage that belong to one wavefront: with the piece assignment of
// DmaLane, wavefront w is the only one whose fetches write rows 8w..8w+7 and
// 32+8w..32+8w+7 of each of the stage's two tiles - four pieces of 1 KB.  Between
// the end of one work item and the first fetch the same wavefront issues into
// that stage for the next one, those 4 KB are scratch space that needs no
// barrier.  own_piece(i) is the byte offset of piece i from the wavefront's first
// private row (stage base + 1024 * w); `second_tile` is the byte distance between
// the stage's two tiles.
// ---------------------------------------------------------------------------
__device__ __forceinline__ constexpr int own_piece(int i, int second_tile = 8192) {
  return (i >> 1) * second_tile + (i & 1) * 4096;
}

// Issue priority of this wavefront for the coming inner step.  Among wavefronts of
// equal priority a SIMD issues from the oldest one first, so of the workgroups
// that share a compute unit the first-placed one runs ahead and the last-placed
// one is left to finish alone, with nobody to overlap its stalls with.  Rotating
// the priority from step to step - workgroup slot `slot` of `slots` per compute
// unit (launch order: blockIdx / number of compute units) is favoured every
// `slots`-th step - lets them advance side by side (measured: the workgroups'
// finishing times move together, and the kernels end 2-3 % earlier).
__device__ __forceinline__ void rotate_priority(int step, int slot, int slots) {
  const int p = (step + slot) % slots;
  if (p == 0)
    __builtin_amdgcn_s_setprio(0);
  else if (p == 1)
    __builtin_amdgcn_s_setprio(1);
  else
    __builtin_amdgcn_s_setprio(2);
}

// Lane number, recomputed from the execution mask (all 64 lanes active): two
// instructions where it is needed beat a register - and everything the compiler
// would derive from it ahead of time - held through the hot loop.  Volatile, so
// that it stays where it is written.
__device__ __forceinline__ int lane_id() {
  int x;
  asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(x));
  return x;
}

// A wavefront's 32 x 64 result tile, held transposed in MFMA layout (x[cb][r] =
// channel 32cb + 8(r/4) + 4g + r%4 of row ln), scaled, rounded to T and written to
// global memory as whole 128-byte rows (row 0 of the tile is at out_tensor + out_offset, a
// wave-uniform position): the tile is turned around in the
// wavefront's private pieces of `stage` (piece r/8 holds rows 8(r/8)..+7, 16-byte
// chunk c of row r at position c ^ swz(r)), so that each store instruction covers
// 8 complete rows instead of 16 bytes in each of 32.  Rows >= n_rows are not stored.  All 64 lanes must be active.
template <typename T>
__device__ __forceinline__ void store_rows(const f32x16 (&x)[2], float scale, uint16_t* stage, int wave,
                                           uint16_t* out_tensor, int64_t out_offset, int64_t out_stride, int n_rows,
                                           int second_tile = 8192) {
  // lane-derived addresses are computed here rather than kept in registers by the caller
  const int lane = lane_id();
  const int g = lane >> 5, ln = lane & 31;
  uint16_t* so = stage + 512 * wave;
  uint16_t* wr = so + own_piece(ln >> 3, second_tile) / 2 + (ln & 7) * 64 + 4 * g;
  const int sw = swz(ln);
#pragma unroll
  for (int cb = 0; cb < 2; cb++)
#pragma unroll
    for (int j = 0; j < 4; j++) {
      u32x2 w = {Op<T>::pack2(x[cb][4 * j] * scale, x[cb][4 * j + 1] * scale),
                 Op<T>::pack2(x[cb][4 * j + 2] * scale, x[cb][4 * j + 3] * scale)};
      *reinterpret_cast<u32x2*>(wr + (((4 * cb + j) ^ sw) << 3)) = w;
    }
  __builtin_amdgcn_wave_barrier();  // same wavefront: its LDS operations execute in order
  const int chunk = lane & 7;
  // `out` is the same in all lanes: base in scalar registers, 32-bit byte offsets per lane
  char* ob = reinterpret_cast<char*>(out_tensor + uniform_i64(out_offset));
  const uint32_t row_bytes = (uint32_t)out_stride * 2u;
#pragma unroll
  for (int i = 0; i < 4; i++) {
    const int row = 8 * i + (lane >> 3);
    const u32x4 w = *reinterpret_cast<const u32x4*>(so + own_piece(i, second_tile) / 2 + (lane >> 3) * 64 +
                                                    ((chunk ^ swz(row)) << 3));
    if (row < n_rows) *reinterpret_cast<u32x4*>(ob + ((uint32_t)row * row_bytes + 16u * chunk)) = w;
  }
}

// The same through a 4 KB scratch tile that belongs to the calling wavefront alone (32 rows of
// 128 bytes, 16-byte chunk c of row r at position c ^ swz(r)).  The scratch may be reused
// right after the call: the wavefront's LDS operations execute in program order.
template <typename T>
__device__ __forceinline__ void store_rows32(const f32x16 (&x)[2], float scale, uint16_t* scratch,
                                             uint16_t* out_tensor, int64_t out_offset, int64_t out_stride,
                                             int n_rows) {
  const int lane = lane_id();
  const int g = lane >> 5, ln = lane & 31;
  uint16_t* wr = scratch + ln * 64 + 4 * g;
  const int sw = swz(ln);
#pragma unroll
  for (int cb = 0; cb < 2; cb++)
#pragma unroll
    for (int j = 0; j < 4; j++) {
      u32x2 w = {Op<T>::pack2(x[cb][4 * j] * scale, x[cb][4 * j + 1] * scale),
                 Op<T>::pack2(x[cb][4 * j + 2] * scale, x[cb][4 * j + 3] * scale)};
      *reinterpret_cast<u32x2*>(wr + (((4 * cb + j) ^ sw) << 3)) = w;
    }
  __builtin_amdgcn_wave_barrier();
  const int chunk = lane & 7;
  char* ob = reinterpret_cast<char*>(out_tensor + uniform_i64(out_offset));
  const uint32_t row_bytes = (uint32_t)out_stride * 2u;
#pragma unroll
  for (int i = 0; i < 4; i++) {
    const int row = 8 * i + (lane >> 3);
    const u32x4 w = *reinterpret_cast<const u32x4*>(scratch + row * 64 + ((chunk ^ swz(row)) << 3));
    if (row < n_rows) *reinterpret_cast<u32x4*>(ob + ((uint32_t)row * row_bytes + 16u * chunk)) = w;
  }
  __builtin_amdgcn_wave_barrier();
}

}  // namespace fmha
