// gfx950 building blocks shared by the bf16 forward and backward kernels:
// MFMA wrappers and operand layouts, LDS transpose reads, bf16 packing, tile staging.
//
// v_mfma_f32_32x32x16_bf16 (one wavefront, lane l, half g = l / 32, r = l % 32):
//   A (32 x 16): lane holds row r,    k = 8g .. 8g+7   (8 bf16)
//   B (16 x 32): lane holds column r, k = 8g .. 8g+7   (8 bf16)
//   C (32 x 32): lane holds column r, rows 8*(v/4) + 4g + v%4 for v = 0..15 (16 fp32)
// The k order inside a contraction is free as long as A and B agree, which lets a C-layout
// tile be fed back as a B operand without any cross-lane movement (see pack_c_as_b).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace st {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2;

#define ST_LDS __attribute__((address_space(3)))

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// fp32 pair -> packed bf16 pair, round to nearest even (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  f32x2 f = {lo, hi};
  bf16x2 h = __builtin_convertvector(f, bf16x2);
  return __builtin_bit_cast(uint32_t, h);
}

// Eight consecutive C-layout values (v = 8m .. 8m+7) as a B (or A) operand.
// Slot e of the operand then stands for row 16m + 8*(e/4) + 4g + e%4 of the C tile.
__device__ __forceinline__ bf16x8 pack_c_as_b(const f32x16& c, int m) {
  u32x4 u;
  u[0] = pack_bf16(c[8 * m + 0], c[8 * m + 1]);
  u[1] = pack_bf16(c[8 * m + 2], c[8 * m + 3]);
  u[2] = pack_bf16(c[8 * m + 4], c[8 * m + 5]);
  u[3] = pack_bf16(c[8 * m + 6], c[8 * m + 7]);
  return __builtin_bit_cast(bf16x8, u);
}

// ds_read_b64_tr_b16: inside each group of 16 lanes, lane i receives element (i % 4) of the four
// 8-byte rows addressed by lanes i/4, i/4 + 4, i/4 + 8, i/4 + 12 of its group.
__device__ __forceinline__ u32x2 lds_read_tr16(const ST_LDS char* p) {
  s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((ST_LDS s16x4*)p);
  return __builtin_bit_cast(u32x2, r);
}

__device__ __forceinline__ bf16x8 lds_read_b128(const ST_LDS char* p) {
  return *reinterpret_cast<const ST_LDS bf16x8*>(p);
}

// A-operand fragment of X^T for a row-major LDS tile X[row][col] (cols contiguous):
// the lane gets column (col0 + l % 32) at the eight rows
//   row0 + 4g + {0,1,2,3}  and  row0 + 8 + 4g + {0,1,2,3},
// which is exactly the slot order pack_c_as_b produces for C rows 16m .. 16m+15 (row0 = 16m).
// lane_off = byte offset of this lane's source row/col inside such a fragment (see tr_lane_offset).
__device__ __forceinline__ bf16x8 lds_read_tr_frag(const ST_LDS char* tile, int row0, int col0, int stride,
                                                   int lane_off) {
  const ST_LDS char* p = tile + row0 * stride + col0 * 2 + lane_off;
  u32x2 lo = lds_read_tr16(p);
  u32x2 hi = lds_read_tr16(p + 8 * stride);
  u32x4 u = {lo[0], lo[1], hi[0], hi[1]};
  return __builtin_bit_cast(bf16x8, u);
}

// source address of lane l inside a transposed fragment: row 4g + (l%16)/4, col 16*((l/16)%2) + 4*(l%4)
__device__ __forceinline__ int tr_lane_offset(int lane, int stride) {
  const int g = lane >> 5, s = lane & 15, half = (lane >> 4) & 1;
  return (4 * g + (s >> 2)) * stride + (16 * half + 4 * (s & 3)) * 2;
}

// ---- XOR-swizzled LDS tiles -------------------------------------------------------------------
// A tile of ROWS x D bf16 is stored row-major without padding (D*2 bytes per row) in 16-byte
// chunks; chunk c of row r lives at chunk position c ^ f(r).  f is chosen so that both access
// patterns of the MFMA operands are bank-conflict free:
//   * 16-byte reads of one chunk column by 16 consecutive rows (A/B operand, k along D)
//   * transpose reads of 4 consecutive rows x 64 contiguous bytes (A operand of the transposed tile)
template <int D>
__device__ __forceinline__ int swz(int row, int chunk) {
  const int f = (D == 128) ? (((row & 3) << 2) | ((row >> 2) & 3)) : ((((row >> 1) & 1) << 2) | ((row >> 2) & 3));
  return row * (D * 2) + ((chunk ^ f) << 4);
}

// operand fragment with k along D: row (row0 + l % 32), elements 16 ks + 8 g .. + 7
template <int D>
__device__ __forceinline__ bf16x8 lds_frag(const ST_LDS char* tile, int row0, int ks, int lane) {
  return lds_read_b128(tile + swz<D>(row0 + (lane & 31), 2 * ks + (lane >> 5)));
}

// A-operand fragment of the TRANSPOSED tile: column (col0 + l % 32) at rows
// row0 + 4g + {0..3} and row0 + 8 + 4g + {0..3} (the slot order of pack_c_as_b); row0 % 16 == 0, col0 % 32 == 0
template <int D>
__device__ __forceinline__ bf16x8 lds_frag_tr(const ST_LDS char* tile, int row0, int col0, int lane) {
  const int g = lane >> 5, s = lane & 15, half = (lane >> 4) & 1;
  const int row = row0 + 4 * g + (s >> 2);
  const int chunk = col0 / 8 + 2 * half + ((s & 3) >> 1);
  const int sub = (s & 1) * 8;
  u32x2 lo = lds_read_tr16(tile + swz<D>(row, chunk) + sub);
  u32x2 hi = lds_read_tr16(tile + swz<D>(row + 8, chunk) + sub);
  u32x4 u = {lo[0], lo[1], hi[0], hi[1]};
  return __builtin_bit_cast(bf16x8, u);
}

// global -> registers -> swizzled LDS staging of a ROWS x D bf16 tile by 256 threads.
// Rows at or beyond row_limit read as zero (no out-of-bounds access).
template <int D, int ROWS>
struct StageRegs {
  static constexpr int kN = ROWS * (D / 8) / 256;
  static_assert(kN >= 1 && ROWS * (D / 8) % 256 == 0, "tile must split evenly over 256 threads");
  u32x4 x[kN];
};

template <int D, int ROWS>
__device__ __forceinline__ void stage_load(StageRegs<D, ROWS>& r, const char* base, int64_t row_stride_elems,
                                           int row0, int row_limit, int tid) {
  constexpr int PPR = D / 8;
#pragma unroll
  for (int j = 0; j < StageRegs<D, ROWS>::kN; ++j) {
    const int p = tid + 256 * j;
    const int row = p / PPR, chunk = p % PPR;
    if (row0 + row < row_limit)
      r.x[j] = *reinterpret_cast<const u32x4*>(base + ((int64_t)(row0 + row) * row_stride_elems + chunk * 8) * 2);
    else
      r.x[j] = u32x4{0, 0, 0, 0};
  }
}

template <int D, int ROWS>
__device__ __forceinline__ void stage_store(const StageRegs<D, ROWS>& r, ST_LDS char* tile, int tid) {
  constexpr int PPR = D / 8;
#pragma unroll
  for (int j = 0; j < StageRegs<D, ROWS>::kN; ++j) {
    const int p = tid + 256 * j;
    *reinterpret_cast<ST_LDS u32x4*>(tile + swz<D>(p / PPR, p % PPR)) = r.x[j];
  }
}

// Direct global -> LDS staging (no staging registers, no LDS write instructions): one wavefront-wide
// global_load_lds_dwordx4 moves 64 x 16 bytes to 1 KiB of consecutive LDS, lane L to byte 16 L.  The
// swizzle is therefore applied on the global side: the lane that fills chunk position pc of a row
// fetches chunk pc ^ f(row).  Rows at or beyond row_limit (>= 1) re-read row row_limit - 1; every
// consumer masks such rows, so only finiteness of their contents matters.  The caller must wait
// (s_waitcnt vmcnt(0), which the compiler places before the workgroup barrier) before reading.
typedef __attribute__((address_space(1))) const void* st_global_ptr;
typedef __attribute__((address_space(3))) void* st_lds_ptr;

template <int D, int ROWS>
__device__ __forceinline__ void stage_dma(const char* base, int64_t row_stride_elems, int row0, int row_limit,
                                          ST_LDS char* tile, int tid) {
  constexpr int PPR = D / 8;                 // 16-byte chunks per row
  constexpr int RPI = 64 / PPR;              // rows per instruction
  constexpr int PER_WAVE = ROWS / RPI / 4;   // instructions per wavefront (4 wavefronts)
  static_assert(ROWS % (RPI * 4) == 0, "tile must split evenly over 4 wavefronts");
  const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
  for (int j = 0; j < PER_WAVE; ++j) {
    const int instr = j * 4 + wave;
    const int row = instr * RPI + lane / PPR;
    const int pc = lane % PPR;
    const int f = (D == 128) ? (((row & 3) << 2) | ((row >> 2) & 3)) : ((((row >> 1) & 1) << 2) | ((row >> 2) & 3));
    int grow = row0 + row;
    grow = grow < row_limit ? grow : row_limit - 1;
    const char* src = base + ((int64_t)grow * row_stride_elems + (pc ^ f) * 8) * 2;
    __builtin_amdgcn_global_load_lds((st_global_ptr)src, (st_lds_ptr)(tile + instr * 1024), 16, 0, 0);
  }
}

// operand fragment straight from global memory: row `row` (zero if row >= row_limit), elements 16 ks + 8 g .. + 7
__device__ __forceinline__ bf16x8 global_frag(const char* base, int64_t row_stride_elems, int row, int row_limit,
                                              int ks, int g) {
  if (row < row_limit)
    return *reinterpret_cast<const bf16x8*>(base + ((int64_t)row * row_stride_elems + 16 * ks + 8 * g) * 2);
  return __builtin_bit_cast(bf16x8, u32x4{0, 0, 0, 0});
}

// x *= a in ONE asm statement with all sixteen registers tied in place.  Used on rarely taken
// paths (accumulator rescale): written as plain C++ the product gets a fresh register tuple and the
// path that skips the multiply has to copy the whole accumulator.
__device__ __forceinline__ void scale_in_place(f32x16& x, float a) {
  float x0 = x[0], x1 = x[1], x2 = x[2], x3 = x[3], x4 = x[4], x5 = x[5], x6 = x[6], x7 = x[7];
  float x8 = x[8], x9 = x[9], xa = x[10], xb = x[11], xc = x[12], xd = x[13], xe = x[14], xf = x[15];
  // the leading s_nop covers the wait states a transcendental result (a) needs before a VALU use;
  // the compiler does not insert them for operands of an asm statement
  asm volatile(
      "s_nop 4\n\t"
      "v_mul_f32 %0, %16, %0\n\tv_mul_f32 %1, %16, %1\n\tv_mul_f32 %2, %16, %2\n\tv_mul_f32 %3, %16, %3\n\t"
      "v_mul_f32 %4, %16, %4\n\tv_mul_f32 %5, %16, %5\n\tv_mul_f32 %6, %16, %6\n\tv_mul_f32 %7, %16, %7\n\t"
      "v_mul_f32 %8, %16, %8\n\tv_mul_f32 %9, %16, %9\n\tv_mul_f32 %10, %16, %10\n\tv_mul_f32 %11, %16, %11\n\t"
      "v_mul_f32 %12, %16, %12\n\tv_mul_f32 %13, %16, %13\n\tv_mul_f32 %14, %16, %14\n\tv_mul_f32 %15, %16, %15"
      : "+v"(x0), "+v"(x1), "+v"(x2), "+v"(x3), "+v"(x4), "+v"(x5), "+v"(x6), "+v"(x7), "+v"(x8), "+v"(x9),
        "+v"(xa), "+v"(xb), "+v"(xc), "+v"(xd), "+v"(xe), "+v"(xf)
      : "v"(a));
  x = f32x16{x0, x1, x2, x3, x4, x5, x6, x7, x8, x9, xa, xb, xc, xd, xe, xf};
}

__device__ __forceinline__ float xhalf_max(float x) { return fmaxf(x, __shfl_xor(x, 32)); }
__device__ __forceinline__ float xhalf_sum(float x) { return x + __shfl_xor(x, 32); }

// XCD-aware block order: consecutive hardware block ids land on different XCDs (8 of them, each with
// its own L2), so give every XCD a contiguous range of logical tiles.
__device__ __forceinline__ int xcd_logical_block(int id, int total) {
  return (total % 8 == 0) ? (id % 8) * (total / 8) + id / 8 : id;
}

}  // namespace st
