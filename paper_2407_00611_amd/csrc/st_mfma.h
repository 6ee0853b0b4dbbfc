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

// Eight bf16 values times c, rounded to bf16 again (round to nearest even).  Every bf16 kernel of the path
// evaluates its scores from the SAME exponent operand Q' = bf16(Q * scale * log2 e) (the MFMA then delivers
// exponents in log2 units and no per-score multiply is needed), so forward and backward agree on every score:
// the probabilities the backward recomputes sum to one over a row, whichever kernel computed which tile.
__device__ __forceinline__ u32x4 scale_bf16x8(u32x4 x, float c) {
  u32x4 y;
#pragma unroll
  for (int j = 0; j < 4; ++j)
    y[j] = pack_bf16(__uint_as_float(x[j] << 16) * c, __uint_as_float(x[j] & 0xffff0000u) * c);
  return y;
}
__device__ __forceinline__ bf16x8 scale_bf16x8(bf16x8 x, float c) {
  return __builtin_bit_cast(bf16x8, scale_bf16x8(__builtin_bit_cast(u32x4, x), c));
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

// The same staging with the DMA written as inline asm: the compiler then does not track it, so it
// places no vmcnt wait in front of later LDS reads and several tiles can be in flight; the caller
// waits explicitly (wait_vmcnt<N>: at most N of this wavefront's loads still outstanding).
// (m0 is a reserved register: naming it as a clobber draws a warning, but the surrounding code is compiled C++
// that may use m0 itself, so the statement says what it overwrites)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void dma16_asm(const char* src, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
               :: "s"(lds_addr), "v"(src) : "memory", "m0");
}
#pragma clang diagnostic pop

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

template <int D, int ROWS>
struct DmaPlan {
  static constexpr int PPR = D / 8;                 // 16-byte chunks per row
  static constexpr int RPI = 64 / PPR;              // rows per instruction
  static constexpr int PER_WAVE = ROWS / RPI / 4;   // instructions per wavefront and tile
};

template <int D, int ROWS>
__device__ __forceinline__ void stage_dma_asm(const char* base, int64_t row_stride_elems, int row0, int row_limit,
                                              uint32_t tile_lds_addr, int tid) {
  using P = DmaPlan<D, ROWS>;
  static_assert(ROWS % (P::RPI * 4) == 0, "tile must split evenly over 4 wavefronts");
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
#pragma unroll
  for (int j = 0; j < P::PER_WAVE; ++j) {
    const int instr = j * 4 + wave;
    const int row = instr * P::RPI + lane / P::PPR;
    const int pc = lane % P::PPR;
    const int f = (D == 128) ? (((row & 3) << 2) | ((row >> 2) & 3)) : ((((row >> 1) & 1) << 2) | ((row >> 2) & 3));
    int grow = row0 + row;
    grow = grow < row_limit ? grow : row_limit - 1;
    dma16_asm(base + ((int64_t)grow * row_stride_elems + (pc ^ f) * 8) * 2, tile_lds_addr + instr * 1024);
  }
}

// Rarely taken in-place edits of a whole MFMA accumulator tuple (mask, rescale).  They are single asm
// statements whose only tuple operand is pinned to a[0:15]: with sixteen scalar operands LLVM splits
// the tuple into scalars around the branch and copies the whole accumulator on the path that skips the
// edit; with a VGPR constraint the allocator keeps the accumulator in VGPRs for the whole loop and
// copies it to AGPRs around every MFMA.  The leading wait states cover an MFMA that has just written
// the tuple and a transcendental that has just produced a scalar input: the compiler inserts no hazard
// nops in front of the operands of an asm statement.

// x[v] = (cv(v) < lim) ? x[v] : -inf, cv(v) = 8 (v / 4) + v % 4: the C-layout row offset of element v
// without the lane's 4 g term (the caller folds that and the block base into lim).
__device__ __forceinline__ void mask_rows_in_place(f32x16& x, int lim) {
  f32x16 t = x;
  float t0;
  const float ninf = -INFINITY;
#define ST_MASK1(i, cv)                                                                                     \
  "v_accvgpr_read_b32 %1, a" #i "\n\tv_cmp_gt_i32_e64 vcc, %2, " #cv "\n\ts_nop 1\n\t"                    \
  "v_cndmask_b32_e32 %1, %3, %1, vcc\n\ts_nop 1\n\tv_accvgpr_write_b32 a" #i ", %1\n\t"
  asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 3\n\t"
               ST_MASK1(0, 0) ST_MASK1(1, 1) ST_MASK1(2, 2) ST_MASK1(3, 3) ST_MASK1(4, 8) ST_MASK1(5, 9)
               ST_MASK1(6, 10) ST_MASK1(7, 11) ST_MASK1(8, 16) ST_MASK1(9, 17) ST_MASK1(10, 18) ST_MASK1(11, 19)
               ST_MASK1(12, 24) ST_MASK1(13, 25) ST_MASK1(14, 26) ST_MASK1(15, 27) "s_nop 3"
               : "+{a[0:15]}"(t), "=&v"(t0)
               : "v"(lim), "v"(ninf)
               : "vcc");
#undef ST_MASK1
  x = t;
}

// operand fragment straight from global memory: row `row` (zero if row >= row_limit), elements 16 ks + 8 g .. + 7
__device__ __forceinline__ bf16x8 global_frag(const char* base, int64_t row_stride_elems, int row, int row_limit,
                                              int ks, int g) {
  if (row < row_limit)
    return *reinterpret_cast<const bf16x8*>(base + ((int64_t)row * row_stride_elems + 16 * ks + 8 * g) * 2);
  return __builtin_bit_cast(bf16x8, u32x4{0, 0, 0, 0});
}

// x *= a
__device__ __forceinline__ void scale_in_place(f32x16& x, float a) {
  f32x16 t = x;
  float t0, t1;
#define ST_SC2(i, j)                                                                            \
  "v_accvgpr_read_b32 %1, a" #i "\n\tv_accvgpr_read_b32 %2, a" #j "\n\ts_nop 1\n\t"           \
  "v_mul_f32 %1, %3, %1\n\tv_mul_f32 %2, %3, %2\n\ts_nop 1\n\t"                              \
  "v_accvgpr_write_b32 a" #i ", %1\n\tv_accvgpr_write_b32 a" #j ", %2\n\t"
  asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 3\n\t"
               ST_SC2(0, 1) ST_SC2(2, 3) ST_SC2(4, 5) ST_SC2(6, 7) ST_SC2(8, 9) ST_SC2(10, 11) ST_SC2(12, 13)
               ST_SC2(14, 15) "s_nop 3"
               : "+{a[0:15]}"(t), "=&v"(t0), "=&v"(t1)
               : "v"(a));
#undef ST_SC2
  x = t;
}

__device__ __forceinline__ float xhalf_max(float x) { return fmaxf(x, __shfl_xor(x, 32)); }
__device__ __forceinline__ float xhalf_sum(float x) { return x + __shfl_xor(x, 32); }

// XCD-aware block order: consecutive hardware block ids land on different XCDs (kDispatchXcds of them on the
// MI355X, each with its own L2), so give every XCD a contiguous range of logical tiles.  The count only shapes
// the order in which work is handed out: on a device with another count every tile is still computed exactly
// once, and only L2 locality is lost.
constexpr int kDispatchXcds = 8;
__device__ __forceinline__ int xcd_logical_block(int id, int total) {
  return (total % kDispatchXcds == 0) ? (id % kDispatchXcds) * (total / kDispatchXcds) + id / kDispatchXcds : id;
}

// Block id -> (query tile, head-and-batch index) for the query-stationary kernels.  Every XCD gets a
// contiguous range of heads (their K / V stay in that XCD's L2); inside the range the query tile is the
// slow index and, under a causal mask, runs from the last tile down: later tiles see more keys, and
// handing out the heaviest workgroups first keeps the tail of the launch short.
__device__ __forceinline__ void qtile_block(int id, int total, int n_qt, int causal, int& qt, int& hb) {
  const int n_hb = total / n_qt;
  int qi;
  if (n_hb % kDispatchXcds == 0) {
    const int per = n_hb / kDispatchXcds, j = id / kDispatchXcds;
    hb = (id % kDispatchXcds) * per + j % per;
    qi = j / per;
  } else {
    hb = id % n_hb;
    qi = id / n_hb;
  }
  qt = causal ? n_qt - 1 - qi : qi;
}

}  // namespace st
