// HBM-bound passes: log-sum-exp merge of two partial states, combine of n partial states,
// Delta = rowsum(dO * O),
// fp32 -> storage-dtype casts and the (O = 0, lse = -inf) state fill.
// One 16-byte vector per lane, rows never straddle a lane; grid sized to the data.
#include "st_internal.h"
#include "st_mfma.h"

namespace st {
namespace {

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;   // NaN stays NaN
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return f32_to_bf16_rne(lo) | (f32_to_bf16_rne(hi) << 16);
}
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// ---- merge: thread = up to U float4 of one (b, i, h) row ---------------------------------------
// A row occupies a power-of-two group of lanes; lane `sub` of the group takes the vectors sub, sub + lanes, ...
// of the row, so consecutive lanes read consecutive 16-byte pieces (whole 128-byte lines once the group has
// eight lanes), the row's two lse are read once per U vectors and its weights are computed once.
// The group never straddles a wavefront: every lane of the row has read lse_acc before lane 0 overwrites it.
// Weights: w_acc = exp(lse_acc - lse'), w_part = exp(lse_part - lse'), lse' = max + log(sum).
// A side with lse = -inf gets weight 0 without ever forming (-inf) - (-inf), and its O is not read into the sum.
// U = vectors per thread (1, 2 or 4): all loads of a thread are in flight before its first store.
template <bool kLowp, int U>
__global__ __launch_bounds__(256) void merge_kernel(float* __restrict__ o_acc, float* __restrict__ lse_acc,
                                                    const float* __restrict__ o_part,
                                                    const float* __restrict__ lse_part, int64_t n_rows,
                                                    int32_t Sq, int32_t Hq, int32_t vec_per_row,
                                                    int32_t lane_shift, uint2* __restrict__ o_lowp) {
  const int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t row = tid >> lane_shift;               // (b * Sq + i) * Hq + h
  const int32_t sub = (int32_t)(tid & ((1 << lane_shift) - 1));
  if (row >= n_rows) return;
  const int32_t h = (int32_t)(row % Hq);
  const int64_t bi = row / Hq;
  const int64_t sidx = ((bi / Sq) * Hq + h) * Sq + (bi % Sq);
  const float la = lse_acc[sidx], lp = lse_part[sidx];
  int64_t v[U];
  bool live[U];
  float4 a[U], p[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int32_t vi = sub + (u << lane_shift);
    live[u] = vi < vec_per_row;
    v[u] = row * vec_per_row + (live[u] ? vi : 0);     // a slot beyond the row reads its first vector and stores nothing
    a[u] = reinterpret_cast<const float4*>(o_acc)[v[u]];
    typedef float f32x4_t __attribute__((ext_vector_type(4)));
    const f32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(o_part) + v[u]);   // read once
    p[u] = make_float4(t.x, t.y, t.z, t.w);
  }
  const float m = fmaxf(la, lp);
  float wa = 0.f, wp = 0.f, lnew = -INFINITY;
  if (m != -INFINITY) {
    const float ea = expf(la - m), ep = expf(lp - m);  // exp(-inf) = 0 for an empty side
    const float sum = ea + ep;
    lnew = m + logf(sum);
    const float inv = 1.f / sum;
    wa = ea * inv;
    wp = ep * inv;
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    if (!live[u]) continue;
    // a side whose weight is exactly 0 (an empty state) is left out, so that a non-finite value in its O
    // (never written, or stale) cannot turn the result into NaN; the combine pass does the same
    const float4 za = wa != 0.f ? a[u] : make_float4(0.f, 0.f, 0.f, 0.f);
    const float4 zp = wp != 0.f ? p[u] : make_float4(0.f, 0.f, 0.f, 0.f);
    float4 r;
    r.x = wa * za.x + wp * zp.x;
    r.y = wa * za.y + wp * zp.y;
    r.z = wa * za.z + wp * zp.z;
    r.w = wa * za.w + wp * zp.w;
    reinterpret_cast<float4*>(o_acc)[v[u]] = r;
    if (kLowp) o_lowp[v[u]] = make_uint2(pack_bf16x2(r.x, r.y), pack_bf16x2(r.z, r.w));
  }
  if (sub == 0) lse_acc[sidx] = lnew;
}

// ---- combine: n partial states of the same rows -> one state, keeping a run of rows -----------
// Thread = one float4 of one kept (b, i, h) row, lanes per row as in the merge.  The weights are
// w_x = exp(lse_x - m) / sum_y exp(lse_y - m) with m the largest lse, so an empty state (lse = -inf)
// weighs 0 and (-inf) - (-inf) is never formed; a row empty in every state gives O = 0, lse = -inf.
// The O loads of kCombineUnroll states are in flight together.
constexpr int kCombineUnroll = 4;
constexpr int kCombineFew = 2 * kCombineUnroll;

template <bool kLowp, bool kFew>
__global__ __launch_bounds__(256) void combine_kernel(const CombineArgs a, int32_t vec_per_row, int32_t lane_shift) {
  const int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t row = tid >> lane_shift;               // (b * Sq_out + i) * Hq + h
  const int32_t sub = (int32_t)(tid & ((1 << lane_shift) - 1));
  const int64_t n_rows = (int64_t)a.B * a.Sq_out * a.Hq;
  if (row >= n_rows || sub >= vec_per_row) return;
  const int32_t h = (int32_t)(row % a.Hq);
  const int64_t bi = row / a.Hq;
  const int64_t b = bi / a.Sq_out;
  const int32_t i = (int32_t)(bi % a.Sq_out);
  const int64_t l_in = (b * a.Hq + h) * a.Sq_in + a.row0 + i;
  const int64_t v_in = ((b * a.Sq_in + a.row0 + i) * a.Hq + h) * vec_per_row + sub;

  typedef float f32x4_t __attribute__((ext_vector_type(4)));
  auto load_o = [&](int x) {
    const f32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(a.o[x]) + v_in);   // read once
    return make_float4(t.x, t.y, t.z, t.w);
  };
  // a weight of exactly 0 must not turn a non-finite value of an empty state into NaN
  auto add = [](float4& r, float w, const float4& p) {
    if (w != 0.f) {
      r.x = fmaf(w, p.x, r.x);
      r.y = fmaf(w, p.y, r.y);
      r.z = fmaf(w, p.z, r.z);
      r.w = fmaf(w, p.w, r.w);
    }
  };
  float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
  float lnew = -INFINITY;
  if (kFew) {
    // up to kCombineFew states (a team): every lse is read once and kept, and the first O loads do not wait for them
    float l[kCombineFew];
    float4 p[kCombineUnroll];
#pragma unroll
    for (int x = 0; x < kCombineFew; ++x) l[x] = x < a.n ? a.lse[x][l_in] : -INFINITY;
#pragma unroll
    for (int u = 0; u < kCombineUnroll; ++u) p[u] = load_o(u < a.n ? u : a.n - 1);
    float m = -INFINITY;
#pragma unroll
    for (int x = 0; x < kCombineFew; ++x) m = fmaxf(m, l[x]);
    if (m != -INFINITY) {
      float sum = 0.f;
#pragma unroll
      for (int x = 0; x < kCombineFew; ++x) {
        l[x] = expf(l[x] - m);                           // exp(-inf) = 0 for an empty state and for x >= n
        sum += l[x];
      }
      lnew = m + logf(sum);
      const float inv = 1.f / sum;
#pragma unroll
      for (int u = 0; u < kCombineUnroll; ++u) add(r, u < a.n ? l[u] * inv : 0.f, p[u]);
      if (a.n > kCombineUnroll) {
#pragma unroll
        for (int u = 0; u < kCombineUnroll; ++u) p[u] = load_o(kCombineUnroll + u < a.n ? kCombineUnroll + u : a.n - 1);
#pragma unroll
        for (int u = 0; u < kCombineUnroll; ++u) add(r, kCombineUnroll + u < a.n ? l[kCombineUnroll + u] * inv : 0.f, p[u]);
      }
    }
  } else {
    float m = -INFINITY;
    for (int x = 0; x < a.n; ++x) m = fmaxf(m, a.lse[x][l_in]);
    if (m != -INFINITY) {
      float sum = 0.f;
      for (int x = 0; x < a.n; ++x) sum += expf(a.lse[x][l_in] - m);
      lnew = m + logf(sum);
      const float inv = 1.f / sum;
      for (int x0 = 0; x0 < a.n; x0 += kCombineUnroll) {
        float4 p[kCombineUnroll];
        float w[kCombineUnroll];
#pragma unroll
        for (int u = 0; u < kCombineUnroll; ++u) {
          const int x = x0 + u < a.n ? x0 + u : a.n - 1;
          p[u] = load_o(x);
          w[u] = x0 + u < a.n ? expf(a.lse[x][l_in] - m) * inv : 0.f;
        }
#pragma unroll
        for (int u = 0; u < kCombineUnroll; ++u) add(r, w[u], p[u]);
      }
    }
  }
  const int64_t v_out = row * vec_per_row + sub;
  reinterpret_cast<float4*>(a.o_out)[v_out] = r;
  if (kLowp) reinterpret_cast<uint2*>(a.o_lowp)[v_out] = make_uint2(pack_bf16x2(r.x, r.y), pack_bf16x2(r.z, r.w));
  if (sub == 0) a.lse_out[(b * a.Hq + h) * a.Sq_out + i] = lnew;
}

// fp32 "lowp" copy for the fp32 storage dtype
__global__ __launch_bounds__(256) void copy_f32_kernel(const float4* __restrict__ src, float4* __restrict__ dst,
                                                       int64_t n_vec) {
  const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (v < n_vec) dst[v] = src[v];
}

// ---- delta: 16 lanes per row, 16-byte loads, shuffle reduction inside the 16-lane group -------
template <bool kDoBf16, bool kOBf16>
__global__ __launch_bounds__(256) void delta_kernel(View d_o, View o, float* __restrict__ delta, int32_t B,
                                                    int32_t Sq, int32_t Hq, int32_t D) {
  const int64_t row = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 4;
  const int sub = threadIdx.x & 15;
  const int64_t n_rows = (int64_t)B * Sq * Hq;
  float acc = 0.f;
  if (row < n_rows) {
    const int32_t h = (int32_t)(row % Hq);
    const int64_t bi = row / Hq;
    const int32_t i = (int32_t)(bi % Sq);
    const int64_t b = bi / Sq;
    const int64_t off_d = b * d_o.sb + (int64_t)i * d_o.ss + (int64_t)h * d_o.sh;
    const int64_t off_o = b * o.sb + (int64_t)i * o.ss + (int64_t)h * o.sh;
    for (int d = sub * 8; d < D; d += 128) {           // 8 elements per lane per step
      float x[8], y[8];
      if (kDoBf16) {
        const uint4 u = *reinterpret_cast<const uint4*>((const uint16_t*)d_o.ptr + off_d + d);
        x[0] = bf16_lo(u.x); x[1] = bf16_hi(u.x); x[2] = bf16_lo(u.y); x[3] = bf16_hi(u.y);
        x[4] = bf16_lo(u.z); x[5] = bf16_hi(u.z); x[6] = bf16_lo(u.w); x[7] = bf16_hi(u.w);
      } else {
        const float4 u0 = *reinterpret_cast<const float4*>((const float*)d_o.ptr + off_d + d);
        const float4 u1 = *reinterpret_cast<const float4*>((const float*)d_o.ptr + off_d + d + 4);
        x[0] = u0.x; x[1] = u0.y; x[2] = u0.z; x[3] = u0.w; x[4] = u1.x; x[5] = u1.y; x[6] = u1.z; x[7] = u1.w;
      }
      if (kOBf16) {
        const uint4 u = *reinterpret_cast<const uint4*>((const uint16_t*)o.ptr + off_o + d);
        y[0] = bf16_lo(u.x); y[1] = bf16_hi(u.x); y[2] = bf16_lo(u.y); y[3] = bf16_hi(u.y);
        y[4] = bf16_lo(u.z); y[5] = bf16_hi(u.z); y[6] = bf16_lo(u.w); y[7] = bf16_hi(u.w);
      } else {
        const float4 u0 = *reinterpret_cast<const float4*>((const float*)o.ptr + off_o + d);
        const float4 u1 = *reinterpret_cast<const float4*>((const float*)o.ptr + off_o + d + 4);
        y[0] = u0.x; y[1] = u0.y; y[2] = u0.z; y[3] = u0.w; y[4] = u1.x; y[5] = u1.y; y[6] = u1.z; y[7] = u1.w;
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) acc = fmaf(x[e], y[e], acc);
    }
  }
#pragma unroll
  for (int s = 8; s > 0; s >>= 1) acc += __shfl_xor(acc, s);
  if (row < n_rows && sub == 0) {
    const int32_t h = (int32_t)(row % Hq);
    const int64_t bi = row / Hq;
    delta[((bi / Sq) * Hq + h) * Sq + (bi % Sq)] = acc;
  }
}

__global__ __launch_bounds__(256) void cast_bf16_kernel(const float4* __restrict__ src, uint2* __restrict__ dst,
                                                        int64_t n_vec, const float* __restrict__ src_tail,
                                                        uint16_t* __restrict__ dst_tail, int tail) {
  const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (v < n_vec) {
    const float4 x = src[v];
    dst[v] = make_uint2(pack_bf16x2(x.x, x.y), pack_bf16x2(x.z, x.w));
  } else if (v - n_vec < tail) {
    dst_tail[v - n_vec] = (uint16_t)f32_to_bf16_rne(src_tail[v - n_vec]);
  }
}

// ---- Q' = bf16(Q * c): thread = 8 elements (16 bytes) of one (b, i, h) row; dense output -----------------
__global__ __launch_bounds__(256) void scale_q_kernel(View q, u32x4* __restrict__ dst, int32_t B, int32_t Sq,
                                                      int32_t Hq, int32_t D, float c) {
  const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int32_t per_row = D / 8;
  const int64_t row = v / per_row;
  if (row >= (int64_t)B * Sq * Hq) return;
  const int32_t chunk = (int32_t)(v % per_row);
  const int32_t h = (int32_t)(row % Hq);
  const int64_t bi = row / Hq;
  const int64_t off = (bi / Sq) * q.sb + (bi % Sq) * q.ss + (int64_t)h * q.sh + chunk * 8;
  dst[v] = scale_bf16x8(*reinterpret_cast<const u32x4*>((const uint16_t*)q.ptr + off), c);
}

__global__ __launch_bounds__(256) void fill_state_kernel(float* __restrict__ o, float* __restrict__ lse,
                                                         int64_t n_o, int64_t n_lse) {
  const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (v < n_o) o[v] = 0.f;
  if (v < n_lse) lse[v] = -INFINITY;
}

// n dwords to zero, four per lane (the tail lane by lane)
__global__ __launch_bounds__(256) void zero_kernel(uint32_t* __restrict__ dst, int64_t n) {
  const int64_t v = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (v + 4 <= n && (reinterpret_cast<uintptr_t>(dst) & 15) == 0) {
    *reinterpret_cast<uint4*>(dst + v) = make_uint4(0u, 0u, 0u, 0u);
  } else {
    for (int64_t i = v; i < n && i < v + 4; ++i) dst[i] = 0u;
  }
}

inline unsigned blocks_for(int64_t n) { return (unsigned)((n + 255) / 256); }

}  // namespace

hipError_t launch_merge(float* o_acc, float* lse_acc, const float* o_part, const float* lse_part, int32_t B,
                        int32_t Sq, int32_t Hq, int32_t D, void* o_lowp, int lowp_dtype, hipStream_t s) {
  const int64_t n_rows = (int64_t)B * Sq * Hq;
  const int64_t n_vec = n_rows * (D / 4);
  if (n_vec == 0) return hipSuccess;
  // lanes per row and vectors per lane: eight lanes where the row has that many vectors (a group then reads whole
  // 128-byte lines), up to four vectors each, more lanes for the longest rows (D <= 256: at most 16)
  const int vec = D / 4;
  int lane_shift = 0;
  while ((1 << lane_shift) < 8 && (1 << lane_shift) < vec) ++lane_shift;
  while ((4 << lane_shift) < vec) ++lane_shift;
  const int per_lane = (vec + (1 << lane_shift) - 1) >> lane_shift;      // 1 .. 4
  const unsigned blocks = blocks_for(n_rows << lane_shift);
  const bool lowp = o_lowp != nullptr && lowp_dtype == ST_BF16;
  ProfScope prof("merge", s);
#define ST_LAUNCH_MERGE(LOWP, U)                                                                                    \
  hipLaunchKernelGGL((merge_kernel<LOWP, U>), dim3(blocks), dim3(256), 0, s, o_acc, lse_acc, o_part, lse_part, n_rows, \
                     Sq, Hq, vec, lane_shift, (uint2*)(LOWP ? o_lowp : nullptr))
  if (lowp) {
    if (per_lane == 1) ST_LAUNCH_MERGE(true, 1);
    else if (per_lane == 2) ST_LAUNCH_MERGE(true, 2);
    else ST_LAUNCH_MERGE(true, 4);
    return hipGetLastError();
  }
  if (per_lane == 1) ST_LAUNCH_MERGE(false, 1);
  else if (per_lane == 2) ST_LAUNCH_MERGE(false, 2);
  else ST_LAUNCH_MERGE(false, 4);
#undef ST_LAUNCH_MERGE
  hipError_t e = hipGetLastError();
  if (e == hipSuccess && o_lowp != nullptr) {
    hipLaunchKernelGGL(copy_f32_kernel, dim3(blocks_for(n_vec)), dim3(256), 0, s, (const float4*)o_acc,
                       (float4*)o_lowp, n_vec);
    e = hipGetLastError();
  }
  return e;
}

hipError_t launch_combine(const CombineArgs& a, int lowp_dtype, hipStream_t s) {
  const int64_t n_rows = (int64_t)a.B * a.Sq_out * a.Hq;
  const int64_t n_vec = n_rows * (a.D / 4);
  if (n_vec == 0) return hipSuccess;
  int lane_shift = 0;
  while ((1 << lane_shift) < a.D / 4) ++lane_shift;
  const unsigned blocks = blocks_for(n_rows << lane_shift);
  ProfScope prof("combine", s);
  if (a.o_lowp != nullptr && lowp_dtype == ST_BF16) {
    if (a.n <= kCombineFew) hipLaunchKernelGGL((combine_kernel<true, true>), dim3(blocks), dim3(256), 0, s, a, a.D / 4, lane_shift);
    else hipLaunchKernelGGL((combine_kernel<true, false>), dim3(blocks), dim3(256), 0, s, a, a.D / 4, lane_shift);
    return hipGetLastError();
  }
  if (a.n <= kCombineFew) hipLaunchKernelGGL((combine_kernel<false, true>), dim3(blocks), dim3(256), 0, s, a, a.D / 4, lane_shift);
  else hipLaunchKernelGGL((combine_kernel<false, false>), dim3(blocks), dim3(256), 0, s, a, a.D / 4, lane_shift);
  hipError_t e = hipGetLastError();
  if (e == hipSuccess && a.o_lowp != nullptr) {
    hipLaunchKernelGGL(copy_f32_kernel, dim3(blocks_for(n_vec)), dim3(256), 0, s, (const float4*)a.o_out,
                       (float4*)a.o_lowp, n_vec);
    e = hipGetLastError();
  }
  return e;
}

hipError_t launch_delta(const View& d_o, int d_o_dtype, const View& o, int o_dtype, float* delta, int32_t B,
                        int32_t Sq, int32_t Hq, int32_t D, hipStream_t s) {
  const int64_t n_rows = (int64_t)B * Sq * Hq;
  if (n_rows == 0) return hipSuccess;
  const dim3 grid(blocks_for(n_rows * 16)), block(256);
  const bool db = d_o_dtype == ST_BF16, ob = o_dtype == ST_BF16;
  ProfScope prof("delta", s);
  if (db && ob) hipLaunchKernelGGL((delta_kernel<true, true>), grid, block, 0, s, d_o, o, delta, B, Sq, Hq, D);
  else if (db) hipLaunchKernelGGL((delta_kernel<true, false>), grid, block, 0, s, d_o, o, delta, B, Sq, Hq, D);
  else if (ob) hipLaunchKernelGGL((delta_kernel<false, true>), grid, block, 0, s, d_o, o, delta, B, Sq, Hq, D);
  else hipLaunchKernelGGL((delta_kernel<false, false>), grid, block, 0, s, d_o, o, delta, B, Sq, Hq, D);
  return hipGetLastError();
}

hipError_t launch_cast(const float* src, void* dst, int64_t n, int dst_dtype, hipStream_t s) {
  if (n == 0) return hipSuccess;
  if (dst_dtype == ST_F32) return hipMemcpyAsync(dst, src, n * sizeof(float), hipMemcpyDeviceToDevice, s);
  const int64_t n_vec = n / 4;
  const int tail = (int)(n - n_vec * 4);
  ProfScope prof("cast", s);
  hipLaunchKernelGGL(cast_bf16_kernel, dim3(blocks_for(n_vec + tail)), dim3(256), 0, s, (const float4*)src,
                     (uint2*)dst, n_vec, src + n_vec * 4, (uint16_t*)dst + n_vec * 4, tail);
  return hipGetLastError();
}

hipError_t launch_scale_q(const View& q, void* dst, int32_t B, int32_t Sq, int32_t Hq, int32_t D, float scale,
                          hipStream_t s) {
  const int64_t n_vec = (int64_t)B * Sq * Hq * (D / 8);
  if (n_vec == 0) return hipSuccess;
  ProfScope prof("scale_q", s);
  hipLaunchKernelGGL(scale_q_kernel, dim3(blocks_for(n_vec)), dim3(256), 0, s, q, (u32x4*)dst, B, Sq, Hq, D,
                     scale * 1.4426950408889634f);
  return hipGetLastError();
}

hipError_t launch_zero(void* dst, int64_t bytes, hipStream_t s) {
  if (bytes <= 0) return hipSuccess;
  const int64_t n = bytes / 4;
  ProfScope prof("zero", s);
  hipLaunchKernelGGL(zero_kernel, dim3(blocks_for((n + 3) / 4)), dim3(256), 0, s, (uint32_t*)dst, n);
  return hipGetLastError();
}

hipError_t launch_fill_state(float* o, float* lse, int64_t n_o, int64_t n_lse, hipStream_t s) {
  const int64_t n = n_o > n_lse ? n_o : n_lse;
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(fill_state_kernel, dim3(blocks_for(n)), dim3(256), 0, s, o, lse, n_o, n_lse);
  return hipGetLastError();
}

}  // namespace st
