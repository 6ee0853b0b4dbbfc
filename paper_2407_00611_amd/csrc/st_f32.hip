// fp32 reference-precision kernels: any D <= 256 (multiple of 4), any Sq / Sk.
// Plain VALU code, one wavefront per query row (forward, dQ) or per key row (dK, dV):
// deterministic, no atomics.  These serve the fp32 storage dtype; the bf16 MFMA
// kernels are the throughput path.
#include "st_internal.h"

namespace st {
namespace {

constexpr int kWaves = 4;          // rows per workgroup
constexpr int kMaxD = 256;
constexpr int kDV = kMaxD / 64;    // d-values owned by a lane

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
  return x;
}

__device__ __forceinline__ float dot_row(const float* __restrict__ lds_vec, const float* __restrict__ row, int D) {
  float acc = 0.f;
  for (int d = 0; d < D; d += 4) {
    const float4 x = *reinterpret_cast<const float4*>(row + d);
    acc = fmaf(lds_vec[d], x.x, acc);
    acc = fmaf(lds_vec[d + 1], x.y, acc);
    acc = fmaf(lds_vec[d + 2], x.z, acc);
    acc = fmaf(lds_vec[d + 3], x.w, acc);
  }
  return acc;
}

// number of leading keys of a chunk that query position qpos may see
__device__ __forceinline__ int visible_keys(const Shape& s, int64_t qpos, int64_t k0) {
  if (!s.causal) return s.Sk;
  int64_t n = qpos - k0 + 1;
  return n < 0 ? 0 : (n > s.Sk ? s.Sk : (int)n);
}

// ---------------------------------------------------------------- forward
__global__ __launch_bounds__(kWaves * 64) void fwd_f32_kernel(const FwdArgs a) {
  __shared__ float qs[kWaves][kMaxD];
  const Shape& s = a.s;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int i = blockIdx.x * kWaves + w, h = blockIdx.y, b = blockIdx.z;
  const int g = h / (s.Hq / s.Hkv);
  const bool live = i < s.Sq;
  if (live) {
    const float* qrow = (const float*)a.q.ptr + b * a.q.sb + (int64_t)i * a.q.ss + h * a.q.sh;
    for (int d = lane; d < s.D; d += 64) qs[w][d] = qrow[d];
  }
  __syncthreads();
  if (!live) return;

  const int64_t qpos = q_pos(s, i);
  float m = -INFINITY, l = 0.f, acc[kDV] = {0.f, 0.f, 0.f, 0.f};
  for (int c = 0; c < a.t.n; ++c) {
    const float* kb = (const float*)a.t.k[c] + b * a.t.ksb + g * a.t.ksh;
    const float* vb = (const float*)a.t.v[c] + b * a.t.vsb + g * a.t.vsh;
    const int nvis = visible_keys(s, qpos, a.t.k_offset[c]);
    for (int t0 = 0; t0 < nvis; t0 += 64) {
      const int t = t0 + lane;
      const bool valid = t < nvis;
      const float sc = valid ? s.scale * dot_row(qs[w], kb + (int64_t)t * a.t.kss, s.D) : -INFINITY;
      const float m_new = fmaxf(m, wave_max(sc));          // finite: lane 0 is always valid
      const float p = valid ? expf(sc - m_new) : 0.f;
      const float alpha = expf(m - m_new);                 // m = -inf on the first tile -> 0
      l = l * alpha + wave_sum(p);
#pragma unroll
      for (int x = 0; x < kDV; ++x) acc[x] *= alpha;
      const int nt = min(64, nvis - t0);
      for (int tt = 0; tt < nt; ++tt) {
        const float pt = __shfl(p, tt);
        const float* vrow = vb + (int64_t)(t0 + tt) * a.t.vss;
#pragma unroll
        for (int x = 0; x < kDV; ++x) {
          const int d = lane + 64 * x;
          if (d < s.D) acc[x] = fmaf(pt, vrow[d], acc[x]);
        }
      }
      m = m_new;
    }
  }
  const float inv = l > 0.f ? 1.f / l : 0.f;
  const int64_t orow = (((int64_t)b * s.Sq + i) * s.Hq + h) * s.D;
#pragma unroll
  for (int x = 0; x < kDV; ++x) {
    const int d = lane + 64 * x;
    if (d < s.D) {
      a.o[orow + d] = acc[x] * inv;
      if (a.o_lowp) ((float*)a.o_lowp)[orow + d] = acc[x] * inv;   // storage dtype is fp32 here
    }
  }
  if (lane == 0) a.lse[((int64_t)b * s.Hq + h) * s.Sq + i] = l > 0.f ? m + logf(l) : -INFINITY;
}

// ---------------------------------------------------------------- backward: dQ
__global__ __launch_bounds__(kWaves * 64) void bwd_dq_f32_kernel(const BwdArgs a) {
  __shared__ float qs[kWaves][kMaxD];
  __shared__ float dos[kWaves][kMaxD];
  const Shape& s = a.s;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int i = blockIdx.x * kWaves + w, h = blockIdx.y, b = blockIdx.z;
  const int g = h / (s.Hq / s.Hkv);
  const bool live = i < s.Sq;
  if (live) {
    const float* qrow = (const float*)a.q.ptr + b * a.q.sb + (int64_t)i * a.q.ss + h * a.q.sh;
    const float* drow = (const float*)a.d_o.ptr + b * a.d_o.sb + (int64_t)i * a.d_o.ss + h * a.d_o.sh;
    for (int d = lane; d < s.D; d += 64) {
      qs[w][d] = qrow[d];
      dos[w][d] = drow[d];
    }
  }
  __syncthreads();
  if (!live) return;

  const int64_t stat = ((int64_t)b * s.Hq + h) * s.Sq + i;
  const float lse = a.lse[stat], dl = a.delta[stat];
  if (lse == -INFINITY) return;                            // empty row: no gradient
  const int64_t qpos = q_pos(s, i);
  float acc[kDV] = {0.f, 0.f, 0.f, 0.f};
  for (int c = 0; c < a.t.n; ++c) {
    const float* kb = (const float*)a.t.k[c] + b * a.t.ksb + g * a.t.ksh;
    const float* vb = (const float*)a.t.v[c] + b * a.t.vsb + g * a.t.vsh;
    const int nvis = visible_keys(s, qpos, a.t.k_offset[c]);
    for (int t0 = 0; t0 < nvis; t0 += 64) {
      const int t = t0 + lane;
      float ds = 0.f;
      if (t < nvis) {
        const float sc = s.scale * dot_row(qs[w], kb + (int64_t)t * a.t.kss, s.D);
        const float p = expf(sc - lse);
        const float dp = dot_row(dos[w], vb + (int64_t)t * a.t.vss, s.D);
        ds = p * (dp - dl);
      }
      const int nt = min(64, nvis - t0);
      for (int tt = 0; tt < nt; ++tt) {
        const float dst = __shfl(ds, tt);
        const float* krow = kb + (int64_t)(t0 + tt) * a.t.kss;
#pragma unroll
        for (int x = 0; x < kDV; ++x) {
          const int d = lane + 64 * x;
          if (d < s.D) acc[x] = fmaf(dst, krow[d], acc[x]);
        }
      }
    }
  }
  const int64_t orow = (((int64_t)b * s.Sq + i) * s.Hq + h) * s.D;
#pragma unroll
  for (int x = 0; x < kDV; ++x) {
    const int d = lane + 64 * x;
    if (d < s.D) a.dq[orow + d] += s.scale * acc[x];
  }
}

// ---------------------------------------------------------------- backward: dK, dV
// grid: (ceil(Sk / kWaves), Hkv, B * n_chunks)
__global__ __launch_bounds__(kWaves * 64) void bwd_dkv_f32_kernel(const BwdArgs a) {
  __shared__ float ks[kWaves][kMaxD];
  __shared__ float vs[kWaves][kMaxD];
  const Shape& s = a.s;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int t = blockIdx.x * kWaves + w, g = blockIdx.y;
  const int c = blockIdx.z / s.B, b = blockIdx.z % s.B;
  const int G = s.Hq / s.Hkv;
  const bool live = t < s.Sk;
  if (live) {
    const float* krow = (const float*)a.t.k[c] + b * a.t.ksb + (int64_t)t * a.t.kss + g * a.t.ksh;
    const float* vrow = (const float*)a.t.v[c] + b * a.t.vsb + (int64_t)t * a.t.vss + g * a.t.vsh;
    for (int d = lane; d < s.D; d += 64) {
      ks[w][d] = krow[d];
      vs[w][d] = vrow[d];
    }
  }
  __syncthreads();
  if (!live) return;

  const int64_t kpos = a.t.k_offset[c] + t;
  int i_first = 0;                                          // first query row that sees this key
  if (s.causal) {
    i_first = q_row_of(s, kpos);
    if (i_first >= s.Sq) return;
  }
  float acc_k[kDV] = {0.f, 0.f, 0.f, 0.f}, acc_v[kDV] = {0.f, 0.f, 0.f, 0.f};
  for (int hh = 0; hh < G; ++hh) {
    const int h = g * G + hh;
    const float* qb = (const float*)a.q.ptr + b * a.q.sb + h * a.q.sh;
    const float* db = (const float*)a.d_o.ptr + b * a.d_o.sb + h * a.d_o.sh;
    const int64_t stat = ((int64_t)b * s.Hq + h) * s.Sq;
    for (int i0 = i_first; i0 < s.Sq; i0 += 64) {
      const int i = i0 + lane;
      float p = 0.f, ds = 0.f;
      if (i < s.Sq) {
        const float lse = a.lse[stat + i];
        if (lse != -INFINITY) {
          const float sc = s.scale * dot_row(ks[w], qb + (int64_t)i * a.q.ss, s.D);
          p = expf(sc - lse);
          const float dp = dot_row(vs[w], db + (int64_t)i * a.d_o.ss, s.D);
          ds = p * (dp - a.delta[stat + i]);
        }
      }
      const int ni = min(64, s.Sq - i0);
      for (int ii = 0; ii < ni; ++ii) {
        const float pi = __shfl(p, ii), dsi = __shfl(ds, ii);
        const float* qrow = qb + (int64_t)(i0 + ii) * a.q.ss;
        const float* drow = db + (int64_t)(i0 + ii) * a.d_o.ss;
#pragma unroll
        for (int x = 0; x < kDV; ++x) {
          const int d = lane + 64 * x;
          if (d < s.D) {
            acc_k[x] = fmaf(dsi, qrow[d], acc_k[x]);
            acc_v[x] = fmaf(pi, drow[d], acc_v[x]);
          }
        }
      }
    }
  }
  const int64_t orow = (((int64_t)b * s.Sk + t) * s.Hkv + g) * s.D;
#pragma unroll
  for (int x = 0; x < kDV; ++x) {
    const int d = lane + 64 * x;
    if (d < s.D) {
      a.dk[c][orow + d] += s.scale * acc_k[x];
      a.dv[c][orow + d] += acc_v[x];
    }
  }
}

}  // namespace

hipError_t launch_fwd_f32(const FwdArgs& a, hipStream_t stream) {
  const dim3 grid((a.s.Sq + kWaves - 1) / kWaves, a.s.Hq, a.s.B);
  ProfScope prof("fwd_f32", stream);
  hipLaunchKernelGGL(fwd_f32_kernel, grid, dim3(kWaves * 64), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_bwd_f32(const BwdArgs& a, hipStream_t stream) {
  const dim3 grid_q((a.s.Sq + kWaves - 1) / kWaves, a.s.Hq, a.s.B);
  {
    ProfScope prof("bwd_dq_f32", stream);
    hipLaunchKernelGGL(bwd_dq_f32_kernel, grid_q, dim3(kWaves * 64), 0, stream, a);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || a.t.n == 0 || a.s.Sk == 0) return e;
  const dim3 grid_k((a.s.Sk + kWaves - 1) / kWaves, a.s.Hkv, a.s.B * a.t.n);
  ProfScope prof("bwd_dkv_f32", stream);
  hipLaunchKernelGGL(bwd_dkv_f32_kernel, grid_k, dim3(kWaves * 64), 0, stream, a);
  return hipGetLastError();
}

}  // namespace st
