// bf16 forward: attention of a resident Q tile against a table of KV chunks, visited in order,
// with the online-softmax state (row max, row sum, O accumulator) kept in registers for the whole
// walk.  One launch with a 1-entry table is st_attn_block_fwd; with the full table it is the fused
// ring forward.
//
// Workgroup = 4 wavefronts, 256 queries of one head (64 per wavefront, as two 32-query blocks).
// Per 64-key tile and wavefront:
//   S^T = K Q^T        A = K fragment (LDS, 16-byte reads), B = Q fragment (registers, loaded once)
//   online softmax in the C layout: a lane owns ONE query column, so the row statistics are
//                      per-lane scalars and only one cross-half exchange per tile is needed
//   O^T += V^T P^T     A = V^T fragment (LDS transpose reads), B = P^T straight from the S registers
// K/V tiles go global -> LDS directly (XOR-swizzled, double buffered), one barrier per tile.
#include <cstdlib>
#include <type_traits>

#include "st_internal.h"
#include "st_mfma.h"

namespace st {
namespace {

constexpr int kBN = 64;       // keys per tile
#ifndef ST_FWD_WQ
#define ST_FWD_WQ 32
#endif
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kRescaleGap = 8.f;   // log2 units

// visible prefix of a chunk for a query at global position qpos
__device__ __forceinline__ int visible_keys(int causal, int Sk, int64_t qpos, int64_t k0) {
  if (!causal) return Sk;
  const int64_t n = qpos - k0 + 1;
  return n < 0 ? 0 : (n > Sk ? Sk : (int)n);
}

// kWQ = queries per wavefront: 64 (one wavefront per SIMD) or 32 (two workgroups per CU, so that one
// wavefront's softmax overlaps another's MFMAs)
template <int D, int kWQ>
__global__ __launch_bounds__(256, kWQ == 32 ? 2 : 1) void fwd_bf16_kernel(const FwdArgs a) {
  constexpr int kBM = 4 * kWQ;   // queries per workgroup
  constexpr int QB = kWQ / 32;   // 32-query blocks per wavefront
  constexpr int KB = kBN / 32;   // 32-key blocks per tile
  constexpr int KS = D / 16;     // contraction steps of S^T = K Q^T
  constexpr int DB = D / 32;     // 32-row blocks of O^T
  constexpr int kTile = kBN * D * 2;          // bytes of one K (or V) tile, XOR-swizzled, unpadded
  __shared__ __attribute__((aligned(1024))) char smem_raw[4 * kTile];   // 2 stages x (K, V)
  ST_LDS char* smem = (ST_LDS char*)smem_raw;

  const Shape& s = a.s;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, r = lane & 31;

  const int n_qt = (s.Sq + kBM - 1) / kBM;
  const int logical = xcd_logical_block(blockIdx.x, gridDim.x);
  const int qt = logical % n_qt;
  const int h = (logical / n_qt) % s.Hq;
  const int b = logical / (n_qt * s.Hq);
  const int hk = h / (s.Hq / s.Hkv);

  // ---- Q fragments (B operand of S^T): query column r of block qb, d = 16 ks + 8 g .. +7
  const int q_row0 = qt * kBM + wave * kWQ;
  bf16x8 qf[QB][KS];
  int64_t qpos[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int i = q_row0 + 32 * qb + r;
    qpos[qb] = s.q_offset + i;
    const char* qrow = (const char*)a.q.ptr + ((int64_t)b * a.q.sb + (int64_t)i * a.q.ss + (int64_t)h * a.q.sh) * 2;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      if (i < s.Sq) qf[qb][ks] = *reinterpret_cast<const bf16x8*>(qrow + (16 * ks + 8 * g) * 2);
      else qf[qb][ks] = __builtin_bit_cast(bf16x8, u32x4{0, 0, 0, 0});
    }
  }

  // rows of this workgroup / wavefront that exist
  const int wg_last_row = min(qt * kBM + kBM, s.Sq) - 1;
  const int wave_first_row = q_row0;
  const int wave_last_row = min(q_row0 + kWQ, s.Sq) - 1;   // < wave_first_row if the wavefront has no rows
  const bool wave_live = wave_last_row >= wave_first_row;

  f32x16 acc_o[DB][QB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc_o[db][qb][v] = 0.f;
  float m_run[QB], l_run[QB];   // running max (in units of raw scores) and this lane's partial row sum
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    m_run[qb] = -INFINITY;
    l_run[qb] = 0.f;
  }
  const float c_exp = s.scale * kLog2e;

  // ---- flattened (chunk, tile) walk with one-tile lookahead
  // number of tiles the workgroup needs from chunk c: up to the last key its last row may see
  auto chunk_tiles = [&](int c) -> int {
    const int nv = visible_keys(s.causal, s.Sk, s.q_offset + wg_last_row, a.t.k_offset[c]);
    return (nv + kBN - 1) / kBN;
  };
  int c_cur = 0, t_cur = 0, n_cur = 0;          // current chunk, tile, tiles in chunk
  while (c_cur < a.t.n && (n_cur = chunk_tiles(c_cur)) == 0) ++c_cur;

  auto issue_load = [&](int c, int t, int stage) {
    const char* kb = (const char*)a.t.k[c] + ((int64_t)b * a.t.ksb + (int64_t)hk * a.t.ksh) * 2;
    const char* vb = (const char*)a.t.v[c] + ((int64_t)b * a.t.vsb + (int64_t)hk * a.t.vsh) * 2;
    stage_dma<D, kBN>(kb, a.t.kss, t * kBN, s.Sk, smem + stage * 2 * kTile, tid);
    stage_dma<D, kBN>(vb, a.t.vss, t * kBN, s.Sk, smem + stage * 2 * kTile + kTile, tid);
  };

  int buf = 0;
  if (c_cur < a.t.n) issue_load(c_cur, 0, 0);
  __syncthreads();

  while (c_cur < a.t.n) {
    // next (chunk, tile)
    int c_nxt = c_cur, t_nxt = t_cur + 1, n_nxt = n_cur;
    if (t_nxt >= n_cur) {
      t_nxt = 0;
      ++c_nxt;
      while (c_nxt < a.t.n && (n_nxt = chunk_tiles(c_nxt)) == 0) ++c_nxt;
    }
    const bool have_next = c_nxt < a.t.n;
    if (have_next) issue_load(c_nxt, t_nxt, buf ^ 1);

    // ---- compute on the staged tile
    const int64_t k0 = a.t.k_offset[c_cur];
    const int tile_k0 = t_cur * kBN;
    // visible-prefix lengths: first / last live row of the wavefront and this lane's rows
    const int nv_wave_min = visible_keys(s.causal, s.Sk, s.q_offset + wave_first_row, k0);
    {  // every wavefront computes every tile the workgroup walks; rows that see nothing of it are masked
      const ST_LDS char* ktile = smem + buf * 2 * kTile;
      const ST_LDS char* vtile = ktile + kTile;
      f32x16 sc[KB][QB];
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
          for (int v = 0; v < 16; ++v) sc[kb][qb][v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
          const bf16x8 kf = lds_frag<D>(ktile, 32 * kb, ks, lane);
#pragma unroll
          for (int qb = 0; qb < QB; ++qb) sc[kb][qb] = mfma32(kf, qf[qb][ks], sc[kb][qb]);
        }

      const bool need_mask = tile_k0 + kBN > nv_wave_min;     // wave-uniform
      float mx[QB];
      bool jump = false;
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        if (need_mask) {
          const int nv = visible_keys(s.causal, s.Sk, qpos[qb], k0) - tile_k0;   // visible keys of this tile
#pragma unroll
          for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              const int key = 32 * kb + 8 * (v / 4) + 4 * g + (v % 4);
              if (key >= nv) sc[kb][qb][v] = -INFINITY;
            }
        }
        float x = sc[0][qb][0];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
          for (int v = 0; v < 16; ++v) x = fmaxf(x, sc[kb][qb][v]);
        mx[qb] = xhalf_max(x);
        jump = jump || (mx[qb] - m_run[qb]) * c_exp > kRescaleGap || (m_run[qb] == -INFINITY && mx[qb] != -INFINITY);
      }

      // Lazy rescale: the exponent reference m_run only moves when some row's tile maximum exceeds it
      // by more than kRescaleGap (log2 units), so p <= 2^kRescaleGap and the O accumulator is rescaled
      // rarely.  Exact in real arithmetic: O and l stay consistent with whatever reference is in use,
      // and lse = m_run * scale + ln(l) at the end.  The rest of the tile exists twice (with and
      // without the rescale) so that the common path carries the accumulators through untouched.
      auto rescale_rows = [&]() {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
          const float m_new = fmaxf(m_run[qb], mx[qb]);
          const float m_use = m_new == -INFINITY ? 0.f : m_new;
          const float alpha = __builtin_amdgcn_exp2f((m_run[qb] - m_use) * c_exp);
          l_run[qb] *= alpha;
          m_run[qb] = m_new;
#pragma unroll
          for (int db = 0; db < DB; ++db) scale_in_place(acc_o[db][qb], alpha);
        }
      };
      auto finish_tile = [&]() {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
          const float mc = (m_run[qb] == -INFINITY ? 0.f : m_run[qb]) * c_exp;
          float psum = 0.f;
#pragma unroll
          for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              const float p = __builtin_amdgcn_exp2f(fmaf(sc[kb][qb][v], c_exp, -mc));
              sc[kb][qb][v] = p;
              psum += p;
            }
          l_run[qb] += psum;
        }
        // O^T += V^T P^T : contraction over the tile's keys in steps of 16 (kb, m)
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
          for (int m = 0; m < 2; ++m) {
            bf16x8 pf[QB];
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) pf[qb] = pack_c_as_b(sc[kb][qb], m);
#pragma unroll
            for (int db = 0; db < DB; ++db) {
              const bf16x8 vf = lds_frag_tr<D>(vtile, 32 * kb + 16 * m, 32 * db, lane);
#pragma unroll
              for (int qb = 0; qb < QB; ++qb) acc_o[db][qb] = mfma32(vf, pf[qb], acc_o[db][qb]);
            }
          }
      };
      if (__builtin_expect(__any(jump), 0)) rescale_rows();
      finish_tile();
    }

    __syncthreads();
    buf ^= 1;
    c_cur = c_nxt;
    t_cur = t_nxt;
    n_cur = n_nxt;
  }

  // ---- epilogue: O = acc / l, lse = m * scale + ln(l)
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int i = q_row0 + 32 * qb + r;
    const float l = xhalf_sum(l_run[qb]);
    const float inv = l > 0.f ? 1.f / l : 0.f;
    if (i < s.Sq) {
      const int64_t orow = (((int64_t)b * s.Sq + i) * s.Hq + h) * D;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int d = 32 * db + 8 * q4 + 4 * g;
          float4 o;
          o.x = acc_o[db][qb][4 * q4 + 0] * inv;
          o.y = acc_o[db][qb][4 * q4 + 1] * inv;
          o.z = acc_o[db][qb][4 * q4 + 2] * inv;
          o.w = acc_o[db][qb][4 * q4 + 3] * inv;
          *reinterpret_cast<float4*>(a.o + orow + d) = o;
          if (a.o_lowp) {
            uint2 w = make_uint2(pack_bf16(o.x, o.y), pack_bf16(o.z, o.w));
            *reinterpret_cast<uint2*>((uint16_t*)a.o_lowp + orow + d) = w;
          }
        }
      if (g == 0) a.lse[((int64_t)b * s.Hq + h) * s.Sq + i] = l > 0.f ? m_run[qb] * s.scale + logf(l) : -INFINITY;
    }
  }
}

}  // namespace

template <int kWQ>
hipError_t launch_fwd_bf16_wq(const FwdArgs& a, hipStream_t stream) {
  constexpr int kBM = 4 * kWQ;
  const int n_qt = (a.s.Sq + kBM - 1) / kBM;
  const int64_t total = (int64_t)n_qt * a.s.Hq * a.s.B;
  if (total <= 0) return hipSuccess;
  if (total > 0x7fffffff) return hipErrorInvalidValue;
  ProfScope prof("fwd_bf16", stream);
  if (a.s.D == 128) hipLaunchKernelGGL((fwd_bf16_kernel<128, kWQ>), dim3((unsigned)total), dim3(256), 0, stream, a);
  else if (a.s.D == 64) hipLaunchKernelGGL((fwd_bf16_kernel<64, kWQ>), dim3((unsigned)total), dim3(256), 0, stream, a);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_fwd_bf16(const FwdArgs& a, hipStream_t stream) {
  // tuning override: ST_FWD_WQ=64 selects one wavefront per SIMD with 64 queries each
  static const int wq = [] {
    const char* e = getenv("ST_FWD_WQ");
    return e ? atoi(e) : ST_FWD_WQ;
  }();
  return wq == 64 ? launch_fwd_bf16_wq<64>(a, stream) : launch_fwd_bf16_wq<32>(a, stream);
}

}  // namespace st
