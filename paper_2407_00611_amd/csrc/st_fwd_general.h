// General bf16 forward (masked and ragged tiles, any visible prefix) as a device function, so that it can be a
// kernel of its own (st_fwd_bf16.hip) and run side by side with the hand-scheduled loop in one launch
// (st_fwd_fast.hip).
//
// Attention of a resident Q tile against a table of KV chunks, visited in order, with the online-softmax state
// (row max, row sum, O accumulator) kept in registers for the whole walk.
// Workgroup = 4 wavefronts, 4 * kWQ queries of one head.  Per 64-key tile and wavefront:
//   S^T = K Q'^T       A = K fragment (LDS, 16-byte reads), B = Q' fragment (registers, loaded once)
//   online softmax in the C layout: a lane owns ONE query column, so the row statistics are
//                      per-lane scalars and only one cross-half exchange per tile is needed
//   O^T += V^T P^T     A = V^T fragment (LDS transpose reads), B = P^T straight from the S registers
// K/V tiles go global -> LDS directly (XOR-swizzled, double buffered), one barrier per tile.
#pragma once

#include "st_internal.h"
#include "st_mfma.h"

namespace st {
namespace {

constexpr int kBN = 64;       // keys per tile
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kRescaleGap = 8.f;   // log2 units

// visible prefix of a chunk for a query at global position qpos
__device__ __forceinline__ int visible_keys(int causal, int Sk, int64_t qpos, int64_t k0) {
  if (!causal) return Sk;
  const int64_t n = qpos - k0 + 1;
  return n < 0 ? 0 : (n > Sk ? Sk : (int)n);
}

// Body of the general forward kernel.  kWQ = queries per wavefront: 64 (one wavefront per SIMD) or 32 (two
// workgroups per CU, so that one wavefront's softmax overlaps another's MFMAs).
//   block_x, grid_x  position of this workgroup among the query tiles (XCD-aware mapping, see qtile_block)
//   split            which share of the chunk table it walks (0 when the launch is not split)
//   smem_raw         4 * 64 * D * 2 bytes of LDS, 1 KiB aligned
// With a.fwd_fast == 1 the fast kernel's partial result is already in the output state and this kernel folds
// its own into it; with a.fwd_fast == 2 (both run in ONE launch, side by side) it walks the whole table, takes
// only the tiles that are not the fast kernel's, and writes a state of its own in split slot a.n_split.
template <int D, int kWQ>
__device__ __forceinline__ void fwd_general_body(const FwdArgs& a, int block_x, int grid_x, int split, char* smem_raw) {
  constexpr int kBM = 4 * kWQ;   // queries per workgroup
  constexpr int QB = kWQ / 32;   // 32-query blocks per wavefront
  constexpr int KB = kBN / 32;   // 32-key blocks per tile
  constexpr int KS = D / 16;     // contraction steps of S^T = K Q^T
  constexpr int DB = D / 32;     // 32-row blocks of O^T
  constexpr int kTile = kBN * D * 2;          // bytes of one K (or V) tile, XOR-swizzled, unpadded
  ST_LDS char* smem = (ST_LDS char*)smem_raw;                          // 2 stages x (K, V)

  const Shape& s = a.s;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, r = lane & 31;

  const int n_qt = (s.Sq + kBM - 1) / kBM;
  int qt, hb;
  qtile_block(block_x, grid_x, n_qt, s.causal, qt, hb);
  const int h = hb % s.Hq;
  const int b = hb / s.Hq;
  const int hk = h / (s.Hq / s.Hkv);

  // ---- Q fragments (B operand of S^T): query column r of block qb, d = 16 ks + 8 g .. +7, as the exponent
  // operand Q' = bf16(Q scale log2 e) that every bf16 kernel uses: the scores come out in log2 units
  const int q_row0 = qt * kBM + wave * kWQ;
  const float q_mul = s.scale * kLog2e;
  bf16x8 qf[QB][KS];
  int64_t qpos[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int i = q_row0 + 32 * qb + r;
    qpos[qb] = q_pos(s, i);
    const char* qrow = (const char*)a.q.ptr + ((int64_t)b * a.q.sb + (int64_t)i * a.q.ss + (int64_t)h * a.q.sh) * 2;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      if (i < s.Sq) qf[qb][ks] = scale_bf16x8(*reinterpret_cast<const bf16x8*>(qrow + (16 * ks + 8 * g) * 2), q_mul);
      else qf[qb][ks] = __builtin_bit_cast(bf16x8, u32x4{0, 0, 0, 0});
    }
  }

  // rows of this workgroup / wavefront that exist
  const int wg_last_row = min(qt * kBM + kBM, s.Sq) - 1;
  const int wave_first_row = q_row0;

  f32x16 acc_o[DB][QB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc_o[db][qb][v] = 0.f;
  float m_run[QB], l_run[QB];   // running max (log2 units, like the scores) and this lane's partial row sum
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    m_run[qb] = -INFINITY;
    l_run[qb] = 0.f;
  }
  constexpr float c_exp = 1.f;   // the scores are exponents already

  // ---- flattened (chunk, tile) walk with one-tile lookahead
  // number of tiles the workgroup needs from chunk c: up to the last key its last row may see
  auto chunk_tiles = [&](int c) -> int {
    const int nv = visible_keys(s.causal, s.Sk, q_pos(s, wg_last_row), a.t.k_offset[c]);
    return (nv + kBN - 1) / kBN;
  };
  // first tile of a chunk that is this kernel's: the leading ones may belong to the fast kernel, whose
  // partial (O, lse) is then already in the output buffers and is merged with this kernel's in the epilogue
  const int fast_row0 = qt * kBM / kQTileFastRows * kQTileFastRows;
  const bool fast_on = a.fwd_fast && kBN == kQTileFastKeys && fast_row0 + kQTileFastRows <= s.Sq;
  auto chunk_t0 = [&](int c) -> int {
    return fast_on ? qtile_fast_tiles(s, fast_row0, a.t.k_offset[c]) : 0;
  };
  // this workgroup's share of the table and its output state (one share, the whole table, unless the launch is split)
  const bool side_by_side = a.fwd_fast == 2;
  int c_lo = 0, c_hi = a.t.n;
  if (!side_by_side) split_range(a.t.n, a.n_split, split, c_lo, c_hi);
  const int slot = side_by_side ? a.n_split : split;
  float* const out_o = a.o + (int64_t)slot * a.split_o;
  float* const out_lse = a.lse + (int64_t)slot * a.split_l;
  bool fast_wrote = false;
  if (fast_on && !side_by_side)
    for (int c = c_lo; c < c_hi; ++c) fast_wrote = fast_wrote || chunk_t0(c) > 0;
  int c_cur = c_lo, t_cur = 0, n_cur = 0;       // current chunk, tile, tiles in chunk
  while (c_cur < c_hi && (n_cur = chunk_tiles(c_cur)) <= (t_cur = chunk_t0(c_cur))) ++c_cur;

  auto issue_load = [&](int c, int t, int stage) {
    const char* kb = (const char*)a.t.k[c] + ((int64_t)b * a.t.ksb + (int64_t)hk * a.t.ksh) * 2;
    const char* vb = (const char*)a.t.v[c] + ((int64_t)b * a.t.vsb + (int64_t)hk * a.t.vsh) * 2;
    stage_dma<D, kBN>(kb, a.t.kss, t * kBN, s.Sk, smem + stage * 2 * kTile, tid);
    stage_dma<D, kBN>(vb, a.t.vss, t * kBN, s.Sk, smem + stage * 2 * kTile + kTile, tid);
  };

  int buf = 0;
  if (c_cur < c_hi) issue_load(c_cur, t_cur, 0);
  __syncthreads();

  while (c_cur < c_hi) {
    // next (chunk, tile)
    int c_nxt = c_cur, t_nxt = t_cur + 1, n_nxt = n_cur;
    if (t_nxt >= n_cur) {
      ++c_nxt;
      while (c_nxt < c_hi && (n_nxt = chunk_tiles(c_nxt)) <= (t_nxt = chunk_t0(c_nxt))) ++c_nxt;
    }
    const bool have_next = c_nxt < c_hi;
    if (have_next) issue_load(c_nxt, t_nxt, buf ^ 1);

    // ---- compute on the staged tile
    const int64_t k0 = a.t.k_offset[c_cur];
    const int tile_k0 = t_cur * kBN;
    // visible-prefix lengths: first / last live row of the wavefront and this lane's rows
    const int nv_wave_min = visible_keys(s.causal, s.Sk, q_pos(s, wave_first_row), k0);
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
      // and lse = m_run ln 2 + ln(l) at the end.  The rest of the tile exists twice (with and
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

  // ---- epilogue: O = acc / l, lse = m ln 2 + ln(l); folded into the fast kernel's partial result if there is one
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int i = q_row0 + 32 * qb + r;
    const float l = xhalf_sum(l_run[qb]);
    const float inv = l > 0.f ? 1.f / l : 0.f;
    if (i < s.Sq) {
      const int64_t orow = (((int64_t)b * s.Sq + i) * s.Hq + h) * D;
      const int64_t srow = ((int64_t)b * s.Hq + h) * s.Sq + i;
      float lse_own = l > 0.f ? m_run[qb] * kLn2 + logf(l) : -INFINITY;
      float w_own = inv, w_prev = 0.f;          // weights of this kernel's accumulator and of the stored partial O
      if (fast_wrote) {
        const float lse_prev = out_lse[srow];
        const float mx = fmaxf(lse_prev, lse_own);
        if (mx != -INFINITY) {
          const float e_prev = expf(lse_prev - mx), e_own = expf(lse_own - mx);
          const float tot = e_prev + e_own;
          w_prev = e_prev / tot;
          w_own = inv * (e_own / tot);
          lse_own = mx + logf(tot);
        }
      }
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int d = 32 * db + 8 * q4 + 4 * g;
          float4 o;
          o.x = acc_o[db][qb][4 * q4 + 0] * w_own;
          o.y = acc_o[db][qb][4 * q4 + 1] * w_own;
          o.z = acc_o[db][qb][4 * q4 + 2] * w_own;
          o.w = acc_o[db][qb][4 * q4 + 3] * w_own;
          if (fast_wrote) {
            const float4 p = *reinterpret_cast<const float4*>(out_o + orow + d);
            o.x = fmaf(p.x, w_prev, o.x);
            o.y = fmaf(p.y, w_prev, o.y);
            o.z = fmaf(p.z, w_prev, o.z);
            o.w = fmaf(p.w, w_prev, o.w);
          }
          *reinterpret_cast<float4*>(out_o + orow + d) = o;
          if (a.o_lowp) {
            uint2 w = make_uint2(pack_bf16(o.x, o.y), pack_bf16(o.z, o.w));
            *reinterpret_cast<uint2*>((uint16_t*)a.o_lowp + orow + d) = w;
          }
        }
      if (g == 0) out_lse[srow] = lse_own;
      // side by side with the fast kernel: rows outside the full query tiles have no fast workgroup, so the
      // split states, which only fast workgroups write, are marked empty there
      if (side_by_side && !fast_on && g == 0)
        for (int y = 0; y < a.n_split; ++y) a.lse[(int64_t)y * a.split_l + srow] = -INFINITY;
    }
  }
}

}  // namespace
}  // namespace st
