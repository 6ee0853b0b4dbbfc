// bf16 backward of one GPU's ring-attention share, as two deterministic kernels (no atomics):
//
//   dq kernel   (query-stationary, mirrors the forward):  a workgroup owns 256 queries of one head
//               and walks the KV chunks; per 64-key tile
//                 S^T  = K Q^T,  dP^T = V dO^T            (K, V fragments from LDS; Q, dO in registers)
//                 dS^T = exp(S^T - lse) o (dP^T - Delta)  (lane owns one query column)
//                 dQ^T += K^T dS^T                        (K^T by LDS transpose reads)
//   dkv kernel  (key-stationary): a workgroup owns 256 keys of one KV head of one chunk (64 per
//               wavefront, K and V fragments resident in registers) and walks the query heads of
//               the group and their 64-query tiles
//                 S  = Q K^T,  dP = dO V^T,  P = exp(S - lse),  dS = P o (dP - Delta)
//                 dV^T += dO^T P,  dK^T += Q^T dS         (dO^T, Q^T by LDS transpose reads)
//
// Both recompute S and dP (seven contractions instead of five) so that every accumulator has a
// single owner: dQ is written once per launch, dK/dV once per workgroup, bit-reproducibly.
#include <cstdlib>

#include <utility>

#include "st_internal.h"
#include "st_mfma.h"

namespace st {
namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ int visible_keys(int causal, int Sk, int64_t qpos, int64_t k0) {
  if (!causal) return Sk;
  const int64_t n = qpos - k0 + 1;
  return n < 0 ? 0 : (n > Sk ? Sk : (int)n);
}

// =============================================================================================
// dQ kernel
// =============================================================================================
#ifndef ST_DQ_WQ
#define ST_DQ_WQ 32
#endif
#ifndef ST_DKV_WK
#define ST_DKV_WK 32
#endif
constexpr int kQ_BN = 64;        // keys per staged tile
constexpr int kQ_WQ = ST_DQ_WQ;  // queries per wavefront (32: two workgroups per CU)
constexpr int kQ_BM = 4 * kQ_WQ;

template <int D>
__global__ __launch_bounds__(256, kQ_WQ == 32 ? 2 : 1) void bwd_dq_bf16_kernel(const BwdArgs a) {
  constexpr int QB = kQ_WQ / 32, KB = kQ_BN / 32, KS = D / 16, DB = D / 32;
  constexpr int kTile = kQ_BN * D * 2;           // bytes of one K (or V) tile
  __shared__ __attribute__((aligned(1024))) char smem_raw[4 * kTile];   // 2 stages x (K, V)
  ST_LDS char* smem = (ST_LDS char*)smem_raw;

  const Shape& s = a.s;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, r = lane & 31;
  const int n_qt = (s.Sq + kQ_BM - 1) / kQ_BM;
  int qt, hb;
  qtile_block(blockIdx.x, gridDim.x, n_qt, s.causal, qt, hb);
  const int h = hb % s.Hq;
  const int b = hb / s.Hq;
  const int hk = h / (s.Hq / s.Hkv);

  const int q_row0 = qt * kQ_BM + wave * kQ_WQ;
  const char* qbase = (const char*)a.q.ptr + ((int64_t)b * a.q.sb + (int64_t)h * a.q.sh) * 2;
  const char* dobase = (const char*)a.d_o.ptr + ((int64_t)b * a.d_o.sb + (int64_t)h * a.d_o.sh) * 2;
  bf16x8 qf[QB][KS], dof[QB][KS];
  float lse2[QB], dlt[QB];   // lse * log2(e) (+inf for rows that do not exist or are empty), Delta
  int64_t qpos[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int i = q_row0 + 32 * qb + r;
    qpos[qb] = q_pos(s, i);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      qf[qb][ks] = scale_bf16x8(global_frag(qbase, a.q.ss, i, s.Sq, ks, g), s.scale * kLog2e);   // Q': scores in log2 units
      dof[qb][ks] = global_frag(dobase, a.d_o.ss, i, s.Sq, ks, g);
    }
    lse2[qb] = INFINITY;
    dlt[qb] = 0.f;
    if (i < s.Sq) {
      const int64_t st = ((int64_t)b * s.Hq + h) * s.Sq + i;
      const float l = a.lse[st];
      if (l != -INFINITY) lse2[qb] = l * kLog2e;
      dlt[qb] = a.delta[st];
    }
  }
  const int wg_last_row = min(qt * kQ_BM + kQ_BM, s.Sq) - 1;
  const int wave_first_row = q_row0;

  f32x16 acc[DB][QB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[db][qb][v] = 0.f;
  constexpr float c_exp = 1.f;   // the Q operand is Q' = bf16(Q scale log2 e): the scores are exponents already

  auto chunk_tiles = [&](int c) -> int {
    const int nv = visible_keys(s.causal, s.Sk, q_pos(s, wg_last_row), a.t.k_offset[c]);
    return (nv + kQ_BN - 1) / kQ_BN;
  };
  // first tile of a chunk that is this kernel's: the leading ones may belong to the fast kernel
  const int fast_row0 = qt * kQ_BM / kDqFastRows * kDqFastRows;
  const bool fast_on = a.dq_fast && kQ_BN == kDqFastKeys && fast_row0 + kDqFastRows <= s.Sq;
  auto chunk_t0 = [&](int c) -> int {
    return fast_on ? dq_fast_tiles(s, fast_row0, a.t.k_offset[c]) : 0;
  };
  int c_cur = 0, t_cur = 0, n_cur = 0;
  while (c_cur < a.t.n && (n_cur = chunk_tiles(c_cur)) <= (t_cur = chunk_t0(c_cur))) ++c_cur;

  auto issue_load = [&](int c, int t, int stage) {
    const char* kb = (const char*)a.t.k[c] + ((int64_t)b * a.t.ksb + (int64_t)hk * a.t.ksh) * 2;
    const char* vb = (const char*)a.t.v[c] + ((int64_t)b * a.t.vsb + (int64_t)hk * a.t.vsh) * 2;
    stage_dma<D, kQ_BN>(kb, a.t.kss, t * kQ_BN, s.Sk, smem + stage * 2 * kTile, tid);
    stage_dma<D, kQ_BN>(vb, a.t.vss, t * kQ_BN, s.Sk, smem + stage * 2 * kTile + kTile, tid);
  };
  int buf = 0;
  if (c_cur < a.t.n) issue_load(c_cur, t_cur, 0);
  __syncthreads();

  while (c_cur < a.t.n) {
    int c_nxt = c_cur, t_nxt = t_cur + 1, n_nxt = n_cur;
    if (t_nxt >= n_cur) {
      ++c_nxt;
      while (c_nxt < a.t.n && (n_nxt = chunk_tiles(c_nxt)) <= (t_nxt = chunk_t0(c_nxt))) ++c_nxt;
    }
    const bool have_next = c_nxt < a.t.n;
    if (have_next) issue_load(c_nxt, t_nxt, buf ^ 1);

    const int64_t k0 = a.t.k_offset[c_cur];
    const int tile_k0 = t_cur * kQ_BN;
    const int nv_wave_min = visible_keys(s.causal, s.Sk, q_pos(s, wave_first_row), k0);
    const ST_LDS char* ktile = smem + buf * 2 * kTile;
    const ST_LDS char* vtile = ktile + kTile;
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
      const int blk_k0 = tile_k0 + 32 * kb;
      {  // every wavefront computes every block the workgroup walks; invisible pairs are masked
        f32x16 sc[QB], dp[QB];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            sc[qb][v] = 0.f;
            dp[qb][v] = 0.f;
          }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const bf16x8 kf = lds_frag<D>(ktile, 32 * kb, ks, lane);
          const bf16x8 vf = lds_frag<D>(vtile, 32 * kb, ks, lane);
#pragma unroll
          for (int qb = 0; qb < QB; ++qb) {
            sc[qb] = mfma32(kf, qf[qb][ks], sc[qb]);
            dp[qb] = mfma32(vf, dof[qb][ks], dp[qb]);
          }
        }
        const bool need_mask = blk_k0 + 32 > nv_wave_min;      // wave-uniform
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
          const int nv = visible_keys(s.causal, s.Sk, qpos[qb], k0) - blk_k0;
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            float p = __builtin_amdgcn_exp2f(fmaf(sc[qb][v], c_exp, -lse2[qb]));
            if (need_mask) {
              const int key = 8 * (v / 4) + 4 * g + (v % 4);
              p = key < nv ? p : 0.f;
            }
            sc[qb][v] = p * (dp[qb][v] - dlt[qb]);             // dS^T
          }
        }
#pragma unroll
        for (int m = 0; m < 2; ++m) {
          bf16x8 dsf[QB];
#pragma unroll
          for (int qb = 0; qb < QB; ++qb) dsf[qb] = pack_c_as_b(sc[qb], m);
#pragma unroll
          for (int db = 0; db < DB; ++db) {
            const bf16x8 ktf = lds_frag_tr<D>(ktile, 32 * kb + 16 * m, 32 * db, lane);
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) acc[db][qb] = mfma32(ktf, dsf[qb], acc[db][qb]);
          }
        }
      }
    }

    __syncthreads();
    buf ^= 1;
    c_cur = c_nxt;
    t_cur = t_nxt;
    n_cur = n_nxt;
  }

  // dq_acc += scale * dQ   (this workgroup is the only writer of its rows in this launch)
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int i = q_row0 + 32 * qb + r;
    if (i < s.Sq) {
      float* orow = a.dq + (((int64_t)b * s.Sq + i) * s.Hq + h) * D;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          float4* p = reinterpret_cast<float4*>(orow + 32 * db + 8 * q4 + 4 * g);
          float4 o = *p;
          o.x += s.scale * acc[db][qb][4 * q4 + 0];
          o.y += s.scale * acc[db][qb][4 * q4 + 1];
          o.z += s.scale * acc[db][qb][4 * q4 + 2];
          o.w += s.scale * acc[db][qb][4 * q4 + 3];
          *p = o;
        }
    }
  }
}

// =============================================================================================
// dK / dV kernel
// =============================================================================================
constexpr int kK_WK = ST_DKV_WK;  // keys per wavefront (32: two workgroups per CU)
constexpr int kK_BK = 4 * kK_WK;  // keys per workgroup
constexpr int kK_BQ = ST_DKV_WK == 32 ? 32 : 64;   // queries per staged tile

template <int D>
__global__ __launch_bounds__(256, 1) void bwd_dkv_bf16_kernel(const BwdArgs a) {
  constexpr int NB = kK_WK / 32;   // 32-key blocks per wavefront
  constexpr int QB = kK_BQ / 32;   // 32-query blocks per staged tile
  constexpr int KS = D / 16, DB = D / 32;
  constexpr int kTile = kK_BQ * D * 2;
  // 2 stages x (Q tile, dO tile, lse2[64], delta[64])
  constexpr int kStage = 2 * kTile + 2 * kK_BQ * 4;
  __shared__ __attribute__((aligned(16))) char smem_raw[2 * kStage];
  ST_LDS char* smem = (ST_LDS char*)smem_raw;

  const Shape& s = a.s;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, r = lane & 31;
  const int G = s.Hq / s.Hkv;
  const int n_kt = (s.Sk + kK_BK - 1) / kK_BK;
  // logical order: key tile fastest, then chunk, then batch, KV head slowest: with the XCD mapping
  // a KV head (and the Q, dO of its query heads) stays on one XCD's L2 when Hkv * B % 8 == 0.  The launcher
  // sorts a causal table by position, so inside a head the workgroups come in order of falling work
  // (earlier keys are seen by more query rows) and the tail of the launch stays short.
  const int logical = xcd_logical_block(blockIdx.x, gridDim.x);
  const int kt = logical % n_kt;
  const int c = (logical / n_kt) % a.t.n;
  const int b = (logical / (a.t.n * n_kt)) % s.B;
  const int hk = logical / (a.t.n * n_kt * s.B);

  const int64_t k0 = a.t.k_offset[c];
  const int wg_key0 = kt * kK_BK;
  const int wave_key0 = wg_key0 + wave * kK_WK;

  // first query row that can see the first key of this workgroup / wavefront
  int wg_i0 = 0;
  if (s.causal) {
    wg_i0 = q_row_of(s, k0 + wg_key0);
    if (wg_i0 >= s.Sq) return;
  }
  const int q_tile_first = wg_i0 / kK_BQ;
  const int n_q_tiles = (s.Sq + kK_BQ - 1) / kK_BQ;
  if (q_tile_first >= n_q_tiles) return;
  // Query blocks of this workgroup: [q_tile_first, q_split) and [q_resume, n_q_tiles).  The gap, if any,
  // belongs to the fast kernel (full blocks that see every key of the enclosing full 256-key tile).
  int q_split = n_q_tiles, q_resume = n_q_tiles;
  if (a.dkv_fast && kK_BQ == kDkvFastRows) {
    const int tile_key0 = wg_key0 / kDkvFastKeys * kDkvFastKeys;
    if (tile_key0 + kDkvFastKeys <= s.Sk) {
      const int fb = dkv_fast_first_block(s, k0, tile_key0), n_full = s.Sq / kDkvFastRows;
      if (fb < n_full) {
        q_split = fb > q_tile_first ? fb : q_tile_first;
        q_resume = n_full;
      }
    }
  }

  // resident K, V fragments (B operands, column = key)
  const char* kbase = (const char*)a.t.k[c] + ((int64_t)b * a.t.ksb + (int64_t)hk * a.t.ksh) * 2;
  const char* vbase = (const char*)a.t.v[c] + ((int64_t)b * a.t.vsb + (int64_t)hk * a.t.vsh) * 2;
  bf16x8 kf[NB][KS], vf[NB][KS];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      kf[nb][ks] = global_frag(kbase, a.t.kss, wave_key0 + 32 * nb + r, s.Sk, ks, g);
      vf[nb][ks] = global_frag(vbase, a.t.vss, wave_key0 + 32 * nb + r, s.Sk, ks, g);
    }
  int kpos_rel[NB];       // first query row that sees the key: row i sees it iff i >= kpos_rel
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) kpos_rel[nb] = q_row_of(s, k0 + wave_key0 + 32 * nb + r);

  f32x16 acc_k[DB][NB], acc_v[DB][NB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        acc_k[db][nb][v] = 0.f;
        acc_v[db][nb][v] = 0.f;
      }
  constexpr float c_exp = 1.f;   // the Q operand is Q' = bf16(Q scale log2 e): the scores are exponents already

  // flattened (head of the group, query tile) walk
  const int n_head_lo = q_split - q_tile_first;
  const int tiles_per_head = n_head_lo + (n_q_tiles - q_resume);
  if (tiles_per_head <= 0) return;
  const int n_steps = G * tiles_per_head;
  auto tile_of = [&](int step) -> int {
    const int j = step % tiles_per_head;
    return j < n_head_lo ? q_tile_first + j : q_resume + (j - n_head_lo);
  };
  StageRegs<D, kK_BQ> rq, rdo;
  float stat_reg = 0.f;   // threads 0..63: lse2 of row tid; threads 64..127: delta of row tid-64
  auto issue_load = [&](int step) {
    const int h = hk * G + step / tiles_per_head;
    const int i0 = tile_of(step) * kK_BQ;
    const char* qb_ = (const char*)a.q.ptr + ((int64_t)b * a.q.sb + (int64_t)h * a.q.sh) * 2;
    const char* dob_ = (const char*)a.d_o.ptr + ((int64_t)b * a.d_o.sb + (int64_t)h * a.d_o.sh) * 2;
    // the Q tile holds Q' = bf16(Q scale log2 e), converted here in the staging registers: the scores come out
    // in log2 units, and dK^T = Q'^T dS carries a factor scale log2 e (the epilogue multiplies by ln 2, not by scale)
    stage_load<D, kK_BQ>(rq, qb_, a.q.ss, i0, s.Sq, tid);
#pragma unroll
    for (int j = 0; j < StageRegs<D, kK_BQ>::kN; ++j) rq.x[j] = scale_bf16x8(rq.x[j], s.scale * kLog2e);
    stage_load<D, kK_BQ>(rdo, dob_, a.d_o.ss, i0, s.Sq, tid);
    if (tid < 2 * kK_BQ) {
      const int row = i0 + (tid & (kK_BQ - 1));
      const int64_t st = ((int64_t)b * s.Hq + h) * s.Sq + row;
      if (tid < kK_BQ) {
        float l = INFINITY;                       // rows that do not exist or are empty give P = 0
        if (row < s.Sq) {
          const float x = a.lse[st];
          if (x != -INFINITY) l = x * kLog2e;
        }
        stat_reg = l;
      } else {
        stat_reg = row < s.Sq ? a.delta[st] : 0.f;
      }
    }
  };
  auto store_stage = [&](int bufi) {
    ST_LDS char* st = smem + bufi * kStage;
    stage_store<D, kK_BQ>(rq, st, tid);
    stage_store<D, kK_BQ>(rdo, st + kTile, tid);
    if (tid < 2 * kK_BQ) reinterpret_cast<ST_LDS float*>(st + 2 * kTile)[tid] = stat_reg;
  };

  issue_load(0);
  store_stage(0);
  __syncthreads();
  int buf = 0;
  for (int step = 0; step < n_steps; ++step) {
    const bool have_next = step + 1 < n_steps;
    if (have_next) issue_load(step + 1);

    const int i0 = tile_of(step) * kK_BQ;
    const ST_LDS char* qtile = smem + buf * kStage;
    const ST_LDS char* dotile = qtile + kTile;
    const ST_LDS float* lse_s = reinterpret_cast<const ST_LDS float*>(qtile + 2 * kTile);
    const ST_LDS float* dlt_s = lse_s + kK_BQ;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const int blk_i0 = i0 + 32 * qb;
      {  // every block of the walk is computed; (row, key) pairs that are not visible are masked
        f32x16 sc[NB], dp[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            sc[nb][v] = 0.f;
            dp[nb][v] = 0.f;
          }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const bf16x8 qa = lds_frag<D>(qtile, 32 * qb, ks, lane);
          const bf16x8 da = lds_frag<D>(dotile, 32 * qb, ks, lane);
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) {
            sc[nb] = mfma32(qa, kf[nb][ks], sc[nb]);
            dp[nb] = mfma32(da, vf[nb][ks], dp[nb]);
          }
        }
        // per-row statistics for the 16 rows this lane holds: rows 8j + 4g + {0..3}
        f32x4 lrow[4], drow[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          lrow[j] = *reinterpret_cast<const ST_LDS f32x4*>(lse_s + 32 * qb + 8 * j + 4 * g);
          drow[j] = *reinterpret_cast<const ST_LDS f32x4*>(dlt_s + 32 * qb + 8 * j + 4 * g);
        }
        // wave-uniform: is some (row, key) pair of this block masked?
        const bool need_mask = s.causal && (q_pos(s, blk_i0) < k0 + wave_key0 + kK_WK - 1);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          const int first_row = kpos_rel[nb] - blk_i0;     // block row index from which the key is visible
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            float p = __builtin_amdgcn_exp2f(fmaf(sc[nb][v], c_exp, -lrow[v / 4][v % 4]));
            if (need_mask) {
              const int row = 8 * (v / 4) + 4 * g + (v % 4);
              p = row >= first_row ? p : 0.f;
            }
            sc[nb][v] = p;
            dp[nb][v] = p * (dp[nb][v] - drow[v / 4][v % 4]);
          }
        }
#pragma unroll
        for (int m = 0; m < 2; ++m) {
          bf16x8 pf[NB], dsf[NB];
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) {
            pf[nb] = pack_c_as_b(sc[nb], m);
            dsf[nb] = pack_c_as_b(dp[nb], m);
          }
#pragma unroll
          for (int db = 0; db < DB; ++db) {
            const bf16x8 dot = lds_frag_tr<D>(dotile, 32 * qb + 16 * m, 32 * db, lane);
            const bf16x8 qt_ = lds_frag_tr<D>(qtile, 32 * qb + 16 * m, 32 * db, lane);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
              acc_v[db][nb] = mfma32(dot, pf[nb], acc_v[db][nb]);
              acc_k[db][nb] = mfma32(qt_, dsf[nb], acc_k[db][nb]);
            }
          }
        }
      }
    }

    if (have_next) store_stage(buf ^ 1);
    __syncthreads();
    buf ^= 1;
  }

  // dk_acc += scale * dS^T Q = ln 2 * dS^T Q' (Q' = Q scale log2 e), dv_acc += dV  (single owner of these key rows)
  const float k_mul = kLn2;
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const int t = wave_key0 + 32 * nb + r;
    if (t < s.Sk) {
      const int64_t row = (((int64_t)b * s.Sk + t) * s.Hkv + hk) * D;
      float* dkr = a.dk[c] + row;
      float* dvr = a.dv[c] + row;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int d = 32 * db + 8 * q4 + 4 * g;
          float4 x = *reinterpret_cast<float4*>(dkr + d);
          x.x += k_mul * acc_k[db][nb][4 * q4 + 0];
          x.y += k_mul * acc_k[db][nb][4 * q4 + 1];
          x.z += k_mul * acc_k[db][nb][4 * q4 + 2];
          x.w += k_mul * acc_k[db][nb][4 * q4 + 3];
          *reinterpret_cast<float4*>(dkr + d) = x;
          float4 y = *reinterpret_cast<float4*>(dvr + d);
          y.x += acc_v[db][nb][4 * q4 + 0];
          y.y += acc_v[db][nb][4 * q4 + 1];
          y.z += acc_v[db][nb][4 * q4 + 2];
          y.w += acc_v[db][nb][4 * q4 + 3];
          *reinterpret_cast<float4*>(dvr + d) = y;
        }
    }
  }
}

}  // namespace

hipError_t launch_bwd_bf16(const BwdArgs& a_in, hipStream_t stream) {
  BwdArgs a = a_in;
  if (a.t.n <= 0 || a.s.Sq <= 0 || a.s.Sk <= 0) return hipSuccess;
  const int n_qt = (a.s.Sq + kQ_BM - 1) / kQ_BM;
  const int64_t total_q = (int64_t)n_qt * a.s.Hq * a.s.B;
  const int n_kt = (a.s.Sk + kK_BK - 1) / kK_BK;
  const int64_t total_k = (int64_t)n_kt * a.s.Hkv * a.s.B * a.t.n;
  if (total_q > 0x7fffffff || total_k > 0x7fffffff) return hipErrorInvalidValue;
  if (a.s.D != 128 && a.s.D != 64) return hipErrorInvalidValue;
  a.dkv_fast = (knobs().dkv_fast && dkv_fast_usable(a)) ? 1 : 0;
  if (a.s.causal) {
    // earlier chunks first (the backward does not depend on the order of the table): their keys are seen by
    // more query rows, and workgroups are handed out in table order
    for (int i = 1; i < a.t.n; ++i)
      for (int j = i; j > 0 && a.t.k_offset[j] < a.t.k_offset[j - 1]; --j) {
        std::swap(a.t.k[j], a.t.k[j - 1]);
        std::swap(a.t.v[j], a.t.v[j - 1]);
        std::swap(a.t.k_offset[j], a.t.k_offset[j - 1]);
        std::swap(a.dk[j], a.dk[j - 1]);
        std::swap(a.dv[j], a.dv[j - 1]);
        std::swap(a.dk_lowp[j], a.dk_lowp[j - 1]);
        std::swap(a.dv_lowp[j], a.dv_lowp[j - 1]);
        const uint64_t bj = (a.kv_assign >> j) & 1, bi = (a.kv_assign >> (j - 1)) & 1;
        a.kv_assign = (a.kv_assign & ~((1ull << j) | (1ull << (j - 1)))) | (bi << j) | (bj << (j - 1));
      }
  }
  // Assignment and bf16 copies can be left to the fast dK/dV kernel for the chunks it alone writes: full tiles
  // only, every query row sees every key.  Every other chunk is zeroed here first (then added to as usual) and
  // cast by a launch of its own at the end.
  const int64_t n_kv = (int64_t)a.s.B * a.s.Sk * a.s.Hkv * a.s.D;
  void* cast_dk[kMaxTable];
  void* cast_dv[kMaxTable];
  for (int c = 0; c < a.t.n; ++c) {
    cast_dk[c] = cast_dv[c] = nullptr;
    const bool fast_only = a.dkv_fast && dkv_chunk_fast_only(a.s, a.t.k_offset[c]);
    if (fast_only && ((a.dk_lowp[c] == nullptr) == (a.dv_lowp[c] == nullptr))) continue;
    if ((a.kv_assign >> c) & 1) {
      hipError_t ez = launch_zero(a.dk[c], n_kv * (int64_t)sizeof(float), stream);
      if (ez == hipSuccess) ez = launch_zero(a.dv[c], n_kv * (int64_t)sizeof(float), stream);
      if (ez != hipSuccess) return ez;
      a.kv_assign &= ~(1ull << c);
    }
    cast_dk[c] = a.dk_lowp[c];
    cast_dv[c] = a.dv_lowp[c];
    a.dk_lowp[c] = a.dv_lowp[c] = nullptr;
  }
  hipError_t e = hipSuccess;
  {
    // With the fast kernel on, the general one only has the masked and ragged blocks left: chunks whose every
    // block is the fast kernel's (dkv_chunk_fast_only) are left out of its grid, which would otherwise consist
    // mostly of workgroups that find nothing to do.
    BwdArgs g = a;
    if (a.dkv_fast) {
      g.t.n = 0;
      for (int c = 0; c < a.t.n; ++c) {
        if (dkv_chunk_fast_only(a.s, a.t.k_offset[c])) continue;
        g.t.k[g.t.n] = a.t.k[c];
        g.t.v[g.t.n] = a.t.v[c];
        g.t.k_offset[g.t.n] = a.t.k_offset[c];
        g.dk[g.t.n] = a.dk[c];
        g.dv[g.t.n] = a.dv[c];
        ++g.t.n;
      }
    }
    if (g.t.n > 0) {
      ProfScope prof(a.dkv_fast ? "bwd_dkv_edge" : "bwd_dkv_bf16", stream);
      const unsigned grid = (unsigned)((int64_t)n_kt * a.s.Hkv * a.s.B * g.t.n);
      if (a.s.D == 128) hipLaunchKernelGGL(bwd_dkv_bf16_kernel<128>, dim3(grid), dim3(256), 0, stream, g);
      else hipLaunchKernelGGL(bwd_dkv_bf16_kernel<64>, dim3(grid), dim3(256), 0, stream, g);
      e = hipGetLastError();
    }
  }
  if (e != hipSuccess) return e;
  if (a.dkv_fast) {
    e = launch_bwd_dkv_fast(a, stream);
    if (e != hipSuccess) return e;
  }
  for (int c = 0; c < a.t.n; ++c) {
    if (cast_dk[c]) e = launch_cast(a.dk[c], cast_dk[c], n_kv, ST_BF16, stream);
    if (e == hipSuccess && cast_dv[c]) e = launch_cast(a.dv[c], cast_dv[c], n_kv, ST_BF16, stream);
    if (e != hipSuccess) return e;
  }
  a.dq_fast = (knobs().dq_fast && dq_fast_usable(a)) ? 1 : 0;
  {
    ProfScope prof(a.dq_fast ? "bwd_dq_edge" : "bwd_dq_bf16", stream);
    if (a.s.D == 128) hipLaunchKernelGGL(bwd_dq_bf16_kernel<128>, dim3((unsigned)total_q), dim3(256), 0, stream, a);
    else hipLaunchKernelGGL(bwd_dq_bf16_kernel<64>, dim3((unsigned)total_q), dim3(256), 0, stream, a);
  }
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (a.dq_fast) return launch_bwd_dq_fast(a, stream);
  return hipSuccess;
}

}  // namespace st
