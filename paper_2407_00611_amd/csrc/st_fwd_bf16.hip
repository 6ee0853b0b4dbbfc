// bf16 forward, general kernels and the launcher of the whole forward.  The general kernel's body lives in
// st_fwd_general.h (it also runs side by side with the hand-scheduled loop in one launch, see st_fwd_fast.hip);
// this file wraps it as a kernel of its own, holds the software-pipelined variant used when the hand-scheduled
// loop is switched off, and picks the kernels of a launch.  One launch with a 1-entry table is
// st_attn_block_fwd; with the full table it is the fused ring forward.
#include <cstdlib>
#include <type_traits>

#include "st_internal.h"
#include "st_mfma.h"
#include "st_fwd_general.h"

namespace st {
namespace {

template <int D, int kWQ>
__global__ __launch_bounds__(256, kWQ == 32 ? 2 : 1) void fwd_bf16_kernel(const FwdArgs a) {
  __shared__ __attribute__((aligned(1024))) char smem_raw[4 * kBN * D * 2];   // 2 stages x (K, V)
  fwd_general_body<D, kWQ>(a, blockIdx.x, gridDim.x, blockIdx.y, smem_raw);
}


// =============================================================================================
// Software-pipelined forward: one wavefront per SIMD, 64 queries per wavefront, and the MFMA and
// VALU streams of neighbouring tiles interleaved by hand, one MFMA "slot" at a time:
//   iteration t:  block 1 = S^T(t+1) MFMAs   with  exp / row-sum / bf16-pack of tile t
//                 block 2 = O^T += V^T P^T(t) MFMAs  with the rest of tile t and the row max of t+1
// A wavefront issues in order, so an MFMA followed by a handful of independent VALU instructions
// keeps both pipes busy; the scheduling fences pin that order.  K/V tiles arrive by asm DMA into a
// four-stage LDS ring, three tiles ahead.
// =============================================================================================
#define ST_FENCE() __builtin_amdgcn_sched_barrier(0)

struct TileCursor {
  int c, t, n;   // chunk index in the table, tile in the chunk, tiles the workgroup needs from the chunk
};

template <int D>
__global__ __launch_bounds__(256, 1) void fwd_pipe_kernel(const FwdArgs a) {
  constexpr int kWQ = 64, kBM = 256, QB = 2, KS = D / 16, DB = D / 32, NS = 4;
  constexpr int kTile = kBN * D * 2, kStage = 2 * kTile;
  constexpr int kDmaPerTile = 2 * DmaPlan<D, kBN>::PER_WAVE;   // K + V instructions per wavefront
  __shared__ __attribute__((aligned(1024))) char smem_raw[NS * kStage];
  ST_LDS char* smem = (ST_LDS char*)smem_raw;
  const uint32_t smem_addr = (uint32_t)(uintptr_t)smem;

  const Shape& s = a.s;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, r = lane & 31;
  const int n_qt = (s.Sq + kBM - 1) / kBM;
  int qt, hb;
  qtile_block(blockIdx.x, gridDim.x, n_qt, s.causal, qt, hb);
  const int h = hb % s.Hq;
  const int b = hb / s.Hq;
  const int hk = h / (s.Hq / s.Hkv);

  const int q_row0 = qt * kBM + wave * kWQ;
  const char* qbase = (const char*)a.q.ptr + ((int64_t)b * a.q.sb + (int64_t)h * a.q.sh) * 2;
  bf16x8 qf[QB][KS];
  int64_t qpos[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int i = q_row0 + 32 * qb + r;
    qpos[qb] = q_pos(s, i);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[qb][ks] = scale_bf16x8(global_frag(qbase, a.q.ss, i, s.Sq, ks, g), s.scale * kLog2e);
  }
  const int wg_last_row = min(qt * kBM + kBM, s.Sq) - 1;
  const int wave_first_row = q_row0;

  f32x16 acc_o[DB][QB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc_o[db][qb][v] = 0.f;
  float m_run[QB] = {-INFINITY, -INFINITY}, l_run[QB] = {0.f, 0.f};
  constexpr float c_exp = 1.f;   // Q fragments are Q' = bf16(Q scale log2 e): the scores are exponents already

  // ---- tile walk: cursors for the tile in softmax / PV (cur), in S (nxt) and in flight by DMA (dma)
  auto chunk_tiles = [&](int c) -> int {
    const int nv = visible_keys(s.causal, s.Sk, q_pos(s, wg_last_row), a.t.k_offset[c]);
    return (nv + kBN - 1) / kBN;
  };
  auto first_tile = [&]() -> TileCursor {
    TileCursor x{0, 0, 0};
    while (x.c < a.t.n && (x.n = chunk_tiles(x.c)) == 0) ++x.c;
    return x;
  };
  auto advance = [&](TileCursor x) -> TileCursor {
    if (x.c >= a.t.n) return x;
    if (++x.t >= x.n) {
      x.t = 0;
      ++x.c;
      while (x.c < a.t.n && (x.n = chunk_tiles(x.c)) == 0) ++x.c;
    }
    return x;
  };
  auto valid = [&](const TileCursor& x) { return x.c < a.t.n; };
  auto issue_dma = [&](const TileCursor& x, int stage) {
    const char* kb = (const char*)a.t.k[x.c] + ((int64_t)b * a.t.ksb + (int64_t)hk * a.t.ksh) * 2;
    const char* vb = (const char*)a.t.v[x.c] + ((int64_t)b * a.t.vsb + (int64_t)hk * a.t.vsh) * 2;
    stage_dma_asm<D, kBN>(kb, a.t.kss, x.t * kBN, s.Sk, smem_addr + stage * kStage, tid);
    stage_dma_asm<D, kBN>(vb, a.t.vss, x.t * kBN, s.Sk, smem_addr + stage * kStage + kTile, tid);
  };

  TileCursor cur = first_tile();
  if (valid(cur)) {
    TileCursor nxt = advance(cur);
    TileCursor dma = advance(nxt);
    // Q fragment loads were issued above; then tiles 0, 1, 2 of the walk
    issue_dma(cur, 0);
    if (valid(nxt)) issue_dma(nxt, 1);
    if (valid(dma)) issue_dma(dma, 2);
    // all but the last two DMA groups (and every earlier load) have landed
    if (valid(dma)) wait_vmcnt<2 * kDmaPerTile>();
    else if (valid(nxt)) wait_vmcnt<kDmaPerTile>();
    else wait_vmcnt<0>();
    __syncthreads();
    dma = advance(dma);   // next tile to request (stage 3)

    // ---- per-lane LDS byte offsets inside a tile (see swz): the XOR swizzle is not affine in the
    // fragment indices, so one offset per k-step (natural reads) and per d-block (transpose reads) is
    // kept in a register; 32-row block offsets are immediates.
    constexpr int ROWB = D * 2;
    uint32_t nat_off[KS], tr_lo[DB], tr_hi[DB];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) nat_off[ks] = (uint32_t)swz<D>(r, 2 * ks + g);
    {
      const int s16 = lane & 15, half = (lane >> 4) & 1;
      const int row = 4 * g + (s16 >> 2), lc = 2 * half + ((s16 & 3) >> 1), sub = (s16 & 1) * 8;
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        tr_lo[db] = (uint32_t)(swz<D>(row, 4 * db + lc) + sub);
        tr_hi[db] = (uint32_t)(swz<D>(row + 8, 4 * db + lc) + sub);
      }
    }
    auto k_frag = [&](uint32_t ktile_addr, int kb, int ks) -> bf16x8 {
      return lds_read_b128((const ST_LDS char*)(uintptr_t)(ktile_addr + nat_off[ks]) + 32 * kb * ROWB);
    };
    auto v_frag = [&](uint32_t vtile_addr, int row0, int db) -> bf16x8 {     // row0 % 16 == 0
      const u32x2 lo = lds_read_tr16((const ST_LDS char*)(uintptr_t)(vtile_addr + tr_lo[db]) + row0 * ROWB);
      const u32x2 hi = lds_read_tr16((const ST_LDS char*)(uintptr_t)(vtile_addr + tr_hi[db]) + row0 * ROWB);
      return __builtin_bit_cast(bf16x8, u32x4{lo[0], lo[1], hi[0], hi[1]});
    };

    // Scores of a 32-key block travel between half-iterations as plain VGPR floats: the MFMA that makes
    // them accumulates in AGPRs, the VALU (max, exp) only reads VGPRs, so each score is moved exactly once.
    float sA[QB][16], sB[QB][16];
    float mxn[QB];           // row maxima of the next block

    // mask (if the causal / ragged edge crosses it) the 32-key block kb of tile x held in the accumulators
    auto mask_block = [&](f32x16 (&sc)[QB], const TileCursor& x, int kb) {
      const int64_t k0 = a.t.k_offset[x.c];
      const int blk_k0 = x.t * kBN + 32 * kb;
      const int nv_min = visible_keys(s.causal, s.Sk, q_pos(s, wave_first_row), k0);
      if (blk_k0 + 32 > nv_min) {                                // wave-uniform, rare
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
          mask_rows_in_place(sc[qb], visible_keys(s.causal, s.Sk, qpos[qb], k0) - blk_k0 - 4 * g);
      }
    };
    auto rescale_if_needed = [&](bool jump) {
      if (__builtin_expect(__any(jump), 0)) {                    // wave-uniform, rare after the first tiles
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
          const float m_new = fmaxf(m_run[qb], mxn[qb]);
          const float m_use = m_new == -INFINITY ? 0.f : m_new;
          const float alpha = __builtin_amdgcn_exp2f((m_run[qb] - m_use) * c_exp);
          l_run[qb] *= alpha;
          m_run[qb] = m_new;
#pragma unroll
          for (int db = 0; db < DB; ++db) scale_in_place(acc_o[db][qb], alpha);
        }
      }
    };
    auto jump_of = [&](int qb) -> bool {
      return (mxn[qb] - m_run[qb]) * c_exp > kRescaleGap || (m_run[qb] == -INFINITY && mxn[qb] != -INFINITY);
    };

    // ---- prologue: S^T of block 0 of tile 0, its mask, maxima and the first (always taken) rescale
    {
      f32x16 s0[QB];
#pragma unroll
      for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int v = 0; v < 16; ++v) s0[qb][v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8 kf = k_frag(smem_addr, 0, ks);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) s0[qb] = mfma32(kf, qf[qb][ks], s0[qb]);
      }
      mask_block(s0, cur, 0);
      bool jump = false;
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
#pragma unroll
        for (int v = 0; v < 16; ++v) sA[qb][v] = s0[qb][v];
        float x = sA[qb][0];
#pragma unroll
        for (int v = 1; v < 16; ++v) x = fmaxf(x, sA[qb][v]);
        mxn[qb] = xhalf_max(x);
        jump = jump || jump_of(qb);
      }
      rescale_if_needed(jump);
    }

    // ---- one pipelined half-iteration.
    //   sc: scores of the block in softmax (block kbc of the tile whose V is at vtile_addr), consumed
    //   sv: scores of the following block (block kbn of the tile whose K is at ktile_addr), produced
    auto half_iteration = [&](float (&sc)[QB][16], float (&sv)[QB][16], uint32_t vtile_addr, int kbc,
                              uint32_t ktile_addr, int kbn, const TileCursor& xn, bool xn_valid) {
      float mc[QB], psum[QB] = {0.f, 0.f};
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) mc[qb] = (m_run[qb] == -INFINITY ? 0.f : m_run[qb]) * c_exp;
      // Register-file hint: the Q fragments only ever feed MFMAs, which also read AGPRs; keeping them
      // there leaves the VGPRs to the values the VALU touches.
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+a"(qf[0][ks]), "+a"(qf[1][ks]));
      u32x4 pf[2][QB];   // P^T packed to bf16 per 16-key group m and query block
      float pv[32];   // exp results in flight between the slot that issues them and the slot that retires them
      // Element e of the exp stream: group m = e / 16, query block (e / 8) % 2, value j = e % 8.
      // A wavefront issues in order, so the use of a transcendental result right behind its v_exp
      // stalls everything that follows, MFMAs included: the exponentials of one slot are issued together
      // and retired (row sum, bf16 pack) one slot later.
      // The empty asm statements pin this otherwise pure arithmetic between the scheduling fences of
      // its slot: instruction selection orders side-effect-free code freely, and the fences only bind
      // the later machine scheduler.
      auto exp_issue = [&](int e0, int e1) {     // at most three elements per slot
        float x[3] = {0.f, 0.f, 0.f};
#pragma unroll
        for (int e = e0; e < e1; ++e) x[e - e0] = sc[(e / 8) % 2][8 * (e / 16) + e % 8];
        if (e1 - e0 == 3) asm volatile("" : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]));
        else if (e1 - e0 == 2) asm volatile("" : "+v"(x[0]), "+v"(x[1]));
        else if (e1 - e0 == 1) asm volatile("" : "+v"(x[0]));
#pragma unroll
        for (int e = e0; e < e1; ++e) x[e - e0] = __builtin_amdgcn_exp2f(fmaf(x[e - e0], c_exp, -mc[(e / 8) % 2]));
        if (e1 - e0 == 3) asm volatile("" : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]));
        else if (e1 - e0 == 2) asm volatile("" : "+v"(x[0]), "+v"(x[1]));
        else if (e1 - e0 == 1) asm volatile("" : "+v"(x[0]));
#pragma unroll
        for (int e = e0; e < e1; ++e) pv[e] = x[e - e0];
      };
      auto exp_retire = [&](int e0, int e1) {
#pragma unroll
        for (int e = e0; e < e1; ++e) {
          const int m = e / 16, qb = (e / 8) % 2, j = e % 8;
          psum[qb] += pv[e];
          if (j % 2 == 1) pf[m][qb][j / 2] = pack_bf16(pv[e - 1], pv[e]);
        }
        if (e1 > e0) asm volatile("" : "+v"(psum[0]), "+v"(psum[1]));
      };
      // slot schedule: elements [lo(i), lo(i+1)) are issued in slot i and retired in slot i + 1
      auto exp_slot = [&](int lo_prev, int lo_cur, int lo_next) {
        exp_issue(lo_cur, lo_next);
        // retire in pairs so that a bf16 pack always sees both halves
        exp_retire(lo_prev & ~1, lo_cur & ~1);
      };
      f32x16 sn[QB];   // S^T accumulators of the following block
#pragma unroll
      for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int v = 0; v < 16; ++v) sn[qb][v] = 0.f;

      // ---- block 1: S^T(next block) = K Q^T, 2 KS slots, with exp elements 0..19
      constexpr int kS1 = 2 * KS;
      bf16x8 kf[3];
      kf[0] = k_frag(ktile_addr, kbn, 0);
      kf[1] = k_frag(ktile_addr, kbn, 1);
      ST_FENCE();
#pragma unroll
      for (int i = 0; i < kS1; ++i) {
        const int ks = i / 2, qb = i % 2;
        if (qb == 0 && ks + 2 < KS) kf[(ks + 2) % 3] = k_frag(ktile_addr, kbn, ks + 2);
        sn[qb] = mfma32(kf[ks % 3], qf[qb][ks], sn[qb]);
        ST_FENCE();
        exp_slot(i == 0 ? 0 : 20 * (i - 1) / kS1, 20 * i / kS1, 20 * (i + 1) / kS1);
        ST_FENCE();
      }
      if (xn_valid) mask_block(sn, xn, kbn);
      ST_FENCE();

      // ---- block 2: O^T += V^T P^T, 4 DB slots: exp elements 20..31 in its first half, then the
      // next block's scores are moved to VGPRs (sv) and their row maxima taken
      constexpr int kS2 = 4 * DB, kExp2 = kS2 / 2;
      bf16x8 vf[3];
      vf[0] = v_frag(vtile_addr, 32 * kbc, 0);
      vf[1] = v_frag(vtile_addr, 32 * kbc, 1);
      float mxa[QB] = {-INFINITY, -INFINITY}, mxb[QB] = {-INFINITY, -INFINITY};   // two chains per query block
      ST_FENCE();
#pragma unroll
      for (int i = 0; i < kS2; ++i) {
        const int m = i / (2 * DB), db = (i / 2) % DB, qb = i % 2, f = i / 2;   // fragment f = m * DB + db
        if (qb == 0 && f + 2 < 2 * DB) vf[(f + 2) % 3] = v_frag(vtile_addr, 32 * kbc + 16 * ((f + 2) / DB), (f + 2) % DB);
        acc_o[db][qb] = mfma32(vf[f % 3], __builtin_bit_cast(bf16x8, pf[m][qb]), acc_o[db][qb]);
        ST_FENCE();
        if (i < kExp2) {
          exp_slot(i == 0 ? 20 * (kS1 - 1) / kS1 : 20 + 12 * (i - 1) / kExp2, 20 + 12 * i / kExp2, 20 + 12 * (i + 1) / kExp2);
        } else {
          if (i == kExp2) exp_retire((20 + 12 * (kExp2 - 1) / kExp2) & ~1, 32);
          // 16 pairs (8 per query block) of the next block's scores: to VGPRs, max3 per pair
          const int j = i - kExp2, n2 = kS2 - kExp2, per = (16 + n2 - 1) / n2;
#pragma unroll
          for (int u = j * per; u < (j + 1) * per && u < 16; ++u) {
            const int qq = u / 8, w = u % 8;
            float y0 = sn[qq][2 * w], y1 = sn[qq][2 * w + 1];
            asm volatile("" : "+v"(y0), "+v"(y1));
            sv[qq][2 * w] = y0;
            sv[qq][2 * w + 1] = y1;
            if (w < 4) mxa[qq] = fmaxf(fmaxf(mxa[qq], y0), y1);
            else mxb[qq] = fmaxf(fmaxf(mxb[qq], y0), y1);
          }
          asm volatile("" : "+v"(mxa[0]), "+v"(mxa[1]), "+v"(mxb[0]), "+v"(mxb[1]));
        }
        ST_FENCE();
      }
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) l_run[qb] += psum[qb];
      bool jump = false;
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        mxn[qb] = xhalf_max(fmaxf(mxa[qb], mxb[qb]));
        jump = jump || jump_of(qb);
      }
      rescale_if_needed(jump && xn_valid);
    };

    int stage = 0;   // LDS stage of the current tile; the next tile sits in stage + 1, the DMA goes to stage + 3
    while (true) {
      const bool have_dma = valid(dma);
      if (have_dma) issue_dma(dma, (stage + 3) & (NS - 1));
      const uint32_t cur_addr = smem_addr + stage * kStage, nxt_addr = smem_addr + ((stage + 1) & (NS - 1)) * kStage;
      // blocks (cur,0) -> (cur,1) -> (nxt,0)
      half_iteration(sA, sB, cur_addr + kTile, 0, cur_addr, 1, cur, true);
      half_iteration(sB, sA, cur_addr + kTile, 1, nxt_addr, 0, nxt, valid(nxt));
      // the tile after next must have landed before anyone reads it; only this iteration's DMA may be in flight
      if (have_dma) wait_vmcnt<kDmaPerTile>();
      else wait_vmcnt<0>();
      __syncthreads();
      stage = (stage + 1) & (NS - 1);
      cur = nxt;
      nxt = advance(nxt);
      dma = advance(dma);
      if (!valid(cur)) break;
    }
  }

  // ---- epilogue: O = acc / l, lse = m ln 2 + ln(l)
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
      if (g == 0) a.lse[((int64_t)b * s.Hq + h) * s.Sq + i] = l > 0.f ? m_run[qb] * kLn2 + logf(l) : -INFINITY;
    }
  }
}

}  // namespace

hipError_t launch_fwd_pipe(const FwdArgs& a, hipStream_t stream) {
  constexpr int kBM = 256;
  const int n_qt = (a.s.Sq + kBM - 1) / kBM;
  const int64_t total = (int64_t)n_qt * a.s.Hq * a.s.B;
  if (total <= 0) return hipSuccess;
  if (total > 0x7fffffff) return hipErrorInvalidValue;
  ProfScope prof("fwd_bf16", stream);
  if (a.s.D == 128) hipLaunchKernelGGL(fwd_pipe_kernel<128>, dim3((unsigned)total), dim3(256), 0, stream, a);
  else if (a.s.D == 64) hipLaunchKernelGGL(fwd_pipe_kernel<64>, dim3((unsigned)total), dim3(256), 0, stream, a);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

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

hipError_t launch_fwd_bf16(const FwdArgs& a_in, hipStream_t stream) {
  // tuning switches (see Knobs): the general kernel's variant, and whether the hand-scheduled kernel takes part
  const int wq = knobs().fwd_wq, pipe = knobs().fwd_pipe, fast_env = knobs().fwd_fast;
  if ((fast_env || a_in.n_split > 1) && fwd_fast_usable(a_in)) {
    // fully visible full tiles by the hand-scheduled kernel, then everything else (merged into its result)
    FwdArgs a = a_in;
    if (a.n_split > 1) {
      // under-filled launch: the hand-scheduled workgroups (one per query tile and split) and the general ones
      // (masked / ragged tiles, one more state) run side by side in one launch; the caller combines the states
      a.fwd_fast = 2;
      return launch_fwd_side_by_side(a, stream);
    }
    a.fwd_fast = 1;
    hipError_t e = launch_fwd_fast(a, stream);
    if (e != hipSuccess) return e;
    ProfScope prof("fwd_edge", stream);
    const int n_qt = (a.s.Sq + 127) / 128;
    const int64_t total = (int64_t)n_qt * a.s.Hq * a.s.B;
    if (total > 0x7fffffff) return hipErrorInvalidValue;
    const dim3 grid((unsigned)total, (unsigned)(a.n_split > 1 ? a.n_split : 1));
    if (a.s.D == 128) hipLaunchKernelGGL((fwd_bf16_kernel<128, 32>), grid, dim3(256), 0, stream, a);
    else hipLaunchKernelGGL((fwd_bf16_kernel<64, 32>), grid, dim3(256), 0, stream, a);
    return hipGetLastError();
  }
  if (a_in.n_split > 1) return hipErrorInvalidValue;   // only the fast / edge pair walks a split table
  const FwdArgs& a = a_in;
  // head size 64: the two-wavefronts-per-SIMD kernel is the faster one (21.0 against 28.3 ms on the 24-head,
  // 16384 x 131072 full-mask share); head size 128 without the fast path: the pipelined kernel
  if (pipe && a.s.D == 128) return launch_fwd_pipe(a, stream);
  return wq == 64 ? launch_fwd_bf16_wq<64>(a, stream) : launch_fwd_bf16_wq<32>(a, stream);
}

}  // namespace st
