// Internal launch interface between the C-ABI layer (st_api.cpp) and the HIP kernels.
// Plain structs passed BY VALUE as kernel arguments: no device-side tables to allocate or copy.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/startrail.h"

namespace st {

constexpr int kMaxTable = 64;   // chunks one kernel launch can walk (fits the 4 KiB kernel-argument space)

struct View {                   // [B, S, heads, D] view, element strides, D contiguous
  const void* ptr;
  int64_t sb, ss, sh;
};

struct Shape {
  int32_t B, Hq, Hkv, D, Sq, Sk;
  int64_t q_offset;   // global position of query row 0
  int32_t causal;
  float scale;
  int32_t q_seg;      // 0: one run of rows; > 0: rows [q_seg, Sq) are a second run that starts at q_offset2
  int64_t q_offset2;  //    (two half-shards of a load-balanced causal placement); positions rise with the row
};

// Global position of query row i.
__host__ __device__ inline int64_t q_pos(const Shape& s, int i) {
  return (s.q_seg > 0 && i >= s.q_seg) ? s.q_offset2 + (i - s.q_seg) : s.q_offset + i;
}
// Smallest row index whose position is >= p: under a causal mask row i sees a key at p iff i >= q_row_of(p).
// Sq if no row does.
__host__ __device__ inline int q_row_of(const Shape& s, int64_t p) {
  const int n0 = s.q_seg > 0 ? s.q_seg : s.Sq;
  int64_t i = p - s.q_offset;
  if (i < n0) return i < 0 ? 0 : (int)i;
  if (s.q_seg <= 0) return s.Sq;
  i = p - s.q_offset2;
  if (i < 0) i = 0;
  return i >= s.Sq - n0 ? s.Sq : n0 + (int)i;
}

// Chunks in visit order.  k/v are base pointers of [B,Sk,Hkv,D] views that share one stride set.
struct ChunkTable {
  int32_t n;
  const void* k[kMaxTable];
  const void* v[kMaxTable];
  int64_t k_offset[kMaxTable];
  int64_t ksb, kss, ksh, vsb, vss, vsh;
};

struct FwdArgs {
  Shape s;
  View q;
  ChunkTable t;
  float* o;        // fp32 [B,Sq,Hq,D]
  float* lse;      // fp32 [B,Hq,Sq]
  void* o_lowp;    // nullable, [B,Sq,Hq,D] in the storage dtype
  int32_t fwd_fast;  // 1: the fast forward kernel ran first and owns the tiles qtile_fast_tiles describes
                     // 2: it owns them and runs in the same launch; the general workgroups write state n_split
  // Under-filled launches: n_split > 1 gives every query tile n_split workgroups (blockIdx.y), each walking a
  // contiguous share of the table and writing its own partial state at o + y * split_o, lse + y * split_l
  // (floats); the states are combined afterwards.  0 or 1: one workgroup walks the whole table.
  int32_t n_split;
  int64_t split_o, split_l;
  float gap;         // fast kernel: log2 units a block maximum may exceed the lazy exponent reference by (set by its launcher)
};

// table entries [lo, hi) of split y
__host__ __device__ inline void split_range(int n, int n_split, int y, int& lo, int& hi) {
  if (n_split <= 1) { lo = 0; hi = n; return; }
  lo = (int)((int64_t)n * y / n_split);
  hi = (int)((int64_t)n * (y + 1) / n_split);
}

struct BwdArgs {
  Shape s;
  View q, d_o;
  const void* qs;      // bf16 path: Q' = bf16(Q * scale * log2 e), the exponent operand (see scale_bf16x8), dense
                       // [B,Sq,Hq,D], made by launch_scale_q; nullable: without it the key-stationary pass stays in
                       // the general kernel, which converts the rows it stages itself
  ChunkTable t;
  const float* lse;    // final
  const float* delta;
  float* dq;           // fp32 [B,Sq,Hq,D], +=
  float* dk[kMaxTable];  // fp32 [B,Sk,Hkv,D] per table entry, +=
  float* dv[kMaxTable];
  int32_t dkv_fast;    // 1: the fast dK/dV kernel runs too and owns the blocks dkv_fast_first_block describes
  int32_t dq_fast;     // 1: the fast dQ kernel runs too and owns the tiles dq_fast_tiles describes
  // dK / dV work of a chunk's last visit folded into the launch (bf16 path).  On entry to launch_bwd_bf16 they
  // state what the caller wants for every table entry; the launcher keeps them for the entries whose every
  // block belongs to the fast kernel (their only writer) and serves the others with fill / cast launches.
  uint64_t kv_assign;          // bit c: dk[c] / dv[c] are overwritten, not added to
  void* dk_lowp[kMaxTable];    // nullable per entry: the final dk[c] / dv[c] rounded to bf16, dense [B,Sk,Hkv,D]
  void* dv_lowp[kMaxTable];
  int32_t* queue;      // nullable, kQueueInts ints of device memory: the fast dK/dV kernel hands its key tiles out
                       // through it (one counter per XCD), so that XCDs that run faster take more of them
  int32_t queue_xcds;  // counters in use (the device's XCD count, 1 .. 8); set by the launcher
};
constexpr int kQueueInts = 8 * 32;   // at most 8 counters, 128 bytes apart
// passed by value: the kernel-argument segment holds 4096 bytes, 256 of them the implicit arguments
static_assert(sizeof(BwdArgs) <= 4096 - 256 && sizeof(FwdArgs) <= 4096 - 256, "argument structs must fit the kernel-argument segment");

// n partial states of the same query rows (each O fp32 [B,Sq_in,Hq,D], lse fp32 [B,Hq,Sq_in]) and the run of
// rows [row0, row0 + Sq_out) the combined state keeps.
struct CombineArgs {
  int32_t n;
  const float* o[kMaxTable];
  const float* lse[kMaxTable];
  int32_t B, Sq_in, Hq, D, row0, Sq_out;
  float* o_out;      // fp32 [B,Sq_out,Hq,D]
  float* lse_out;    // fp32 [B,Hq,Sq_out]
  void* o_lowp;      // nullable, [B,Sq_out,Hq,D]
};

// Split of the dK/dV work between the general kernel and the fast one (head_dim 128): the fast kernel
// takes, for every FULL tile of kDkvFastKeys keys, the full kDkvFastRows-query blocks from the first one
// whose rows all see the tile's last key; everything else (masked blocks, ragged tails) stays general.
constexpr int kDkvFastKeys = 256;
constexpr int kDkvFastRows = 32;
__host__ __device__ inline int dkv_fast_first_block(const Shape& s, int64_t k0, int tile_key0) {
  if (!s.causal) return 0;
  const int d = q_row_of(s, k0 + tile_key0 + kDkvFastKeys - 1);     // first row index that sees the last key
  return (d + kDkvFastRows - 1) / kDkvFastRows;
}

// True when the fast dK/dV kernel alone works on a chunk of full tiles: every query row sees either all of the
// chunk's keys or none of them, and the rows that see it start at a block boundary, so no block needs a mask.
// (With one run of rows these are the chunks that end before the shard begins; with two runs also the chunks
// that lie between the two.)
__host__ __device__ inline bool dkv_chunk_fast_only(const Shape& s, int64_t k0) {
  if (s.Sk % kDkvFastKeys != 0 || s.Sq % kDkvFastRows != 0) return false;
  if (!s.causal) return true;
  const int r_any = q_row_of(s, k0), r_all = q_row_of(s, k0 + s.Sk - 1);
  return r_any == r_all && r_all % kDkvFastRows == 0 && r_all < s.Sq;
}

// Tuning and testing switches of the launchers.  The defaults are the product.  They are read from the
// environment ONCE, when the library is loaded (ST_FWD_FAST, ST_DQ_FAST, ST_DKV_FAST, ST_DKV_QUEUE, ST_FWD_WQ,
// ST_FWD_PIPE, ST_FWD_GAP); afterwards only st_testing_set() changes them, an exported entry point for the
// library's own tests that the public header does not declare.  No launcher reads the environment.
struct Knobs {
  int fwd_fast = 1;    // 0: the forward stays in the general kernels
  int dq_fast = 1;     // 0: the dQ pass stays in the general kernel
  int dkv_fast = 1;    // 0: the dK/dV pass stays in the general kernel
  int dkv_queue = 1;   // 0: every dK/dV key tile is a workgroup of its own (no tile queue)
  int fwd_wq = 32;     // general forward without the fast path: queries per wavefront (32 or 64)
  int fwd_pipe = 1;    // general forward without the fast path, head size 128: the pipelined variant
  float fwd_gap = 8.f; // fast forward: log2 units a block maximum may exceed the lazy exponent reference by (0 .. 64)
};
Knobs& knobs();

// Facts about a device that the launchers need, queried once per device and cached.
constexpr int kMaxXcds = 8;
struct DeviceInfo {
  int cus = 0;         // compute units
  int xcds = kMaxXcds; // accelerator complex dies (each with its own L2); kMaxXcds when the runtime does not tell
};
const DeviceInfo& device_info();   // of the current device

// Optional per-kernel timing (st_profile_begin / st_profile_end): while enabled, a ProfScope
// records a HIP event on the launch stream before and after the kernel it brackets.
struct ProfScope {
  ProfScope(const char* name, hipStream_t s);
  ~ProfScope();
  int slot;
  hipStream_t stream;
};

// Split of the query-stationary kernels (forward, dQ; head_dim 128): for every FULL tile of kQTileFastRows
// queries the fast kernel takes, of each chunk, the leading kQTileFastKeys-key tiles that the tile's first
// row (hence every row) sees in full.
constexpr int kQTileFastRows = 256;
constexpr int kQTileFastKeys = 64;
constexpr int kDqFastRows = kQTileFastRows;
constexpr int kDqFastKeys = kQTileFastKeys;
__host__ __device__ inline int qtile_fast_tiles(const Shape& s, int row0, int64_t k0) {
  int64_t nv = s.Sk;
  if (s.causal) {
    nv = q_pos(s, row0) - k0 + 1;
    nv = nv < 0 ? 0 : (nv > s.Sk ? s.Sk : nv);
  }
  return (int)(nv / kQTileFastKeys);
}
__host__ __device__ inline int dq_fast_tiles(const Shape& s, int row0, int64_t k0) {
  return qtile_fast_tiles(s, row0, k0);
}

// ---- launchers (each returns hipGetLastError() after the launch) ----
hipError_t launch_fwd_f32(const FwdArgs& a, hipStream_t s);
hipError_t launch_bwd_f32(const BwdArgs& a, hipStream_t s);
hipError_t launch_fwd_bf16(const FwdArgs& a, hipStream_t s);
bool fwd_fast_usable(const FwdArgs& a);
hipError_t launch_fwd_fast(const FwdArgs& a, hipStream_t s);
// split launches (a.n_split > 1): fast and general workgroups in one launch, n_split + 1 partial states
hipError_t launch_fwd_side_by_side(const FwdArgs& a, hipStream_t s);
hipError_t launch_bwd_bf16(const BwdArgs& a, hipStream_t s);
bool dkv_fast_usable(const BwdArgs& a);
hipError_t launch_bwd_dkv_fast(const BwdArgs& a, hipStream_t s);
bool dq_fast_usable(const BwdArgs& a);
hipError_t launch_bwd_dq_fast(const BwdArgs& a, hipStream_t s);

hipError_t launch_merge(float* o_acc, float* lse_acc, const float* o_part, const float* lse_part,
                        int32_t B, int32_t Sq, int32_t Hq, int32_t D, void* o_lowp, int lowp_dtype,
                        hipStream_t s);
hipError_t launch_combine(const CombineArgs& a, int lowp_dtype, hipStream_t s);
hipError_t launch_delta(const View& d_o, int d_o_dtype, const View& o, int o_dtype, float* delta,
                        int32_t B, int32_t Sq, int32_t Hq, int32_t D, hipStream_t s);
hipError_t launch_cast(const float* src, void* dst, int64_t n, int dst_dtype, hipStream_t s);
// dst (dense bf16 [B,Sq,Hq,D]) = bf16(q * scale * log2 e) of a bf16 view q
hipError_t launch_scale_q(const View& q, void* dst, int32_t B, int32_t Sq, int32_t Hq, int32_t D, float scale, hipStream_t s);
hipError_t launch_fill_state(float* o, float* lse, int64_t n_o, int64_t n_lse, hipStream_t s);
hipError_t launch_zero(void* dst, int64_t bytes, hipStream_t s);   // bytes % 4 == 0, dst 4-byte aligned
// benchmark aid: MFMA-only loop, one workgroup per compute unit (see st_probe.hip)
int mfma_probe_blocks();
int mfma_probe_mixes();                              // side-instruction mixes 1 .. mfma_probe_mixes(); 0 = MFMAs only
const char* mfma_probe_mix_name(int mix);
double mfma_probe_flop(int blocks, int mix, int32_t iters);
hipError_t launch_mfma_probe(const void* operands, int64_t operand_bytes, int mix, int32_t iters, float* sink, int blocks,
                             hipStream_t s);

}  // namespace st
