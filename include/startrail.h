/*
 * startrail.h -- C ABI of the one-GPU ring-attention share (StarTrail hot path) for gfx950.
 *
 * The library computes what ONE GPU of a (concentric) ring computes for one
 * attention layer in training: blockwise attention of a resident query shard
 * against the KV chunks the ring delivers step by step, folded into a running
 * (O, lse) state, and the matching backward accumulation of dQ, dK, dV.
 * The ring itself is simulated by visiting chunks that are already resident
 * in device memory; nothing here communicates.
 *
 * General rules for every entry point
 *   - All tensor pointers are DEVICE pointers unless a parameter says "host".
 *     Descriptor structs and the small integer tables are HOST memory and are
 *     read before the call returns.
 *   - The library allocates nothing and owns nothing: every buffer, including
 *     workspaces, is the caller's.  Calls enqueue work on the given HIP stream
 *     (a hipStream_t passed as void*, NULL = the default stream) and return
 *     without synchronising.
 *   - Errors are returned as st_status; nothing aborts or throws.  Arguments
 *     are validated on the host before any launch; on error nothing is enqueued.
 *     st_last_error() gives a text for the calling thread's last failure.
 *   - Tensors Q, K, V, dO are 4-D [B, S, heads, D] views described by element
 *     strides with the D dimension contiguous (st_tensor).  Base pointers and
 *     strides must keep every row 16-byte aligned (ST_ERR_ALIGNMENT otherwise).
 *   - Partial / running outputs are dense fp32: O-like [B, Sq, Hq, D],
 *     lse-like [B, Hq, Sq]; chunk gradients [B, Sk, Hkv, D].
 *   - Query head h reads KV head h / (Hq / Hkv).  Causal masking is by GLOBAL
 *     token position: key t of a chunk is visible to query i iff
 *     k_offset + t <= q_offset + i.  lse is the natural-log log-sum-exp of
 *     scale * <q, k> over visible keys; a row with no visible key has O = 0
 *     and lse = -inf.
 *   - Supported: ST_F32 with D <= 256 (plain kernels), ST_BF16 with D == 128
 *     or D == 64 (MFMA kernels, fp32 accumulation).  Anything else returns
 *     ST_ERR_UNSUPPORTED.
 *   - Precision of the ST_BF16 path: P and dS are rounded to bf16 before the
 *     second contractions, and every kernel, forward and backward, evaluates
 *     the scores from the same operand Q' = bf16(Q * scale * log2 e), so that
 *     the matrix units deliver exponents directly.  That is attention of a
 *     query perturbed by at most 2^-9 relative per element: the scores move by
 *     about 1e-3 of their spread (standard deviation over a row), lse likewise,
 *     and backward and forward stay consistent with each other (recomputed
 *     probabilities sum to one over a row).
 */
#ifndef STARTRAIL_H
#define STARTRAIL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  ST_OK = 0,
  ST_ERR_INVALID_ARG = 1,   /* null pointer, negative size, Hq % Hkv != 0, bad layout (P, C, rank) ... */
  ST_ERR_UNSUPPORTED = 2,   /* dtype / head_dim / size combination that has no kernel */
  ST_ERR_ALIGNMENT = 3,     /* pointer or stride breaks the 16-byte row alignment */
  ST_ERR_HIP = 4,           /* a HIP call or launch failed; see st_last_error() */
  ST_ERR_WORKSPACE = 5      /* workspace missing or smaller than st_ring_workspace_bytes() */
} st_status;

typedef enum { ST_F32 = 0, ST_BF16 = 1 } st_dtype;

/* How the driver walks the visit order. */
typedef enum {
  ST_RING_STEPWISE = 0,     /* one st_attn_block_fwd/bwd + st_attn_merge per visited chunk */
  ST_RING_FUSED = 1         /* one launch per pass; the running state stays in registers */
} st_ring_mode;

#define ST_MAX_CHUNKS 256   /* most chunks one st_ring_* call accepts */

/* 4-D view [B, S, heads, D]; strides in ELEMENTS; D contiguous (stride 1). */
typedef struct {
  void*   ptr;              /* device */
  int64_t stride_b, stride_s, stride_h;
} st_tensor;

/* One (Q shard, KV chunk) pair: the operands of one ring iteration
 * (Algorithm 1, the forward_iteration step). */
typedef struct {
  int32_t dtype;            /* st_dtype of Q, K, V, dO */
  int32_t B, Hq, Hkv, D;
  int32_t Sq, Sk;           /* tokens in the Q shard / in this chunk; Sk may be 0 */
  int64_t q_offset;         /* global position of Q row 0 */
  int64_t k_offset;         /* global position of chunk row 0 */
  int32_t causal;           /* 0: every key visible; 1: visible iff k_offset+t <= position of query row i */
  float   scale;            /* softmax scale, finite and > 0, normally 1/sqrt(D) (Section 2.1 attention equation) */
  int32_t q_seg;            /* 0: the Q rows are one run from q_offset.  > 0: rows [q_seg, Sq) are a second run */
  int64_t q_offset2;        /*    whose row q_seg sits at q_offset2 >= q_offset + q_seg (appendix "Sequence
                             *    Parallelism Dataloader": a rank holds an early and a late piece of the sequence so
                             *    that causal work is equal across ranks); 0 < q_seg < Sq */
} st_block_desc;

/* One GPU's whole share: the Q shard plus the table of chunks the ring delivers
 * (Section 3.2: after the team all-gather each delivered buffer is a run of
 * sequence shards; here every shard is one chunk with its own base pointer). */
typedef struct {
  int32_t dtype;
  int32_t B, Hq, Hkv, D;
  int32_t Sq, Sk;           /* every chunk has Sk tokens */
  int64_t q_offset;
  int32_t causal;
  float   scale;
  int32_t n_chunks;         /* 1 .. ST_MAX_CHUNKS */
  const void* const* k_ptr; /* host array [n_chunks] of device base pointers, chunk j = [B,Sk,Hkv,D] */
  const void* const* v_ptr; /* host array [n_chunks] */
  int64_t k_stride_b, k_stride_s, k_stride_h;   /* shared by all K chunks */
  int64_t v_stride_b, v_stride_s, v_stride_h;   /* shared by all V chunks */
  const int64_t* k_offset;  /* host array [n_chunks]: global position of row 0 of chunk j */
  int32_t q_seg;            /* second run of query rows, as in st_block_desc (0: none) */
  int64_t q_offset2;
} st_ring_desc;

/* ---- ring iteration, forward (Algorithm 1: forward_iteration before its fold) ----
 * Attention of the Q shard against ONE chunk.
 *   o_part   fp32 [B,Sq,Hq,D]  (overwritten)   partial output, already divided by its own row sum
 *   lse_part fp32 [B,Hq,Sq]    (overwritten)
 * A fully masked chunk (or Sk == 0) is legal and writes O = 0, lse = -inf. */
st_status st_attn_block_fwd(const st_block_desc* desc, const st_tensor* q, const st_tensor* k,
                            const st_tensor* v, float* o_part, float* lse_part, void* hip_stream);

/* ---- online-softmax fold / the arithmetic of ReduceScatter_combine (Algorithm 1;
 * Section 3.2 "Forward Propagation": lse and O are updated step by step) ----
 * In place: (o_acc, lse_acc) <- merge((o_acc, lse_acc), (o_part, lse_part)) with
 *   lse' = log(exp(lse_acc) + exp(lse_part)),
 *   O'   = exp(lse_acc - lse') O_acc + exp(lse_part - lse') O_part.
 * A state with lse = -inf is empty (the neutral element; start from O = 0, lse = -inf).
 * o_out_lowp (nullable): also write O' rounded to out_dtype, dense [B,Sq,Hq,D].
 * o_acc/o_part fp32 [B,Sq,Hq,D]; lse_acc/lse_part fp32 [B,Hq,Sq].  o_part may not alias o_acc. */
st_status st_attn_merge(float* o_acc, float* lse_acc, const float* o_part, const float* lse_part,
                        int32_t B, int32_t Sq, int32_t Hq, int32_t D, int32_t out_dtype,
                        void* o_out_lowp, void* hip_stream);

/* ---- ReduceScatter_combine on one GPU (Algorithm 1, last step; Section 3.2 "Forward Propagation": the team
 * members' intermediate results are amalgamated and each member keeps its own portion of the rows) ----
 * n_states partial states of the SAME Sq_in query rows, each over a different part of the keys, are
 * combined in one pass, and only rows [row0, row0 + Sq_out) are kept:
 *   lse' = log(sum_x exp(lse_x)),   O' = sum_x exp(lse_x - lse') O_x.
 *   o_parts, lse_parts  host arrays [n_states] of device pointers: fp32 [B,Sq_in,Hq,D] / fp32 [B,Hq,Sq_in]
 *   o_out fp32 [B,Sq_out,Hq,D], lse_out fp32 [B,Hq,Sq_out] (overwritten; may not alias an input)
 *   o_out_lowp (nullable): O' rounded to out_dtype, dense [B,Sq_out,Hq,D]
 * A state with lse = -inf on a row is empty there; a row empty in every state gives O = 0, lse = -inf.
 * Requires 1 <= n_states <= 64, D <= 256, D % 8 == 0, 0 <= row0, row0 + Sq_out <= Sq_in. */
st_status st_attn_combine(const float* const* o_parts, const float* const* lse_parts, int32_t n_states,
                          int32_t B, int32_t Sq_in, int32_t Hq, int32_t D, int32_t row0, int32_t Sq_out,
                          float* o_out, float* lse_out, int32_t out_dtype, void* o_out_lowp, void* hip_stream);

/* ---- backward preparation (Section 3.2 "Backward Propagation": each iteration mirrors the
 * FlashAttention backward, which needs Delta_i = <dO_i, O_i> of the FINAL merged O) ----
 *   d_o      [B,Sq,Hq,D] in desc->dtype;  o: the final O, in o_dtype (ST_F32 or desc->dtype)
 *   delta    fp32 [B,Hq,Sq] (overwritten).   Only B, Sq, Hq, D, dtype of desc are used. */
st_status st_attn_delta(const st_block_desc* desc, const st_tensor* d_o, const st_tensor* o,
                        int32_t o_dtype, float* delta, void* hip_stream);

/* ---- ring iteration, backward (Section 3.2 "Backward Propagation") ----
 * The Q shard (with its FINAL lse and Delta) meets ONE chunk:
 *   P = exp(scale q k^T - lse),  dV += P^T dO,  dS = P o (dO v^T - Delta),
 *   dQ += scale dS k,  dK += scale dS^T q   (dK, dV summed over the query heads of a KV group).
 *   dq_acc fp32 [B,Sq,Hq,D]   ACCUMULATED (+=): the circulating query gradient
 *   dk_acc, dv_acc fp32 [B,Sk,Hkv,D] ACCUMULATED (+=): stay with the chunk
 * The caller zeroes the accumulators once.  Every accumulator element is owned by one workgroup per
 * launch (read, add, write; no atomic adds), so results are bit-reproducible; calls that add into the same
 * accumulator must be ordered on one stream. */
st_status st_attn_block_bwd(const st_block_desc* desc, const st_tensor* q, const st_tensor* k,
                            const st_tensor* v, const st_tensor* d_o, const float* lse_final,
                            const float* delta, float* dq_acc, float* dk_acc, float* dv_acc,
                            void* workspace, size_t workspace_bytes, void* hip_stream);
/* workspace (nullable): device, 256-byte aligned, at least st_attn_block_bwd_workspace_bytes(desc) bytes (0 for
 * ST_F32).  With it the ST_BF16 path keeps a scaled copy of Q there and its hand-scheduled dK/dV kernel takes
 * part; without it the same values are computed by the general kernel, at a lower rate.  Contents mean nothing
 * between calls; calls that share a workspace must be ordered on one stream. */
size_t st_attn_block_bwd_workspace_bytes(const st_block_desc* desc);

/* ---- fp32 -> storage dtype (round to nearest even), n contiguous elements ---- */
st_status st_cast_from_f32(const float* src, void* dst, int64_t n, int32_t dst_dtype, void* hip_stream);

/* ---- chunk-visit order of the concentric layout (appendix algorithms get_init_send and
 * get_P2P_config; Section 3.2: teams of C, team groups of P/C^2 teams, sub-rings) ----
 * For the Q shard of global rank `rank` (team rank/C): one GPU plays the C members of the team
 * in turn; member a' walks its P/C^2 sub-ring iterations, each delivering the gathered KV of one
 * team = C consecutive sequence shards.
 *   shard_idx host [P] (out): sequence-shard index met at each of the P visits
 *   member_of host [P] (out): team member (0..C-1) whose running state the visit folds into
 * Requires C >= 1, C*C | P, 0 <= rank < P (else ST_ERR_INVALID_ARG).  C = 1 is the plain ring. */
st_status st_visit_order(int32_t P, int32_t C, int32_t rank, int32_t* shard_idx, int32_t* member_of);

/* ---- the literal per-GPU schedule of the concentric layout (Section 3.2: after the team all-gather every
 * member holds the team's Q, K, V of C N/P tokens; member a of team t then walks its sub-ring of P/C^2
 * GPUs and meets one gathered team buffer per iteration) ----
 * For global rank `rank` = t*C + a:
 *   team_buffer host [P/C^2] (out): index tau of the team whose gathered KV (sequence shards
 *                                   tau*C .. tau*C+C-1) is met at iteration i = 0 .. P/C^2-1
 * The rank's partial state covers the C N/P query rows of its team against those buffers; the C members'
 * partial states combined (st_attn_combine) give the team's attention output.
 * Requires C >= 1, C*C | P, 0 <= rank < P (else ST_ERR_INVALID_ARG). */
st_status st_team_visit_order(int32_t P, int32_t C, int32_t rank, int32_t* team_buffer);

/* ---- communication the schedule implies (Section 3.2 "Theoretical Analysis": the three communication
 * expressions, ring attention's P2P, the concentric layout's collectives and its P2P) ----
 * For one attention block forward on one GPU: P GPUs, team size C, batch B, sequence N, hidden size H,
 * bytes_per_element of the exchanged tensors (2 for bf16), link bandwidth W in bytes per second and
 * per-message latency L in seconds.  Byte counts are exact integers, times are fp64:
 *   ring_iterations            P - 1                      startrail_iterations            P / C^2 - 1
 *   ring_p2p_bytes_per_iter    2 B N H e / P              startrail_p2p_bytes_per_iter    2 C B N H e / P
 *   ring_p2p_bytes             product of the two         startrail_p2p_bytes             product of the two
 *   startrail_collective_bytes 4 B N H e (C - 1) / P      (team all-gather of Q, K, V + reduce-scatter of O)
 *   ring_p2p_seconds           iterations * (bytes_per_iter / W + L)        likewise startrail_p2p_seconds
 *   startrail_collective_seconds   collective_bytes / W   (the paper's expression has no latency term)
 * Requires C >= 1, C*C | P, P | N, positive sizes, W > 0, L >= 0 (else ST_ERR_INVALID_ARG).  Host-only,
 * `out` is host memory. */
typedef struct {
  int32_t ring_iterations;
  int32_t startrail_iterations;
  int64_t ring_p2p_bytes_per_iter;
  int64_t startrail_p2p_bytes_per_iter;
  int64_t ring_p2p_bytes;
  int64_t startrail_p2p_bytes;
  int64_t startrail_collective_bytes;
  double ring_p2p_seconds;
  double startrail_p2p_seconds;
  double startrail_collective_seconds;
} st_comm_report;
st_status st_schedule_report(int32_t P, int32_t C, int64_t B, int64_t N, int64_t H, int32_t bytes_per_element,
                             double W, double L, st_comm_report* out);

/* ---- driver: the whole share (Algorithm 1 loop + combine; backward loops of Section 3.2) ----
 * order host [n_visit]: chunk indices into the desc tables, in visit order (each at most once).
 * member_of host [n_visit] (nullable = all 0): running state each visit folds into; the member
 *   states are merged at the end (the combine step).  Chunks lying entirely in the causal future
 *   of the shard are skipped.
 * Forward outputs: o_acc fp32 [B,Sq,Hq,D], lse fp32 [B,Hq,Sq] (overwritten); o_lowp nullable,
 *   [B,Sq,Hq,D] in desc->dtype.
 * workspace: device, >= st_ring_workspace_bytes(desc, mode, backward) bytes, 256-byte aligned.  Its contents
 *   are the library's (partial states, Delta, the tile counters of the dK/dV launch, the scaled copy of Q) and
 *   mean nothing between calls; calls that share a workspace must be ordered on one stream. */
size_t st_ring_workspace_bytes(const st_ring_desc* desc, int32_t mode, int32_t backward);

st_status st_ring_fwd(const st_ring_desc* desc, const st_tensor* q, const int32_t* order,
                      const int32_t* member_of, int32_t n_visit, int32_t mode,
                      float* o_acc, float* lse, void* o_lowp,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/* Backward outputs (all ACCUMULATED, caller zeroes once): dq_acc fp32 [B,Sq,Hq,D];
 * dk_acc, dv_acc host arrays [n_chunks] of device fp32 [B,Sk,Hkv,D] buffers (entries of chunks
 * that are not visited may be NULL).  o: final O in o_dtype; lse_final from st_ring_fwd. */
st_status st_ring_bwd(const st_ring_desc* desc, const st_tensor* q, const st_tensor* d_o,
                      const st_tensor* o, int32_t o_dtype, const float* lse_final,
                      const int32_t* order, int32_t n_visit, int32_t mode,
                      float* dq_acc, float* const* dk_acc, float* const* dv_acc,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/* st_ring_bwd for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving or training loops, harnesses that forbid hipMalloc.  Same arguments and results as
 * st_ring_bwd (bit for bit) without the workspace: Delta, the tile counters of the dK/dV launch and the scaled
 * copy of Q live in a static device array of st_ring_bwd_noalloc_max_bytes() = 40 MiB that every GPU the library
 * runs on holds until the process ends.  The call allocates and frees nothing (no hipMalloc / hipFree, no
 * allocating library routine); the array's device address is looked up once per device, on the first call.
 * A share whose st_ring_workspace_bytes(desc, mode, 1) exceeds the array returns ST_ERR_WORKSPACE and enqueues
 * nothing.  Every call on a GPU uses that GPU's one array (what must start at zero is cleared by the call
 * itself): calls that overlap on one GPU, on different streams or from different threads, race; order them. */
st_status st_ring_bwd_noalloc(const st_ring_desc* desc, const st_tensor* q, const st_tensor* d_o,
                              const st_tensor* o, int32_t o_dtype, const float* lse_final,
                              const int32_t* order, int32_t n_visit, int32_t mode,
                              float* dq_acc, float* const* dk_acc, float* const* dv_acc, void* hip_stream);
size_t st_ring_bwd_noalloc_max_bytes(void);

/* st_ring_bwd for the LAST visit of the listed chunks, with the work that follows a chunk's last visit folded
 * into the kernels that produce dK / dV (Section 3.2 "Backward Propagation": the key and value gradients are
 * complete once the chunk has met every query shard).
 *   kv_flags   ST_KV_ASSIGN: dk_acc[j], dv_acc[j] of every chunk in `order` are OVERWRITTEN with this call's
 *              contribution instead of added to (they need not be zeroed; a listed chunk that lies entirely in
 *              the shard's causal future is set to zero).  0: accumulate, as st_ring_bwd.
 *   dk_lowp, dv_lowp  nullable; host arrays [n_chunks] of device pointers, entries nullable (both or neither of a
 *              chunk): the final dk_acc[j] / dv_acc[j] rounded to desc->dtype, dense [B,Sk,Hkv,D], 16-byte
 *              aligned.  ST_BF16 descriptors only.
 * dq_acc is accumulated as in st_ring_bwd.  Same workspace. */
enum { ST_KV_ASSIGN = 1 };
st_status st_ring_bwd_last(const st_ring_desc* desc, const st_tensor* q, const st_tensor* d_o,
                           const st_tensor* o, int32_t o_dtype, const float* lse_final,
                           const int32_t* order, int32_t n_visit, int32_t mode,
                           float* dq_acc, float* const* dk_acc, float* const* dv_acc,
                           int32_t kv_flags, void* const* dk_lowp, void* const* dv_lowp,
                           void* workspace, size_t workspace_bytes, void* hip_stream);

/* ---- per-kernel timing for benchmarks (not part of the method) ----
 * Between st_profile_begin() and st_profile_end() the library records a HIP event on the launch
 * stream before and after every kernel it launches (this creates hipEvent_t objects; at most 4096
 * launches are recorded, later ones run untimed).  st_profile_end() waits for the recorded events,
 * sums the durations per kernel name into out[0 .. *n_entries) (host memory, at most max_entries
 * entries) and stops recording.  Process-wide; not meant to be used from several threads at once. */
typedef struct {
  char    name[48];
  int32_t launches;
  float   total_ms;
} st_profile_entry;
st_status st_profile_begin(void);
st_status st_profile_end(st_profile_entry* out, int32_t max_entries, int32_t* n_entries);

/* ---- the device as the library sees it, for benchmark reports (not part of the method) ----
 * Facts of the current HIP device: compute units, XCDs (accelerator dies with an L2 each; 8 when the runtime
 * does not tell), the maximum shader and memory clocks, bus width and memory size.  `out` is host memory. */
typedef struct {
  char    name[64];
  char    arch[32];
  int32_t compute_units;
  int32_t xcds;
  int32_t max_clock_mhz;
  int32_t memory_clock_mhz;
  int32_t memory_bus_bits;
  int64_t hbm_bytes;
} st_device_report;
st_status st_device_facts(st_device_report* out);

/* ---- MFMA loops for benchmarks (not part of the method) ----
 * One workgroup of four wavefronts per compute unit; every wavefront loads 16 operand fragments (16 bytes per
 * lane each) from `operands` and then runs `iters` iterations of a loop of v_mfma_f32_32x32x16_bf16 on them.
 * Timed by the caller (events on the stream), it gives the rate the matrix units sustain on THAT data, which is
 * the ceiling to compare an attention kernel with: the chip runs at its power limit, and the limit depends on
 * the operand values and on what is issued beside the MFMAs.
 *   mix       0: nothing but MFMAs (32 per iteration).  1 .. st_mfma_probe_mixes(): side instructions with
 *             independent operands are spread between the MFMAs (st_mfma_probe_mix_name: "valu2" two v_mul_f32
 *             per MFMA, "exp1" one v_exp_f32, "pack2" two v_cvt_pk_bf16_f32, "lds1" one 16-byte LDS read,
 *             "ldstr1" one transposing 8-byte LDS read; "fwd", "dq", "dkv" and "fwd64", "dq64", "dkv64": the
 *             instruction counts per key block of the forward, dQ and dK/dV loops at head sizes 128 and 64,
 *             without their dependencies, barriers and global loads - what such a mix reaches bounds that loop
 *             on the same data)
 *   operands  device, 16-byte aligned, operand_bytes >= 65536 bytes of bf16 values (read with wrap-around)
 *   sink      device, sink_floats >= 256 * compute units floats (overwritten; keeps the loop alive)
 *   flop      host, nullable: floating point operations of the MFMAs the launch executes (2 per multiply-add) */
st_status st_mfma_probe(const void* operands, int64_t operand_bytes, int32_t mix, int32_t iters, float* sink,
                        int64_t sink_floats, double* flop, void* hip_stream);
int32_t     st_mfma_probe_mixes(void);
const char* st_mfma_probe_mix_name(int32_t mix);   /* "" for a mix out of range */

/* ---- misc ---- */
const char* st_status_str(st_status s);
const char* st_last_error(void);      /* thread-local text of the last failure, "" if none */
int32_t     st_version(void);         /* major*10000 + minor*100 + patch */

#ifdef __cplusplus
}
#endif
#endif /* STARTRAIL_H */
