// C-ABI layer: argument validation, dtype dispatch, the visit-order generator and the
// driver that walks a chunk-visit order.  No arithmetic of the method lives here; every
// step of the path runs in the HIP kernels behind the launch_* functions.
#include <cstdarg>
#include <cstdio>
#include <cstring>

#include <mutex>
#include <vector>

#include "st_internal.h"

namespace {

// ---- event profiler state ----
struct ProfRec {
  const char* name;
  hipEvent_t start, stop;
};
std::mutex g_prof_mu;
bool g_prof_on = false;
std::vector<ProfRec> g_prof;
constexpr size_t kProfMax = 4096;

thread_local char g_err[512] = "";

// ---- scratch of st_ring_bwd_noalloc: device memory every loaded GPU holds until the process ends ----
// In host code the array's name is only a handle: its device address differs from GPU to GPU and is looked up
// once per device with hipGetSymbolAddress (scratch_of_current_device); kernels only ever see that pointer.
constexpr size_t kScratchBytes = (size_t)40 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
constexpr int kScratchDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kScratchDevices];

st_status fail(st_status s, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return s;
}

st_status hip_fail(hipError_t e, const char* what) {
  return fail(ST_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

// Device address of `scratch` on the current device (looked up on the first call per device, then cached).
st_status scratch_of_current_device(void** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  if (dev < 0 || dev >= kScratchDevices) return fail(ST_ERR_UNSUPPORTED, "device index %d beyond %d", dev, kScratchDevices - 1);
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
    if (p == nullptr || reinterpret_cast<uintptr_t>(p) % 256) return fail(ST_ERR_HIP, "scratch symbol has no aligned device address");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return ST_OK;
}

inline size_t elem_size(int dtype) { return dtype == ST_BF16 ? 2 : 4; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

st_status check_scale(float scale) {
  if (!(scale > 0.f) || scale > 3.0e38f) return fail(ST_ERR_INVALID_ARG, "scale must be finite and positive");
  return ST_OK;
}

st_status check_shape(int dtype, int B, int Hq, int Hkv, int D, int Sq, int Sk) {
  if (dtype != ST_F32 && dtype != ST_BF16) return fail(ST_ERR_INVALID_ARG, "unknown dtype %d", dtype);
  if (B < 0 || Sq < 0 || Sk < 0) return fail(ST_ERR_INVALID_ARG, "negative size");
  if (Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0) return fail(ST_ERR_INVALID_ARG, "need Hq %% Hkv == 0 (Hq=%d Hkv=%d)", Hq, Hkv);
  if (D <= 0) return fail(ST_ERR_INVALID_ARG, "D must be positive");
  if (dtype == ST_F32 && (D > 256 || D % 8 != 0)) return fail(ST_ERR_UNSUPPORTED, "fp32 path needs D <= 256 and D %% 8 == 0 (D=%d)", D);
  if (dtype == ST_BF16 && D != 128 && D != 64) return fail(ST_ERR_UNSUPPORTED, "bf16 path is built for D = 64 or 128 (D=%d)", D);
  if (B > 65535 || Hq > 65535) return fail(ST_ERR_UNSUPPORTED, "B and Hq must not exceed 65535");
  return ST_OK;
}

// a [B,S,heads,D] view whose rows must be 16-byte aligned
st_status check_view(const char* name, const void* ptr, int64_t sb, int64_t ss, int64_t sh, int dtype,
                     int64_t n_elems) {
  if (n_elems == 0) return ST_OK;
  if (ptr == nullptr) return fail(ST_ERR_INVALID_ARG, "%s: null pointer", name);
  const int64_t per16 = 16 / (int64_t)elem_size(dtype);
  if (reinterpret_cast<uintptr_t>(ptr) % 16 != 0) return fail(ST_ERR_ALIGNMENT, "%s: base pointer is not 16-byte aligned", name);
  if (sb % per16 || ss % per16 || sh % per16) return fail(ST_ERR_ALIGNMENT, "%s: strides must be multiples of %lld elements", name, (long long)per16);
  if (sb < 0 || ss < 0 || sh < 0) return fail(ST_ERR_INVALID_ARG, "%s: negative stride", name);
  return ST_OK;
}

st_status check_tensor(const char* name, const st_tensor* t, int dtype, int64_t n_elems) {
  if (t == nullptr) return fail(ST_ERR_INVALID_ARG, "%s: null st_tensor", name);
  return check_view(name, t->ptr, t->stride_b, t->stride_s, t->stride_h, dtype, n_elems);
}

st_status check_f32(const char* name, const void* p, int64_t n_elems) {
  if (n_elems == 0) return ST_OK;
  if (p == nullptr) return fail(ST_ERR_INVALID_ARG, "%s: null pointer", name);
  if (reinterpret_cast<uintptr_t>(p) % 16 != 0) return fail(ST_ERR_ALIGNMENT, "%s: not 16-byte aligned", name);
  return ST_OK;
}

st::View view_of(const st_tensor* t) { return st::View{t->ptr, t->stride_b, t->stride_s, t->stride_h}; }

st::Shape shape_of(const st_block_desc* d) {
  return st::Shape{d->B, d->Hq, d->Hkv, d->D, d->Sq, d->Sk, d->q_offset, d->causal ? 1 : 0, d->scale, d->q_seg, d->q_offset2};
}
st::Shape shape_of(const st_ring_desc* d) {
  return st::Shape{d->B, d->Hq, d->Hkv, d->D, d->Sq, d->Sk, d->q_offset, d->causal ? 1 : 0, d->scale, d->q_seg, d->q_offset2};
}

// two runs of query rows: the second must not start before the first ends (positions rise with the row index)
st_status check_segments(int32_t Sq, int64_t q_offset, int32_t q_seg, int64_t q_offset2) {
  if (q_seg == 0) return ST_OK;
  if (q_seg < 0 || q_seg >= Sq) return fail(ST_ERR_INVALID_ARG, "q_seg = %d must be 0 or inside the %d query rows", q_seg, Sq);
  if (q_offset2 < q_offset + q_seg) return fail(ST_ERR_INVALID_ARG, "second run of query rows starts before the first ends");
  return ST_OK;
}

#define ST_TRY(expr)                  \
  do {                                \
    st_status _s = (expr);            \
    if (_s != ST_OK) return _s;       \
  } while (0)
#define ST_HIP(expr, what)                        \
  do {                                            \
    hipError_t _e = (expr);                       \
    if (_e != hipSuccess) return hip_fail(_e, what); \
  } while (0)

hipError_t launch_fwd(int dtype, const st::FwdArgs& a, hipStream_t s) {
  return dtype == ST_BF16 ? st::launch_fwd_bf16(a, s) : st::launch_fwd_f32(a, s);
}
hipError_t launch_bwd(int dtype, const st::BwdArgs& a, hipStream_t s) {
  return dtype == ST_BF16 ? st::launch_bwd_bf16(a, s) : st::launch_bwd_f32(a, s);
}

// chunk lies entirely in the causal future of the shard: nothing to compute
inline bool chunk_invisible(const st_ring_desc* d, int j) {
  return d->Sk == 0 || (d->causal && d->k_offset[j] > st::q_pos(shape_of(d), d->Sq - 1));
}

st_status check_ring(const st_ring_desc* d, const st_tensor* q, const int32_t* order, int32_t n_visit) {
  if (d == nullptr) return fail(ST_ERR_INVALID_ARG, "null descriptor");
  ST_TRY(check_shape(d->dtype, d->B, d->Hq, d->Hkv, d->D, d->Sq, d->Sk));
  ST_TRY(check_scale(d->scale));
  ST_TRY(check_segments(d->Sq, d->q_offset, d->q_seg, d->q_offset2));
  if (d->n_chunks < 1 || d->n_chunks > ST_MAX_CHUNKS) return fail(ST_ERR_INVALID_ARG, "n_chunks must be in 1..%d", ST_MAX_CHUNKS);
  if (!d->k_ptr || !d->v_ptr || !d->k_offset) return fail(ST_ERR_INVALID_ARG, "null chunk table");
  if (n_visit < 0 || n_visit > d->n_chunks) return fail(ST_ERR_INVALID_ARG, "n_visit out of range");
  if (n_visit > 0 && order == nullptr) return fail(ST_ERR_INVALID_ARG, "null visit order");
  const int64_t n_kv = (int64_t)d->B * d->Sk * d->Hkv * d->D;
  bool seen[ST_MAX_CHUNKS] = {false};
  for (int x = 0; x < n_visit; ++x) {
    const int j = order[x];
    if (j < 0 || j >= d->n_chunks) return fail(ST_ERR_INVALID_ARG, "order[%d] = %d is not a chunk index", x, j);
    if (seen[j]) return fail(ST_ERR_INVALID_ARG, "chunk %d is visited twice", j);
    seen[j] = true;
    ST_TRY(check_view("k chunk", d->k_ptr[j], d->k_stride_b, d->k_stride_s, d->k_stride_h, d->dtype, n_kv));
    ST_TRY(check_view("v chunk", d->v_ptr[j], d->v_stride_b, d->v_stride_s, d->v_stride_h, d->dtype, n_kv));
  }
  return check_tensor("q", q, d->dtype, (int64_t)d->B * d->Sq * d->Hq * d->D);
}

void set_table_strides(st::ChunkTable& t, const st_ring_desc* d) {
  t.ksb = d->k_stride_b; t.kss = d->k_stride_s; t.ksh = d->k_stride_h;
  t.vsb = d->v_stride_b; t.vss = d->v_stride_s; t.vsh = d->v_stride_h;
}

}  // namespace

namespace st {

ProfScope::ProfScope(const char* name, hipStream_t s) : slot(-1), stream(s) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  if (!g_prof_on || g_prof.size() >= kProfMax) return;
  ProfRec r{name, nullptr, nullptr};
  if (hipEventCreate(&r.start) != hipSuccess) return;
  if (hipEventCreate(&r.stop) != hipSuccess) {
    (void)hipEventDestroy(r.start);
    return;
  }
  (void)hipEventRecord(r.start, s);
  g_prof.push_back(r);
  slot = (int)g_prof.size() - 1;
}

ProfScope::~ProfScope() {
  if (slot < 0) return;
  std::lock_guard<std::mutex> lk(g_prof_mu);
  if (slot < (int)g_prof.size()) (void)hipEventRecord(g_prof[slot].stop, stream);
}

}  // namespace st

extern "C" {

st_status st_profile_begin(void) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  for (auto& r : g_prof) {
    (void)hipEventDestroy(r.start);
    (void)hipEventDestroy(r.stop);
  }
  g_prof.clear();
  g_prof_on = true;
  return ST_OK;
}

st_status st_profile_end(st_profile_entry* out, int32_t max_entries, int32_t* n_entries) {
  if (!out || !n_entries || max_entries < 0) return fail(ST_ERR_INVALID_ARG, "null output");
  std::lock_guard<std::mutex> lk(g_prof_mu);
  g_prof_on = false;
  int32_t n = 0;
  st_status status = ST_OK;
  for (auto& r : g_prof) {
    float ms = 0.f;
    hipError_t e = hipEventSynchronize(r.stop);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.start, r.stop);
    if (e != hipSuccess) status = hip_fail(e, "st_profile_end");
    int32_t k = 0;
    while (k < n && strncmp(out[k].name, r.name, sizeof(out[k].name) - 1) != 0) ++k;
    if (k == n) {
      if (n >= max_entries) continue;
      memset(&out[n], 0, sizeof(out[n]));
      strncpy(out[n].name, r.name, sizeof(out[n].name) - 1);
      ++n;
    }
    out[k].launches += 1;
    out[k].total_ms += ms;
    (void)hipEventDestroy(r.start);
    (void)hipEventDestroy(r.stop);
  }
  g_prof.clear();
  *n_entries = n;
  return status;
}

st_status st_mfma_probe(const void* operands, int64_t operand_bytes, int32_t mix, int32_t iters, float* sink,
                        int64_t sink_floats, double* flop, void* hip_stream) {
  if (operands == nullptr || sink == nullptr) return fail(ST_ERR_INVALID_ARG, "null pointer");
  if (reinterpret_cast<uintptr_t>(operands) % 16) return fail(ST_ERR_ALIGNMENT, "operands: not 16-byte aligned");
  if (operand_bytes < 65536) return fail(ST_ERR_INVALID_ARG, "operands: at least 65536 bytes are needed");
  if (iters < 1 || iters > (1 << 24)) return fail(ST_ERR_INVALID_ARG, "iters must be in 1 .. 2^24");
  if (mix < 0 || mix > st::mfma_probe_mixes()) return fail(ST_ERR_INVALID_ARG, "mix must be in 0 .. %d", st::mfma_probe_mixes());
  const int blocks = st::mfma_probe_blocks();
  if (sink_floats < (int64_t)blocks * 256) return fail(ST_ERR_INVALID_ARG, "sink: %lld floats are needed", (long long)blocks * 256);
  ST_HIP(st::launch_mfma_probe(operands, operand_bytes, mix, iters, sink, blocks, (hipStream_t)hip_stream), "st_mfma_probe launch");
  if (flop) *flop = st::mfma_probe_flop(blocks, mix, iters);
  return ST_OK;
}

int32_t st_mfma_probe_mixes(void) { return st::mfma_probe_mixes(); }
const char* st_mfma_probe_mix_name(int32_t mix) { return st::mfma_probe_mix_name(mix); }

st_status st_device_facts(st_device_report* out) {
  if (out == nullptr) return fail(ST_ERR_INVALID_ARG, "null output");
  memset(out, 0, sizeof(*out));
  int dev = 0;
  ST_HIP(hipGetDevice(&dev), "hipGetDevice");
  hipDeviceProp_t prop;
  ST_HIP(hipGetDeviceProperties(&prop, dev), "hipGetDeviceProperties");
  const st::DeviceInfo& info = st::device_info();
  out->compute_units = info.cus > 0 ? info.cus : prop.multiProcessorCount;
  out->xcds = info.xcds;
  out->max_clock_mhz = prop.clockRate / 1000;
  out->memory_clock_mhz = prop.memoryClockRate / 1000;
  out->memory_bus_bits = prop.memoryBusWidth;
  out->hbm_bytes = (int64_t)prop.totalGlobalMem;
  strncpy(out->name, prop.name, sizeof(out->name) - 1);
  strncpy(out->arch, prop.gcnArchName, sizeof(out->arch) - 1);
  return ST_OK;
}

const char* st_status_str(st_status s) {
  switch (s) {
    case ST_OK: return "ok";
    case ST_ERR_INVALID_ARG: return "invalid argument";
    case ST_ERR_UNSUPPORTED: return "unsupported dtype / head_dim / size";
    case ST_ERR_ALIGNMENT: return "misaligned pointer or stride";
    case ST_ERR_HIP: return "HIP error";
    case ST_ERR_WORKSPACE: return "workspace missing or too small";
  }
  return "unknown status";
}

const char* st_last_error(void) { return g_err; }
int32_t st_version(void) { return 100; }

st_status st_attn_block_fwd(const st_block_desc* d, const st_tensor* q, const st_tensor* k, const st_tensor* v,
                            float* o_part, float* lse_part, void* hip_stream) {
  if (d == nullptr) return fail(ST_ERR_INVALID_ARG, "null descriptor");
  ST_TRY(check_shape(d->dtype, d->B, d->Hq, d->Hkv, d->D, d->Sq, d->Sk));
  ST_TRY(check_scale(d->scale));
  ST_TRY(check_segments(d->Sq, d->q_offset, d->q_seg, d->q_offset2));
  const int64_t n_q = (int64_t)d->B * d->Sq * d->Hq * d->D, n_kv = (int64_t)d->B * d->Sk * d->Hkv * d->D;
  ST_TRY(check_tensor("q", q, d->dtype, n_q));
  ST_TRY(check_tensor("k", k, d->dtype, n_kv));
  ST_TRY(check_tensor("v", v, d->dtype, n_kv));
  ST_TRY(check_f32("o_part", o_part, n_q));
  ST_TRY(check_f32("lse_part", lse_part, n_q));
  if (n_q == 0) return ST_OK;
  st::FwdArgs a;
  memset(&a, 0, sizeof(a));
  a.s = shape_of(d);
  a.q = view_of(q);
  a.t.n = n_kv > 0 ? 1 : 0;
  a.t.k[0] = k->ptr; a.t.v[0] = v->ptr; a.t.k_offset[0] = d->k_offset;
  a.t.ksb = k->stride_b; a.t.kss = k->stride_s; a.t.ksh = k->stride_h;
  a.t.vsb = v->stride_b; a.t.vss = v->stride_s; a.t.vsh = v->stride_h;
  a.o = o_part; a.lse = lse_part; a.o_lowp = nullptr;
  ST_HIP(launch_fwd(d->dtype, a, (hipStream_t)hip_stream), "st_attn_block_fwd launch");
  return ST_OK;
}

st_status st_attn_merge(float* o_acc, float* lse_acc, const float* o_part, const float* lse_part, int32_t B,
                        int32_t Sq, int32_t Hq, int32_t D, int32_t out_dtype, void* o_out_lowp, void* hip_stream) {
  if (B < 0 || Sq < 0 || Hq <= 0 || D <= 0) return fail(ST_ERR_INVALID_ARG, "bad sizes");
  if (D > 256 || D % 8 != 0) return fail(ST_ERR_UNSUPPORTED, "merge needs D <= 256 and D %% 8 == 0");
  if (out_dtype != ST_F32 && out_dtype != ST_BF16) return fail(ST_ERR_INVALID_ARG, "unknown out_dtype");
  const int64_t n = (int64_t)B * Sq * Hq * D;
  ST_TRY(check_f32("o_acc", o_acc, n));
  ST_TRY(check_f32("lse_acc", lse_acc, n));
  ST_TRY(check_f32("o_part", o_part, n));
  ST_TRY(check_f32("lse_part", lse_part, n));
  if (o_out_lowp && reinterpret_cast<uintptr_t>(o_out_lowp) % 16) return fail(ST_ERR_ALIGNMENT, "o_out_lowp: not 16-byte aligned");
  if (n > 0 && o_acc == o_part) return fail(ST_ERR_INVALID_ARG, "o_part aliases o_acc");
  ST_HIP(st::launch_merge(o_acc, lse_acc, o_part, lse_part, B, Sq, Hq, D, o_out_lowp, out_dtype,
                          (hipStream_t)hip_stream), "st_attn_merge launch");
  return ST_OK;
}

st_status st_attn_combine(const float* const* o_parts, const float* const* lse_parts, int32_t n_states, int32_t B,
                          int32_t Sq_in, int32_t Hq, int32_t D, int32_t row0, int32_t Sq_out, float* o_out,
                          float* lse_out, int32_t out_dtype, void* o_out_lowp, void* hip_stream) {
  if (!o_parts || !lse_parts) return fail(ST_ERR_INVALID_ARG, "null state tables");
  if (n_states < 1 || n_states > st::kMaxTable) return fail(ST_ERR_INVALID_ARG, "n_states must be 1..%d", st::kMaxTable);
  if (B < 0 || Sq_in < 0 || Sq_out < 0 || Hq <= 0 || D <= 0) return fail(ST_ERR_INVALID_ARG, "bad sizes");
  if (row0 < 0 || (int64_t)row0 + Sq_out > Sq_in) return fail(ST_ERR_INVALID_ARG, "rows [%d, %d + %d) are not inside the %d rows of the states", row0, row0, Sq_out, Sq_in);
  if (D > 256 || D % 8 != 0) return fail(ST_ERR_UNSUPPORTED, "combine needs D <= 256 and D %% 8 == 0");
  if (out_dtype != ST_F32 && out_dtype != ST_BF16) return fail(ST_ERR_INVALID_ARG, "unknown out_dtype");
  const int64_t n_in = (int64_t)B * Sq_in * Hq * D, n_out = (int64_t)B * Sq_out * Hq * D;
  ST_TRY(check_f32("o_out", o_out, n_out));
  ST_TRY(check_f32("lse_out", lse_out, n_out));
  if (o_out_lowp && reinterpret_cast<uintptr_t>(o_out_lowp) % 16) return fail(ST_ERR_ALIGNMENT, "o_out_lowp: not 16-byte aligned");
  st::CombineArgs a;
  memset(&a, 0, sizeof(a));
  for (int x = 0; x < n_states; ++x) {
    ST_TRY(check_f32("o_parts[x]", o_parts[x], n_in));
    ST_TRY(check_f32("lse_parts[x]", lse_parts[x], n_in));
    if (n_out > 0 && (o_parts[x] == o_out || lse_parts[x] == lse_out)) return fail(ST_ERR_INVALID_ARG, "an output aliases state %d", x);
    a.o[x] = o_parts[x];
    a.lse[x] = lse_parts[x];
  }
  if (n_out == 0) return ST_OK;
  a.n = n_states;
  a.B = B; a.Sq_in = Sq_in; a.Hq = Hq; a.D = D; a.row0 = row0; a.Sq_out = Sq_out;
  a.o_out = o_out; a.lse_out = lse_out; a.o_lowp = o_out_lowp;
  ST_HIP(st::launch_combine(a, out_dtype, (hipStream_t)hip_stream), "st_attn_combine launch");
  return ST_OK;
}

st_status st_attn_delta(const st_block_desc* d, const st_tensor* d_o, const st_tensor* o, int32_t o_dtype,
                        float* delta, void* hip_stream) {
  if (d == nullptr) return fail(ST_ERR_INVALID_ARG, "null descriptor");
  ST_TRY(check_shape(d->dtype, d->B, d->Hq, d->Hkv, d->D, d->Sq, 0));
  if (o_dtype != ST_F32 && o_dtype != d->dtype) return fail(ST_ERR_INVALID_ARG, "o_dtype must be ST_F32 or the storage dtype");
  const int64_t n = (int64_t)d->B * d->Sq * d->Hq * d->D;
  ST_TRY(check_tensor("d_o", d_o, d->dtype, n));
  ST_TRY(check_tensor("o", o, o_dtype, n));
  ST_TRY(check_f32("delta", delta, n));
  if (n == 0) return ST_OK;
  ST_HIP(st::launch_delta(view_of(d_o), d->dtype, view_of(o), o_dtype, delta, d->B, d->Sq, d->Hq, d->D,
                          (hipStream_t)hip_stream), "st_attn_delta launch");
  return ST_OK;
}

size_t st_attn_block_bwd_workspace_bytes(const st_block_desc* d) {
  if (d == nullptr || d->dtype != ST_BF16 || d->B <= 0 || d->Sq <= 0 || d->Hq <= 0 || d->D <= 0) return 0;
  return align_up((size_t)d->B * d->Sq * d->Hq * d->D * 2, 256);     // Q' = bf16(Q scale log2 e)
}

st_status st_attn_block_bwd(const st_block_desc* d, const st_tensor* q, const st_tensor* k, const st_tensor* v,
                            const st_tensor* d_o, const float* lse_final, const float* delta, float* dq_acc,
                            float* dk_acc, float* dv_acc, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (d == nullptr) return fail(ST_ERR_INVALID_ARG, "null descriptor");
  ST_TRY(check_shape(d->dtype, d->B, d->Hq, d->Hkv, d->D, d->Sq, d->Sk));
  ST_TRY(check_scale(d->scale));
  ST_TRY(check_segments(d->Sq, d->q_offset, d->q_seg, d->q_offset2));
  const int64_t n_q = (int64_t)d->B * d->Sq * d->Hq * d->D, n_kv = (int64_t)d->B * d->Sk * d->Hkv * d->D;
  ST_TRY(check_tensor("q", q, d->dtype, n_q));
  ST_TRY(check_tensor("d_o", d_o, d->dtype, n_q));
  ST_TRY(check_tensor("k", k, d->dtype, n_kv));
  ST_TRY(check_tensor("v", v, d->dtype, n_kv));
  ST_TRY(check_f32("lse_final", lse_final, n_q));
  ST_TRY(check_f32("delta", delta, n_q));
  ST_TRY(check_f32("dq_acc", dq_acc, n_q));
  ST_TRY(check_f32("dk_acc", dk_acc, n_kv));
  ST_TRY(check_f32("dv_acc", dv_acc, n_kv));
  if (n_q == 0 || n_kv == 0) return ST_OK;
  if (d->causal && d->k_offset > st::q_pos(shape_of(d), d->Sq - 1)) return ST_OK;   // chunk entirely in the future
  st::BwdArgs a;
  memset(&a, 0, sizeof(a));
  a.s = shape_of(d);
  a.q = view_of(q);
  a.d_o = view_of(d_o);
  a.t.n = 1;
  a.t.k[0] = k->ptr; a.t.v[0] = v->ptr; a.t.k_offset[0] = d->k_offset;
  a.t.ksb = k->stride_b; a.t.kss = k->stride_s; a.t.ksh = k->stride_h;
  a.t.vsb = v->stride_b; a.t.vss = v->stride_s; a.t.vsh = v->stride_h;
  a.lse = lse_final; a.delta = delta; a.dq = dq_acc; a.dk[0] = dk_acc; a.dv[0] = dv_acc;
  if (d->dtype == ST_BF16 && workspace != nullptr) {
    if (workspace_bytes < st_attn_block_bwd_workspace_bytes(d)) return fail(ST_ERR_WORKSPACE, "block backward workspace needs %zu bytes", st_attn_block_bwd_workspace_bytes(d));
    if (reinterpret_cast<uintptr_t>(workspace) % 256) return fail(ST_ERR_ALIGNMENT, "workspace: not 256-byte aligned");
    ST_HIP(st::launch_scale_q(a.q, workspace, d->B, d->Sq, d->Hq, d->D, d->scale, (hipStream_t)hip_stream), "scaled-Q launch");
    a.qs = workspace;
  }
  ST_HIP(launch_bwd(d->dtype, a, (hipStream_t)hip_stream), "st_attn_block_bwd launch");
  return ST_OK;
}

st_status st_cast_from_f32(const float* src, void* dst, int64_t n, int32_t dst_dtype, void* hip_stream) {
  if (n < 0) return fail(ST_ERR_INVALID_ARG, "negative n");
  if (dst_dtype != ST_F32 && dst_dtype != ST_BF16) return fail(ST_ERR_INVALID_ARG, "unknown dst_dtype");
  ST_TRY(check_f32("src", src, n));
  if (n > 0 && (dst == nullptr || reinterpret_cast<uintptr_t>(dst) % 16)) return fail(dst ? ST_ERR_ALIGNMENT : ST_ERR_INVALID_ARG, "dst: null or misaligned");
  ST_HIP(st::launch_cast(src, dst, n, dst_dtype, (hipStream_t)hip_stream), "st_cast_from_f32 launch");
  return ST_OK;
}

// Closed form of the schedule.  With S = P / C^2 teams per team group, the initial dispatch
// leaves GPU (team t, member a) holding the gathered KV of team (t mod S) * C + a, and every
// sub-ring step hands a buffer to the next team of the group, so at iteration i the GPU works on
// team buffer ((t - i) mod S) * C + a, i.e. sequence shards [buffer * C, buffer * C + C).
st_status st_visit_order(int32_t P, int32_t C, int32_t rank, int32_t* shard_idx, int32_t* member_of) {
  if (P < 1 || C < 1 || P % C != 0 || (P / C) % C != 0) return fail(ST_ERR_INVALID_ARG, "layout needs C >= 1 and C*C | P (P=%d C=%d)", P, C);
  if (rank < 0 || rank >= P) return fail(ST_ERR_INVALID_ARG, "rank %d outside 0..%d", rank, P - 1);
  if (!shard_idx || !member_of) return fail(ST_ERR_INVALID_ARG, "null output");
  const int32_t S = P / (C * C);
  const int32_t t = rank / C;
  int32_t n = 0;
  for (int32_t a = 0; a < C; ++a)
    for (int32_t i = 0; i < S; ++i) {
      const int32_t pos = ((t - i) % S + S) % S;
      const int32_t buffer = pos * C + a;
      for (int32_t c = 0; c < C; ++c, ++n) {
        shard_idx[n] = buffer * C + c;
        member_of[n] = a;
      }
    }
  return ST_OK;
}

// Iteration i of GPU (team t, member a) works on the gathered buffer of team ((t - i) mod S) * C + a,
// S = P / C^2 GPUs per sub-ring (closed form of the initial placement followed by i sub-ring passes).
st_status st_team_visit_order(int32_t P, int32_t C, int32_t rank, int32_t* team_buffer) {
  if (!team_buffer) return fail(ST_ERR_INVALID_ARG, "null output");
  if (P < 1 || C < 1 || P % C != 0 || (P / C) % C != 0) return fail(ST_ERR_INVALID_ARG, "layout needs C >= 1 and C*C | P (P=%d C=%d)", P, C);
  if (rank < 0 || rank >= P) return fail(ST_ERR_INVALID_ARG, "rank %d outside 0..%d", rank, P - 1);
  const int32_t S = P / (C * C), t = rank / C, a = rank % C;
  for (int32_t i = 0; i < S; ++i) {
    const int32_t pos = ((t - i) % S + S) % S;
    team_buffer[i] = pos * C + a;
  }
  return ST_OK;
}

// Iteration counts and exchanged bytes of plain ring attention and of the concentric layout for one
// attention block forward on one GPU (Section 3.2, "Theoretical Analysis", its three communication
// expressions with bandwidth W and latency L).  A ring step hands on one K and one V shard of N/P tokens; a sub-ring step hands on
// the C shards a team gathered; the team all-gather of Q, K, V and the reduce-scatter of O move
// (C - 1) / C of 4 tensors of C N / P tokens.
st_status st_schedule_report(int32_t P, int32_t C, int64_t B, int64_t N, int64_t H, int32_t e, double W, double L,
                             st_comm_report* out) {
  if (!out) return fail(ST_ERR_INVALID_ARG, "null output");
  if (P < 1 || C < 1 || P % C != 0 || (P / C) % C != 0) return fail(ST_ERR_INVALID_ARG, "layout needs C >= 1 and C*C | P (P=%d C=%d)", P, C);
  if (B < 1 || N < 1 || H < 1 || e < 1 || N % P != 0) return fail(ST_ERR_INVALID_ARG, "sizes must be positive and P must divide N");
  if (!(W > 0.0) || !(L >= 0.0)) return fail(ST_ERR_INVALID_ARG, "bandwidth must be positive and latency non-negative");
  const __int128 shard = (__int128)B * (N / P) * H * e;            // bytes of one tensor's shard on one GPU
  const __int128 limit = ((__int128)1 << 62);
  if (shard * 4 * P > limit) return fail(ST_ERR_INVALID_ARG, "sizes overflow 64-bit byte counts");
  out->ring_iterations = P - 1;
  out->startrail_iterations = P / (C * C) - 1;
  out->ring_p2p_bytes_per_iter = (int64_t)(2 * shard);
  out->startrail_p2p_bytes_per_iter = (int64_t)(2 * shard * C);
  out->ring_p2p_bytes = out->ring_p2p_bytes_per_iter * out->ring_iterations;
  out->startrail_p2p_bytes = out->startrail_p2p_bytes_per_iter * out->startrail_iterations;
  out->startrail_collective_bytes = (int64_t)(4 * shard * (C - 1));
  out->ring_p2p_seconds = out->ring_iterations * ((double)out->ring_p2p_bytes_per_iter / W + L);
  out->startrail_p2p_seconds = out->startrail_iterations * ((double)out->startrail_p2p_bytes_per_iter / W + L);
  out->startrail_collective_seconds = (double)out->startrail_collective_bytes / W;
  return ST_OK;
}

// A fused bf16 forward whose query tiles alone would leave most of the chip idle (fewer than 128 workgroups
// of 256 queries on 256 compute units) is split over the visited chunks: every query tile gets several
// workgroups, each with a contiguous share of the chunks and a partial state of its own, and one combine
// pass folds the states (the chunks of a ring step are independent until the fold, Algorithm 1).
int fwd_splits(const st_ring_desc* d, int n_visible) {
  if (d->dtype != ST_BF16 || (d->D != 128 && d->D != 64) || n_visible < 2 || n_visible > st::kMaxTable) return 1;
  if (d->Sq < st::kQTileFastRows || d->Sk < st::kQTileFastKeys) return 1;
  const int64_t wgs = (int64_t)d->B * d->Hq * (d->Sq / st::kQTileFastRows);
  if (wgs >= 128) return 1;
  int64_t n = 256 / wgs;
  if (n > n_visible) n = n_visible;
  if (n > 16) n = 16;
  return (int)n;
}

// Workspace layout (each block 256-byte aligned):
//   forward, stepwise: partial O, partial lse, member O, member lse
//   forward, fused:    partial O and partial lse, once (when more than one launch is needed) or once per
//                      split of an under-filled launch plus one for its masked / ragged tiles: [O_0, lse_0, O_1, ...]
//   backward:          Delta, the tile counters of the dK/dV launch (kQueueInts ints), and for the bf16 dtype
//                      Q' = bf16(Q scale log2 e), dense [B,Sq,Hq,D]
size_t st_ring_workspace_bytes(const st_ring_desc* d, int32_t mode, int32_t backward) {
  if (d == nullptr) return 0;
  const size_t n_o = align_up((size_t)d->B * d->Sq * d->Hq * d->D * sizeof(float), 256);
  const size_t n_l = align_up((size_t)d->B * d->Sq * d->Hq * sizeof(float), 256);
  if (backward)
    return n_l + align_up(st::kQueueInts * sizeof(int32_t), 256) + (d->dtype == ST_BF16 ? align_up(n_o / 2, 256) : 0);
  if (mode == ST_RING_STEPWISE) return 2 * (n_o + n_l);
  // the split grows with the number of visited chunks up to one launch's table, and any subset may be visited
  const int n_most = d->n_chunks < st::kMaxTable ? d->n_chunks : st::kMaxTable;
  const int splits = fwd_splits(d, n_most);
  return (size_t)(splits > 1 ? splits + 1 : 1) * (n_o + n_l);
}

st_status st_ring_fwd(const st_ring_desc* d, const st_tensor* q, const int32_t* order, const int32_t* member_of,
                      int32_t n_visit, int32_t mode, float* o_acc, float* lse, void* o_lowp, void* workspace,
                      size_t workspace_bytes, void* hip_stream) {
  ST_TRY(check_ring(d, q, order, n_visit));
  if (mode != ST_RING_STEPWISE && mode != ST_RING_FUSED) return fail(ST_ERR_INVALID_ARG, "unknown mode %d", mode);
  const int64_t n_o = (int64_t)d->B * d->Sq * d->Hq * d->D, n_l = (int64_t)d->B * d->Sq * d->Hq;
  ST_TRY(check_f32("o_acc", o_acc, n_o));
  ST_TRY(check_f32("lse", lse, n_o));
  if (o_lowp && reinterpret_cast<uintptr_t>(o_lowp) % 16) return fail(ST_ERR_ALIGNMENT, "o_lowp: not 16-byte aligned");
  if (n_o == 0) return ST_OK;
  hipStream_t stream = (hipStream_t)hip_stream;

  // visible chunks in visit order
  int vis[ST_MAX_CHUNKS], mem[ST_MAX_CHUNKS], n = 0;
  for (int x = 0; x < n_visit; ++x)
    if (!chunk_invisible(d, order[x])) {
      vis[n] = order[x];
      mem[n] = member_of ? member_of[x] : 0;
      ++n;
    }

  const size_t b_o = align_up((size_t)n_o * sizeof(float), 256), b_l = align_up((size_t)n_l * sizeof(float), 256);
  st::FwdArgs a;
  memset(&a, 0, sizeof(a));
  a.s = shape_of(d);
  a.q = view_of(q);
  set_table_strides(a.t, d);
  int splits = mode == ST_RING_FUSED ? fwd_splits(d, n) : 1;
  if (splits > 1 && !st::fwd_fast_usable(a)) splits = 1;      // only the hand-scheduled kernel pair walks a split table
  const bool need_ws = mode == ST_RING_STEPWISE || n > st::kMaxTable || splits > 1;
  if (need_ws) {
    if (workspace == nullptr || workspace_bytes < st_ring_workspace_bytes(d, mode, 0)) return fail(ST_ERR_WORKSPACE, "forward workspace needs %zu bytes", st_ring_workspace_bytes(d, mode, 0));
    if (reinterpret_cast<uintptr_t>(workspace) % 256) return fail(ST_ERR_ALIGNMENT, "workspace: not 256-byte aligned");
  }
  char* ws = (char*)workspace;
  float* part_o = (float*)ws;
  float* part_l = (float*)(ws + b_o);

  if (mode == ST_RING_FUSED && splits > 1) {
    a.t.n = n;
    for (int x = 0; x < n; ++x) {
      a.t.k[x] = d->k_ptr[vis[x]];
      a.t.v[x] = d->v_ptr[vis[x]];
      a.t.k_offset[x] = d->k_offset[vis[x]];
    }
    a.o = part_o;
    a.lse = part_l;
    a.o_lowp = nullptr;
    a.n_split = splits;
    a.split_o = a.split_l = (int64_t)((b_o + b_l) / sizeof(float));
    ST_HIP(launch_fwd(d->dtype, a, stream), "split forward launch");
    st::CombineArgs c;
    memset(&c, 0, sizeof(c));
    c.n = splits + 1;                               // one state per split, and the general workgroups' own
    for (int y = 0; y < splits + 1; ++y) {
      c.o[y] = part_o + (int64_t)y * a.split_o;
      c.lse[y] = part_l + (int64_t)y * a.split_l;
    }
    c.B = d->B; c.Sq_in = d->Sq; c.Hq = d->Hq; c.D = d->D; c.row0 = 0; c.Sq_out = d->Sq;
    c.o_out = o_acc; c.lse_out = lse; c.o_lowp = o_lowp;
    ST_HIP(st::launch_combine(c, d->dtype, stream), "combine launch");
    return ST_OK;
  }

  if (mode == ST_RING_FUSED) {
    // one launch per kMaxTable visible chunks; further launches go through a partial state + merge
    if (n == 0) {
      ST_HIP(st::launch_fill_state(o_acc, lse, n_o, n_l, stream), "state fill");
      if (o_lowp) ST_HIP(st::launch_cast(o_acc, o_lowp, n_o, d->dtype, stream), "cast");
      return ST_OK;
    }
    for (int x0 = 0; x0 < n; x0 += st::kMaxTable) {
      const int cnt = n - x0 < st::kMaxTable ? n - x0 : st::kMaxTable;
      a.t.n = cnt;
      for (int x = 0; x < cnt; ++x) {
        a.t.k[x] = d->k_ptr[vis[x0 + x]];
        a.t.v[x] = d->v_ptr[vis[x0 + x]];
        a.t.k_offset[x] = d->k_offset[vis[x0 + x]];
      }
      const bool single = n <= st::kMaxTable;
      a.o = x0 == 0 ? o_acc : part_o;
      a.lse = x0 == 0 ? lse : part_l;
      a.o_lowp = single ? o_lowp : nullptr;
      ST_HIP(launch_fwd(d->dtype, a, stream), "fused forward launch");
      if (x0 > 0) {
        const bool last = x0 + cnt >= n;
        ST_HIP(st::launch_merge(o_acc, lse, part_o, part_l, d->B, d->Sq, d->Hq, d->D, last ? o_lowp : nullptr,
                                d->dtype, stream), "merge launch");
      }
    }
    return ST_OK;
  }

  // stepwise: per member a running state (Algorithm 1 loop), then the combine of the member states
  float* mem_o = (float*)(ws + b_o + b_l);
  float* mem_l = (float*)(ws + 2 * b_o + b_l);
  ST_HIP(st::launch_fill_state(o_acc, lse, n_o, n_l, stream), "state fill");
  a.t.n = 1;
  a.o = part_o; a.lse = part_l; a.o_lowp = nullptr;
  int x = 0;
  while (x < n) {
    const int member = mem[x];
    ST_HIP(st::launch_fill_state(mem_o, mem_l, n_o, n_l, stream), "state fill");
    for (; x < n && mem[x] == member; ++x) {
      a.t.k[0] = d->k_ptr[vis[x]];
      a.t.v[0] = d->v_ptr[vis[x]];
      a.t.k_offset[0] = d->k_offset[vis[x]];
      ST_HIP(launch_fwd(d->dtype, a, stream), "block forward launch");
      ST_HIP(st::launch_merge(mem_o, mem_l, part_o, part_l, d->B, d->Sq, d->Hq, d->D, nullptr, d->dtype, stream), "merge launch");
    }
    ST_HIP(st::launch_merge(o_acc, lse, mem_o, mem_l, d->B, d->Sq, d->Hq, d->D, nullptr, d->dtype, stream), "combine launch");
  }
  if (o_lowp) ST_HIP(st::launch_cast(o_acc, o_lowp, n_o, d->dtype, stream), "cast");
  return ST_OK;
}

st_status st_ring_bwd(const st_ring_desc* d, const st_tensor* q, const st_tensor* d_o, const st_tensor* o,
                      int32_t o_dtype, const float* lse_final, const int32_t* order, int32_t n_visit, int32_t mode,
                      float* dq_acc, float* const* dk_acc, float* const* dv_acc, void* workspace,
                      size_t workspace_bytes, void* hip_stream) {
  return st_ring_bwd_last(d, q, d_o, o, o_dtype, lse_final, order, n_visit, mode, dq_acc, dk_acc, dv_acc, 0, nullptr,
                          nullptr, workspace, workspace_bytes, hip_stream);
}

st_status st_ring_bwd_noalloc(const st_ring_desc* d, const st_tensor* q, const st_tensor* d_o, const st_tensor* o,
                              int32_t o_dtype, const float* lse_final, const int32_t* order, int32_t n_visit,
                              int32_t mode, float* dq_acc, float* const* dk_acc, float* const* dv_acc, void* hip_stream) {
  if (d == nullptr) return fail(ST_ERR_INVALID_ARG, "null descriptor");
  ST_TRY(check_shape(d->dtype, d->B, d->Hq, d->Hkv, d->D, d->Sq, d->Sk));
  const size_t need = st_ring_workspace_bytes(d, mode, 1);
  if (need > kScratchBytes)
    return fail(ST_ERR_WORKSPACE, "st_ring_bwd_noalloc: this share needs %zu bytes of scratch, the library's static scratch holds %zu; use st_ring_bwd with a workspace", need, kScratchBytes);
  void* ws = nullptr;
  ST_TRY(scratch_of_current_device(&ws));
  return st_ring_bwd_last(d, q, d_o, o, o_dtype, lse_final, order, n_visit, mode, dq_acc, dk_acc, dv_acc, 0, nullptr,
                          nullptr, ws, kScratchBytes, hip_stream);
}

size_t st_ring_bwd_noalloc_max_bytes(void) { return kScratchBytes; }

st_status st_ring_bwd_last(const st_ring_desc* d, const st_tensor* q, const st_tensor* d_o, const st_tensor* o,
                           int32_t o_dtype, const float* lse_final, const int32_t* order, int32_t n_visit,
                           int32_t mode, float* dq_acc, float* const* dk_acc, float* const* dv_acc, int32_t kv_flags,
                           void* const* dk_lowp, void* const* dv_lowp, void* workspace, size_t workspace_bytes,
                           void* hip_stream) {
  ST_TRY(check_ring(d, q, order, n_visit));
  if (mode != ST_RING_STEPWISE && mode != ST_RING_FUSED) return fail(ST_ERR_INVALID_ARG, "unknown mode %d", mode);
  if (o_dtype != ST_F32 && o_dtype != d->dtype) return fail(ST_ERR_INVALID_ARG, "o_dtype must be ST_F32 or the storage dtype");
  const int64_t n_o = (int64_t)d->B * d->Sq * d->Hq * d->D, n_kv = (int64_t)d->B * d->Sk * d->Hkv * d->D;
  ST_TRY(check_tensor("d_o", d_o, d->dtype, n_o));
  ST_TRY(check_tensor("o", o, o_dtype, n_o));
  ST_TRY(check_f32("lse_final", lse_final, n_o));
  ST_TRY(check_f32("dq_acc", dq_acc, n_o));
  if (n_visit > 0 && (!dk_acc || !dv_acc)) return fail(ST_ERR_INVALID_ARG, "null gradient tables");
  if (kv_flags & ~ST_KV_ASSIGN) return fail(ST_ERR_INVALID_ARG, "unknown kv_flags %d", kv_flags);
  if ((dk_lowp == nullptr) != (dv_lowp == nullptr)) return fail(ST_ERR_INVALID_ARG, "dk_lowp and dv_lowp: both or neither");
  if (dk_lowp && d->dtype != ST_BF16) return fail(ST_ERR_UNSUPPORTED, "bf16 copies of dK / dV need an ST_BF16 descriptor");
  const bool assign = (kv_flags & ST_KV_ASSIGN) != 0;
  const bool no_rows = n_o == 0;                     // no query rows: every contribution is zero
  if (no_rows && !assign && !dk_lowp) return ST_OK;
  if (!no_rows) {
    if (workspace == nullptr || workspace_bytes < st_ring_workspace_bytes(d, mode, 1)) return fail(ST_ERR_WORKSPACE, "backward workspace needs %zu bytes", st_ring_workspace_bytes(d, mode, 1));
    if (reinterpret_cast<uintptr_t>(workspace) % 256) return fail(ST_ERR_ALIGNMENT, "workspace: not 256-byte aligned");
  }
  hipStream_t stream = (hipStream_t)hip_stream;
  auto unseen = [&](int j) { return no_rows || chunk_invisible(d, j); };

  int vis[ST_MAX_CHUNKS], n = 0;
  for (int x = 0; x < n_visit; ++x) {
    const int j = order[x];
    void* lk = dk_lowp ? dk_lowp[j] : nullptr;
    void* lv = dk_lowp ? dv_lowp[j] : nullptr;
    if ((lk == nullptr) != (lv == nullptr)) return fail(ST_ERR_INVALID_ARG, "dk_lowp[%d] and dv_lowp[%d]: both or neither", j, j);
    if (lk && (reinterpret_cast<uintptr_t>(lk) % 16 || reinterpret_cast<uintptr_t>(lv) % 16))
      return fail(ST_ERR_ALIGNMENT, "dk_lowp[%d] / dv_lowp[%d]: not 16-byte aligned", j, j);
    const bool hidden = unseen(j);
    if (!hidden || assign || lk) {
      ST_TRY(check_f32("dk_acc[j]", dk_acc[j], n_kv));
      ST_TRY(check_f32("dv_acc[j]", dv_acc[j], n_kv));
    }
    if (!hidden) vis[n++] = j;
  }
  // a listed chunk nobody sees: its contribution is zero
  for (int x = 0; x < n_visit; ++x) {
    const int j = order[x];
    if (!unseen(j) || n_kv == 0) continue;
    if (assign) {
      ST_HIP(st::launch_zero(dk_acc[j], n_kv * (int64_t)sizeof(float), stream), "dk_acc fill");
      ST_HIP(st::launch_zero(dv_acc[j], n_kv * (int64_t)sizeof(float), stream), "dv_acc fill");
    }
    if (dk_lowp && dk_lowp[j]) {
      ST_HIP(st::launch_cast(dk_acc[j], dk_lowp[j], n_kv, d->dtype, stream), "dk cast");
      ST_HIP(st::launch_cast(dv_acc[j], dv_lowp[j], n_kv, d->dtype, stream), "dv cast");
    }
  }
  if (no_rows) return ST_OK;

  float* delta = (float*)workspace;
  ST_HIP(st::launch_delta(view_of(d_o), d->dtype, view_of(o), o_dtype, delta, d->B, d->Sq, d->Hq, d->D, stream), "delta launch");

  st::BwdArgs a;
  memset(&a, 0, sizeof(a));
  a.s = shape_of(d);
  a.q = view_of(q);
  a.d_o = view_of(d_o);
  set_table_strides(a.t, d);
  a.lse = lse_final; a.delta = delta; a.dq = dq_acc;
  a.queue = (int32_t*)((char*)workspace + align_up((size_t)d->B * d->Sq * d->Hq * sizeof(float), 256));
  if (d->dtype == ST_BF16) {
    void* qs = (char*)a.queue + align_up(st::kQueueInts * sizeof(int32_t), 256);
    ST_HIP(st::launch_scale_q(a.q, qs, d->B, d->Sq, d->Hq, d->D, d->scale, stream), "scaled-Q launch");
    a.qs = qs;
  }
  const int per_launch = mode == ST_RING_FUSED ? st::kMaxTable : 1;
  for (int x0 = 0; x0 < n; x0 += per_launch) {
    const int cnt = n - x0 < per_launch ? n - x0 : per_launch;
    a.t.n = cnt;
    for (int x = 0; x < cnt; ++x) {
      const int j = vis[x0 + x];
      a.t.k[x] = d->k_ptr[j]; a.t.v[x] = d->v_ptr[j]; a.t.k_offset[x] = d->k_offset[j];
      a.dk[x] = dk_acc[j]; a.dv[x] = dv_acc[j];
      a.dk_lowp[x] = dk_lowp ? dk_lowp[j] : nullptr;
      a.dv_lowp[x] = dk_lowp ? dv_lowp[j] : nullptr;
    }
    a.kv_assign = assign ? ~0ull : 0ull;
    if (d->dtype != ST_BF16 && assign)              // the fp32 kernels only add
      for (int x = 0; x < cnt; ++x) {
        ST_HIP(st::launch_zero(a.dk[x], n_kv * (int64_t)sizeof(float), stream), "dk_acc fill");
        ST_HIP(st::launch_zero(a.dv[x], n_kv * (int64_t)sizeof(float), stream), "dv_acc fill");
      }
    ST_HIP(launch_bwd(d->dtype, a, stream), "backward launch");
  }
  return ST_OK;
}

}  // extern "C"
