// Benchmark aid, not part of the method: a loop of nothing but v_mfma_f32_32x32x16_bf16 on caller-supplied
// operands.  It measures what the matrix units of the device sustain on given data (the rate depends on the
// data: the chip runs at its power limit), the ceiling the attention kernels are compared with.
#include "st_internal.h"
#include "st_mfma.h"

namespace st {
namespace {

constexpr int kProbeFrags = 16;        // operand fragments per lane: 8 A and 8 B, 16 bytes each
constexpr int kProbeMfmaPerIter = 32;  // MFMAs per wavefront and loop iteration

__global__ __launch_bounds__(256, 1) void mfma_probe_kernel(const u32x4* __restrict__ in, int64_t n_frag,
                                                            int32_t iters, float* __restrict__ sink) {
  u32x4 a[8], b[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = in[((int64_t)blockIdx.x * 256 * kProbeFrags + threadIdx.x + 256 * i) % n_frag];
    b[i] = in[((int64_t)blockIdx.x * 256 * kProbeFrags + threadIdx.x + 256 * (i + 8)) % n_frag];
  }
  f32x16 c0 = {}, c1 = {}, c2 = {}, c3 = {};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {      // four independent accumulators: back-to-back issue, no dependent pair
      c0 = mfma32(__builtin_bit_cast(bf16x8, a[i]), __builtin_bit_cast(bf16x8, b[i]), c0);
      c1 = mfma32(__builtin_bit_cast(bf16x8, a[i]), __builtin_bit_cast(bf16x8, b[(i + 1) & 7]), c1);
      c2 = mfma32(__builtin_bit_cast(bf16x8, a[(i + 1) & 7]), __builtin_bit_cast(bf16x8, b[i]), c2);
      c3 = mfma32(__builtin_bit_cast(bf16x8, a[(i + 2) & 7]), __builtin_bit_cast(bf16x8, b[(i + 3) & 7]), c3);
    }
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
  sink[(int64_t)blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace

int mfma_probe_blocks() {
  const DeviceInfo& d = device_info();
  return d.cus > 0 ? d.cus : 256;
}

double mfma_probe_flop(int blocks, int32_t iters) {
  return (double)blocks * 4 * (double)iters * kProbeMfmaPerIter * (2.0 * 32 * 32 * 16);
}

hipError_t launch_mfma_probe(const void* operands, int64_t operand_bytes, int32_t iters, float* sink, int blocks,
                             hipStream_t s) {
  ProfScope prof("mfma_probe", s);
  hipLaunchKernelGGL(mfma_probe_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (const u32x4*)operands,
                     operand_bytes / 16, iters, sink);
  return hipGetLastError();
}

}  // namespace st
