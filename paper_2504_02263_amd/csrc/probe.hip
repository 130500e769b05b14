// Two measuring kernels for the roofline's denominators (paper Section 2.3: a GEMM is bound by the
// memory bandwidth B below the ridge batch F / B and by the peak compute F above it). They do no
// part of the layer; a benchmark times them next to the layer's kernels to state what this very
// chip reaches for B (a plain streaming read) and F (matrix-core issue from registers only).
#include "moe_internal.h"

namespace moe {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Every wavefront reads its own contiguous share of the buffer, 16 bytes per lane per load, 16 loads
// in flight, non-temporal (the access pattern of the weight stream). The XOR of everything read is
// stored only if it equals a value it cannot take in practice, which keeps the loads alive.
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4* __restrict__ buf, size_t units_per_wave,
                                                          int waves, u32x4* __restrict__ sink) {
  const int lane = threadIdx.x & 63;
  const int wave = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (wave >= waves) return;
  const u32x4* p = buf + (size_t)wave * units_per_wave + lane;
  u32x4 acc = {0u, 0u, 0u, 0u};
  size_t i = 0;
  for (; i + 16 * 64 <= units_per_wave; i += 16 * 64) {
    u32x4 v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) v[u] = __builtin_nontemporal_load(p + i + u * 64);
#pragma unroll
    for (int u = 0; u < 16; ++u) acc ^= v[u];
  }
  for (; i + 64 <= units_per_wave; i += 64) acc ^= __builtin_nontemporal_load(p + i);
  if (acc[0] == 0x9e3779b9u && acc[1] == 0x7f4a7c15u && acc[2] == 0xf39cc060u && acc[3] == 0x5cedc834u) sink[0] = acc;
}

// 16 independent accumulator tiles per wavefront, one wavefront per SIMD (the large-batch GEMM's
// occupancy), v_mfma_f32_32x32x16_bf16 issued back to back from registers. Operands are 2 KiB of
// caller data (real weights: the matrix cores' power draw, and with it the clock, depends on the
// bit patterns multiplied). Values that are not finite are replaced so the sums stay finite.
__global__ __launch_bounds__(256) void mfma_loop_kernel(const u32x4* __restrict__ operands, int iters,
                                                        float* __restrict__ sink) {
  const int lane = threadIdx.x & 63;
  u32x4 ra = operands[lane], rb = operands[64 + lane];
#pragma unroll
  for (int j = 0; j < 4; ++j) {  // clear the top exponent bit of each bf16: |value| < 2, no inf / NaN
    ra[j] &= 0xbfffbfffu;
    rb[j] &= 0xbfffbfffu;
  }
  const bf16x8 a = __builtin_bit_cast(bf16x8, ra), b = __builtin_bit_cast(bf16x8, rb);
  floatx16 acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += acc[i][lane & 15];
  if (s == 12345.678f) sink[0] = s;
}

}  // namespace

hipError_t launch_probe_stream_read(const void* buf, size_t bytes, void* sink, hipStream_t stream) {
  const int waves = 4096;
  const size_t units_per_wave = bytes / 16 / waves / 64 * 64;  // whole 1 KiB loads only
  if (units_per_wave == 0) return hipSuccess;
  hipLaunchKernelGGL(stream_read_kernel, dim3(waves / 4), dim3(256), 0, stream, static_cast<const u32x4*>(buf),
                     units_per_wave, waves, static_cast<u32x4*>(sink));
  return hipGetLastError();
}

size_t probe_stream_read_bytes(size_t bytes) { return bytes / 16 / 4096 / 64 * 64 * 16 * 4096; }

hipError_t launch_probe_mfma(const void* operands, int iters, int workgroups, void* sink, hipStream_t stream) {
  if (iters <= 0 || workgroups <= 0) return hipSuccess;
  hipLaunchKernelGGL(mfma_loop_kernel, dim3(workgroups), dim3(256), 0, stream, static_cast<const u32x4*>(operands),
                     iters, static_cast<float*>(sink));
  return hipGetLastError();
}

}  // namespace moe
