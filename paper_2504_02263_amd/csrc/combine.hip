// Combine: out[t, :] = sum_j topk_w[t, j] * y[pos[t, j], :] (paper Section 2.2: the layer output
// is the weighted sum of the selected experts' outputs). A gather of k rows per token with a
// float32 accumulator; bound by HBM/L2 bandwidth.
#include "moe_internal.h"

namespace moe {
namespace {

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 v = {(__bf16)a, (__bf16)b};  // round to nearest even
  return __builtin_bit_cast(uint32_t, v);
}

// grid (T, ceil(d/8/256)): one 16-byte column chunk (8 bf16) per thread.
__global__ __launch_bounds__(256) void combine_bf16_kernel(const uint4* __restrict__ y,
                                                           const int32_t* __restrict__ pos,
                                                           const float* __restrict__ topk_w, int A, int k,
                                                           int row_vecs, uint4* __restrict__ out) {
  const int t = blockIdx.x;
  const int c = blockIdx.y * 256 + threadIdx.x;
  if (c >= row_vecs) return;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int j = 0; j < k; ++j) {
    const int r = pos[(size_t)t * k + j];
    if ((unsigned)r >= (unsigned)A) continue;
    const float w = topk_w[(size_t)t * k + j];
    const uint4 v = y[(size_t)r * row_vecs + c];
    acc[0] = fmaf(w, bf16_lo(v.x), acc[0]);
    acc[1] = fmaf(w, bf16_hi(v.x), acc[1]);
    acc[2] = fmaf(w, bf16_lo(v.y), acc[2]);
    acc[3] = fmaf(w, bf16_hi(v.y), acc[3]);
    acc[4] = fmaf(w, bf16_lo(v.z), acc[4]);
    acc[5] = fmaf(w, bf16_hi(v.z), acc[5]);
    acc[6] = fmaf(w, bf16_lo(v.w), acc[6]);
    acc[7] = fmaf(w, bf16_hi(v.w), acc[7]);
  }
  uint4 o;
  o.x = pack_bf16(acc[0], acc[1]);
  o.y = pack_bf16(acc[2], acc[3]);
  o.z = pack_bf16(acc[4], acc[5]);
  o.w = pack_bf16(acc[6], acc[7]);
  out[(size_t)t * row_vecs + c] = o;
}

// grid (T, ceil(d/4/256)): one float4 per thread.
__global__ __launch_bounds__(256) void combine_f32_kernel(const float4* __restrict__ y,
                                                          const int32_t* __restrict__ pos,
                                                          const float* __restrict__ topk_w, int A, int k,
                                                          int row_vecs, float4* __restrict__ out) {
  const int t = blockIdx.x;
  const int c = blockIdx.y * 256 + threadIdx.x;
  if (c >= row_vecs) return;
  float4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int j = 0; j < k; ++j) {
    const int r = pos[(size_t)t * k + j];
    if ((unsigned)r >= (unsigned)A) continue;
    const float w = topk_w[(size_t)t * k + j];
    const float4 v = y[(size_t)r * row_vecs + c];
    acc.x = fmaf(w, v.x, acc.x);
    acc.y = fmaf(w, v.y, acc.y);
    acc.z = fmaf(w, v.z, acc.z);
    acc.w = fmaf(w, v.w, acc.w);
  }
  out[(size_t)t * row_vecs + c] = acc;
}

}  // namespace

hipError_t launch_combine(const void* y, const int32_t* pos, const float* topk_w, int T, int k, int d, int dtype,
                          void* out, hipStream_t stream) {
  if (T == 0) return hipSuccess;
  const int A = T * k;
  if (dtype == MOE_BF16) {
    const int row_vecs = d / 8;
    hipLaunchKernelGGL(combine_bf16_kernel, dim3(T, (row_vecs + 255) / 256), dim3(256), 0, stream,
                       static_cast<const uint4*>(y), pos, topk_w, A, k, row_vecs, static_cast<uint4*>(out));
  } else {
    const int row_vecs = d / 4;
    hipLaunchKernelGGL(combine_f32_kernel, dim3(T, (row_vecs + 255) / 256), dim3(256), 0, stream,
                       static_cast<const float4*>(y), pos, topk_w, A, k, row_vecs, static_cast<float4*>(out));
  }
  return hipGetLastError();
}

}  // namespace moe
