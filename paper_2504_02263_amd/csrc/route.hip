// Routing kernels: top-k selection with softmax over the picks, then per-expert counts and
// offsets (paper Section 2.2 for the routing rule; Section 6 "Fused kernels" for the list of
// by-products: token counts per expert and normalised token weights).
#include <limits.h>
#include "moe_internal.h"

namespace moe {
namespace {

constexpr int kMaxPerLane = 4;  // experts held per lane: E <= 64 * 4

// A group of L lanes (L = 8, 16, 32 or 64, a power of two >= min(E, 64)) owns one token; lane sl
// of the group holds experts sl, sl + L, sl + 2L, ... The k picks are k rounds of an argmax
// butterfly over the group on (value, index) pairs: larger value wins, equal values go to the
// lower index. After a round every lane of the group knows the winner; its owner retires it.
template <int L>
__global__ __launch_bounds__(256) void route_topk_kernel(const float* __restrict__ logits, int T, int E, int k,
                                                         int32_t* __restrict__ topk_idx,
                                                         float* __restrict__ topk_w) {
  constexpr int kTokensPerWave = 64 / L;
  const int lane = threadIdx.x & 63;
  const int wave = (blockIdx.x * 256 + threadIdx.x) >> 6;
  const int sl = lane % L;
  const int t = wave * kTokensPerWave + lane / L;
  const bool valid = t < T;

  float v[kMaxPerLane];
#pragma unroll
  for (int i = 0; i < kMaxPerLane; ++i) {
    const int e = sl + i * L;
    float x = -INFINITY;
    if (valid && e < E) {
      x = logits[(size_t)t * E + e];
      if (x != x) x = -INFINITY;  // NaN ranks as -inf
    }
    v[i] = x;
  }

  unsigned taken = 0;
  float row_max = 0.f, sum = 0.f, my_p = 0.f;
  int my_idx = 0;
  for (int j = 0; j < k; ++j) {
    float bv = -INFINITY;
    int bi = INT_MAX;
#pragma unroll
    for (int i = 0; i < kMaxPerLane; ++i) {
      const int e = sl + i * L;
      if (e < E && !((taken >> i) & 1u) && (bi == INT_MAX || v[i] > bv)) {
        bv = v[i];
        bi = e;
      }
    }
#pragma unroll
    for (int off = L / 2; off >= 1; off >>= 1) {
      const float ov = __shfl_xor(bv, off);
      const int oi = __shfl_xor(bi, off);
      if (ov > bv || (ov == bv && oi < bi)) {
        bv = ov;
        bi = oi;
      }
    }
    if (bi != INT_MAX && sl == bi % L) taken |= 1u << (bi / L);
    if (j == 0) row_max = bv;
    const float p = expf(bv - row_max);
    sum += p;  // every lane adds the picks in order j = 0, 1, ...
    if (sl == j) {
      my_p = p;
      my_idx = bi;
    }
  }
  if (valid && sl < k) {
    topk_idx[(size_t)t * k + sl] = my_idx;
    topk_w[(size_t)t * k + sl] = my_p / sum;
  }
}

// One workgroup: histogram of the A picks in LDS, then an exclusive scan over E <= 256 bins by
// the first wavefront (4 bins per lane).
__global__ __launch_bounds__(1024) void route_count_kernel(const int32_t* __restrict__ topk_idx, int A, int E,
                                                           int32_t* __restrict__ counts,
                                                           int32_t* __restrict__ offsets) {
  __shared__ int hist[kMaxExperts];
  const int tid = threadIdx.x;
  if (tid < kMaxExperts) hist[tid] = 0;
  __syncthreads();
  for (int i = tid; i < A; i += 1024) {
    const int e = topk_idx[i];
    if ((unsigned)e < (unsigned)E) atomicAdd(&hist[e], 1);
  }
  __syncthreads();
  if (tid < 64) {
    int c[4], s = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      c[i] = hist[tid * 4 + i];  // bins >= E are zero
      s += c[i];
    }
    int incl = s;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int o = __shfl_up(incl, off);
      if (tid >= off) incl += o;
    }
    int run = incl - s;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = tid * 4 + i;
      if (e < E) {
        counts[e] = c[i];
        offsets[e] = run;
      }
      run += c[i];
      if (e == E - 1) offsets[E] = run;
    }
  }
}

}  // namespace

hipError_t launch_route(const float* logits, int T, int E, int k, int32_t* topk_idx, float* topk_w, int32_t* counts,
                        int32_t* offsets, hipStream_t stream) {
  if (T > 0) {
    const int L = E <= 8 ? 8 : E <= 16 ? 16 : E <= 32 ? 32 : 64;
    const int tokens_per_block = 4 * (64 / L);
    const dim3 grid((T + tokens_per_block - 1) / tokens_per_block), block(256);
    switch (L) {
      case 8: hipLaunchKernelGGL(route_topk_kernel<8>, grid, block, 0, stream, logits, T, E, k, topk_idx, topk_w); break;
      case 16: hipLaunchKernelGGL(route_topk_kernel<16>, grid, block, 0, stream, logits, T, E, k, topk_idx, topk_w); break;
      case 32: hipLaunchKernelGGL(route_topk_kernel<32>, grid, block, 0, stream, logits, T, E, k, topk_idx, topk_w); break;
      default: hipLaunchKernelGGL(route_topk_kernel<64>, grid, block, 0, stream, logits, T, E, k, topk_idx, topk_w); break;
    }
  }
  hipLaunchKernelGGL(route_count_kernel, dim3(1), dim3(1024), 0, stream, topk_idx, T * k, E, counts, offsets);
  return hipGetLastError();
}

}  // namespace moe
