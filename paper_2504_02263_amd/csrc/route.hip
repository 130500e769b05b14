// Routing kernels: top-k selection with softmax over the picks, then per-expert counts and
// offsets (paper Section 2.2 for the routing rule; Section 6 "Fused kernels" for the list of
// by-products: token counts per expert and normalised token weights).
#include <limits.h>
#include "moe_internal.h"

namespace moe {
namespace {

constexpr int kMaxPerLane = 4;  // experts held per lane: E <= 64 * 4

// A group of L lanes (L = 8, 16, 32 or 64, a power of two >= min(E, 64)) owns one token; lane sl
// of the group holds experts sl, sl + L, sl + 2L, ... in v[]. The k picks are k rounds of an argmax
// butterfly over the group on (value, index) pairs: larger value wins, equal values go to the
// lower index. After a round every lane of the group knows the winner; its owner retires it.
// On return lane sl < k holds pick sl and its softmax-over-the-picks weight.
template <int L>
__device__ __forceinline__ void topk_group(const float (&v)[kMaxPerLane], int sl, int E, int k, int& my_idx,
                                           float& my_w) {
  unsigned taken = 0;
  float row_max = 0.f, sum = 0.f, my_p = 0.f;
  my_idx = 0;
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
  my_w = my_p / sum;
}

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
  int my_idx;
  float my_w;
  topk_group<L>(v, sl, E, k, my_idx, my_w);
  if (valid && sl < k) {
    topk_idx[(size_t)t * k + sl] = my_idx;
    topk_w[(size_t)t * k + sl] = my_w;
  }
}

// Gating GEMM fused with the top-k (the paper fuses these small memory-bound steps with the gating
// computation, Section 6 "Fused kernels"): logits[t, e] = sum_c x[t, c] * w_router[e, c] in float32.
// Workgroup = TT (16 or 32) tokens; thread (tok = tid % TT, eg = tid / TT) accumulates the EPT
// experts eg * EPT .. of its token over all of d, from LDS tiles of x (widened to float32) and
// w_router, 64 columns at a time; the next tile's global loads are in flight while the current one
// is consumed. The finished TT x E logits stay in LDS for the top-k (and go to HBM only if the
// caller asks for them).
template <int TT, int EPT, int L, bool BF16>
__global__ __launch_bounds__(256) void gate_topk_kernel(const void* __restrict__ x_, const float* __restrict__ wr,
                                                        int T, int d, int E, int k, float* __restrict__ logits,
                                                        int32_t* __restrict__ topk_idx, float* __restrict__ topk_w) {
  constexpr int KC = 64, EG = 256 / TT, EMAX = EG * EPT;
  constexpr int WL = (EMAX * (KC / 4) + 255) / 256;  // float4 loads of the w_router tile per thread
  __shared__ float xs[TT][KC + 1];
  __shared__ float ws[EMAX][KC + 1];
  __shared__ float lg[TT][EMAX + 1];
  const int tid = threadIdx.x, tok = tid % TT, eg = tid / TT;
  const int t0 = blockIdx.x * TT;
  float acc[EPT];
#pragma unroll
  for (int j = 0; j < EPT; ++j) acc[j] = 0.f;

  // this thread's share of a tile: x row tid / 8, 8 columns at (tid % 8) * 8; w_router float4 number tid + 256 i
  const int xr = tid >> 3, xc = (tid & 7) * 8;
  const bool x_on = xr < TT && t0 + xr < T;
  uint4 xq = {0u, 0u, 0u, 0u};
  float4 xf[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
  float4 wq[WL];
  auto fetch = [&](int k0) {
    if (x_on) {
      if (BF16) {
        xq = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(x_) + (size_t)(t0 + xr) * d + k0 + xc);
      } else {
        const float* p = static_cast<const float*>(x_) + (size_t)(t0 + xr) * d + k0 + xc;
        xf[0] = *reinterpret_cast<const float4*>(p);
        xf[1] = *reinterpret_cast<const float4*>(p + 4);
      }
    }
#pragma unroll
    for (int i = 0; i < WL; ++i) {
      const int u = tid + 256 * i, e = u / (KC / 4), c = (u % (KC / 4)) * 4;
      wq[i] = e < E ? *reinterpret_cast<const float4*>(wr + (size_t)e * d + k0 + c) : float4{0.f, 0.f, 0.f, 0.f};
    }
  };
  auto stash = [&]() {
    if (xr < TT) {
      float f[8];
      if (BF16) {
        const uint32_t u[4] = {xq.x, xq.y, xq.z, xq.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          f[2 * i] = __uint_as_float(u[i] << 16);
          f[2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u);
        }
      } else {
        f[0] = xf[0].x; f[1] = xf[0].y; f[2] = xf[0].z; f[3] = xf[0].w;
        f[4] = xf[1].x; f[5] = xf[1].y; f[6] = xf[1].z; f[7] = xf[1].w;
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) xs[xr][xc + i] = f[i];
    }
#pragma unroll
    for (int i = 0; i < WL; ++i) {
      const int u = tid + 256 * i, e = u / (KC / 4), c = (u % (KC / 4)) * 4;
      if (e < EMAX) {
        ws[e][c] = wq[i].x; ws[e][c + 1] = wq[i].y; ws[e][c + 2] = wq[i].z; ws[e][c + 3] = wq[i].w;
      }
    }
  };

  fetch(0);
  for (int k0 = 0; k0 < d; k0 += KC) {
    stash();
    __syncthreads();
    if (k0 + KC < d) fetch(k0 + KC);
#pragma unroll 8
    for (int kk = 0; kk < KC; ++kk) {
      const float xv = xs[tok][kk];
#pragma unroll
      for (int j = 0; j < EPT; ++j) acc[j] = fmaf(xv, ws[eg * EPT + j][kk], acc[j]);  // rows >= E are zero
    }
    __syncthreads();
  }
#pragma unroll
  for (int j = 0; j < EPT; ++j) lg[tok][eg * EPT + j] = acc[j];
  __syncthreads();
  if (logits) {
    for (int u = tid; u < TT * E; u += 256) {
      const int r = u / E, e = u % E;
      if (t0 + r < T) logits[(size_t)(t0 + r) * E + e] = lg[r][e];
    }
  }
  // top-k: 256 / L tokens per pass
  const int sl = tid % L;
  for (int base = 0; base < TT; base += 256 / L) {
    const int r = base + tid / L;
    const bool valid = r < TT && t0 + r < T;
    float v[kMaxPerLane];
#pragma unroll
    for (int i = 0; i < kMaxPerLane; ++i) {
      const int e = sl + i * L;
      float q = -INFINITY;
      if (valid && e < E) {
        q = lg[r][e];
        if (q != q) q = -INFINITY;
      }
      v[i] = q;
    }
    int my_idx;
    float my_w;
    topk_group<L>(v, sl, E, k, my_idx, my_w);
    if (valid && sl < k) {
      topk_idx[(size_t)(t0 + r) * k + sl] = my_idx;
      topk_w[(size_t)(t0 + r) * k + sl] = my_w;
    }
  }
}

// The same fusion for few experts (E <= EM = 8 or 16), where the batch is too small to fill the
// chip with 16-token workgroups: one wavefront per token, lanes stride over d in 16-byte pieces,
// w_router comes from L2 (E * d * 4 bytes per token), no LDS and no barrier. Lane sums are combined
// by a butterfly, after which lane e of every EM-lane group holds logit e and the top-k runs in place.
template <int EM, bool BF16>
__global__ __launch_bounds__(256) void gate_topk_wave_kernel(const void* __restrict__ x_, const float* __restrict__ wr,
                                                             int T, int d, int E, int k, float* __restrict__ logits,
                                                             int32_t* __restrict__ topk_idx,
                                                             float* __restrict__ topk_w) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;  // whole wavefront
  float acc[EM];
#pragma unroll
  for (int e = 0; e < EM; ++e) acc[e] = 0.f;
  for (int c = lane * 8; c < d; c += 512) {
    float f[8];
    if (BF16) {
      const uint4 q = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(x_) + (size_t)t * d + c);
      const uint32_t u[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        f[2 * i] = __uint_as_float(u[i] << 16);
        f[2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u);
      }
    } else {
      const float* p = static_cast<const float*>(x_) + (size_t)t * d + c;
      const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
      f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w; f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
    }
#pragma unroll
    for (int e = 0; e < EM; ++e) {
      if (e < E) {
        const float* p = wr + (size_t)e * d + c;
        const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
        float s = acc[e];
        s = fmaf(f[0], a.x, s); s = fmaf(f[1], a.y, s); s = fmaf(f[2], a.z, s); s = fmaf(f[3], a.w, s);
        s = fmaf(f[4], b.x, s); s = fmaf(f[5], b.y, s); s = fmaf(f[6], b.z, s); s = fmaf(f[7], b.w, s);
        acc[e] = s;
      }
    }
  }
  const int sl = lane % EM;
  float mine = 0.f;
#pragma unroll
  for (int e = 0; e < EM; ++e) {
    float s = acc[e];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off);
    if (sl == e) mine = s;
  }
  if (logits && lane < E) logits[(size_t)t * E + lane] = mine;
  float v[kMaxPerLane];
#pragma unroll
  for (int i = 0; i < kMaxPerLane; ++i) v[i] = -INFINITY;
  if (sl < E) v[0] = mine != mine ? -INFINITY : mine;
  int my_idx;
  float my_w;
  topk_group<EM>(v, sl, E, k, my_idx, my_w);
  if (lane < k) {
    topk_idx[(size_t)t * k + lane] = my_idx;
    topk_w[(size_t)t * k + lane] = my_w;
  }
}

// Routing and dispatch pack in ONE launch for decode-sized batches (A = T*k <= kFusedMaxA): the
// paper's fused kernel does top-k, per-expert counts, normalised weights and the scatter together
// because each is a small memory-bound step whose launch costs as much as its work (Section 6,
// "Fused kernels"). There is no grid-wide barrier, so every workgroup redoes the cheap integer part
// for the whole batch in LDS (top-k of all T tokens, histogram, offsets, stable ranks: a few
// microseconds) and then copies its own share of the rows; workgroup 0 alone writes the
// routing results. Same outputs, bit for bit, as route_topk/route_count followed by
// dispatch_rank/dispatch_copy.
constexpr int kFusedMaxA = 2048;
constexpr int kFusedMaxT = 512;
constexpr int kFusedMaxLogits = 8192;  // T * E floats staged in LDS

// EM > 0 (E <= EM = 8 or 16): one lane owns a token and scans its E logits in registers, no
// cross-lane traffic; EM = 0: the L-lane group of topk_group. Both give the same picks and weights.
template <int L, int EM>
__global__ __launch_bounds__(256) void route_dispatch_small_kernel(
    const float* __restrict__ logits, const uint4* __restrict__ x, int T, int E, int k, int row_vecs,
    int32_t* __restrict__ topk_idx, float* __restrict__ topk_w, int32_t* __restrict__ counts,
    int32_t* __restrict__ offsets, uint4* __restrict__ xp, int32_t* __restrict__ pos, int32_t* __restrict__ src) {
  __shared__ float s_logits[kFusedMaxLogits];  // the whole logits matrix: one round of independent loads
  __shared__ int s_idx[kFusedMaxA];            // expert of assignment i = t * k + j
  __shared__ int s_src[kFusedMaxA];            // assignment that owns row r
  __shared__ int s_base[kMaxExperts];          // counts, then the next free row of each expert
  __shared__ int s_in_wave[4][kMaxExperts];    // assignments of e in each wavefront of the current chunk
  __shared__ int s_wave_total[4];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const bool writer = blockIdx.x == 0;
  const int A = T * k;

  // 1. top-k of every token (256 / L tokens per pass)
#pragma unroll 8
  for (int u = tid; u < T * E; u += 256) s_logits[u] = logits[u];
  __syncthreads();
  if constexpr (EM > 0) {
    for (int t = tid; t < T; t += 256) {
      float v[EM];
#pragma unroll
      for (int e = 0; e < EM; ++e) {
        float q = e < E ? s_logits[t * E + e] : -INFINITY;
        v[e] = q != q ? -INFINITY : q;  // NaN ranks as -inf
      }
      unsigned taken = 0;
      float row_max = 0.f, sum = 0.f, p[EM];
      int pick[EM];
#pragma unroll
      for (int j = 0; j < EM; ++j) {
        if (j < k) {
          float bv = -INFINITY;
          int bi = -1;
#pragma unroll
          for (int e = 0; e < EM; ++e)  // ascending scan, strict >: equal logits keep the lower index
            if (e < E && !((taken >> e) & 1u) && (bi < 0 || v[e] > bv)) {
              bv = v[e];
              bi = e;
            }
          taken |= 1u << bi;
          if (j == 0) row_max = bv;
          p[j] = expf(bv - row_max);
          sum += p[j];
          pick[j] = bi;
        }
      }
#pragma unroll
      for (int j = 0; j < EM; ++j) {
        if (j < k) {
          s_idx[t * k + j] = pick[j];
          if (writer) {
            topk_idx[(size_t)t * k + j] = pick[j];
            topk_w[(size_t)t * k + j] = p[j] / sum;
          }
        }
      }
    }
  } else {
    const int sl = tid % L;
    for (int t0 = 0; t0 < T; t0 += 256 / L) {
      const int t = t0 + tid / L;
      const bool valid = t < T;
      float v[kMaxPerLane];
#pragma unroll
      for (int i = 0; i < kMaxPerLane; ++i) {
        const int e = sl + i * L;
        float q = -INFINITY;
        if (valid && e < E) {
          q = s_logits[t * E + e];
          if (q != q) q = -INFINITY;  // NaN ranks as -inf
        }
        v[i] = q;
      }
      int my_idx;
      float my_w;
      topk_group<L>(v, sl, E, k, my_idx, my_w);
      if (valid && sl < k) {
        s_idx[t * k + sl] = my_idx;
        if (writer) {
          topk_idx[(size_t)t * k + sl] = my_idx;
          topk_w[(size_t)t * k + sl] = my_w;
        }
      }
    }
  }
  s_base[tid] = 0;
  __syncthreads();

  // 2. counts and offsets (thread e owns expert e; E <= 256)
  for (int i = tid; i < A; i += 256) atomicAdd(&s_base[s_idx[i]], 1);
  __syncthreads();
  const int cnt = s_base[tid];
  int incl = cnt;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int o = __shfl_up(incl, off);
    if (lane >= off) incl += o;
  }
  if (lane == 63) s_wave_total[w] = incl;
  __syncthreads();
  int first = incl - cnt;
  for (int ww = 0; ww < w; ++ww) first += s_wave_total[ww];
  if (writer && tid < E) {
    counts[tid] = cnt;
    offsets[tid] = first;
    if (tid == E - 1) offsets[E] = first + cnt;
  }
  s_base[tid] = first;

  // 3. stable ranks, 256 assignments at a time in ascending order
  const unsigned long long below = (1ull << lane) - 1ull;
  for (int c0 = 0; c0 < A; c0 += 256) {
#pragma unroll
    for (int i = 0; i < 4; ++i) s_in_wave[i][tid] = 0;
    __syncthreads();  // also orders s_base updates of the previous chunk before the reads below
    const int i = c0 + tid;
    const int e = i < A ? s_idx[i] : -1;
    int rank = 0;
    unsigned long long todo = __ballot(e >= 0);
    while (todo) {  // peel one expert value per round: the one held by the lowest lane still waiting
      const int leader = __ffsll((long long)todo) - 1;
      const int le = __shfl(e, leader);
      const unsigned long long same = __ballot(e == le);
      if (e == le) {
        rank = __popcll(same & below);
        if (lane == leader) s_in_wave[w][le] = __popcll(same);
      }
      todo &= ~same;
    }
    __syncthreads();
    if (e >= 0) {
      int r = s_base[e] + rank;
      for (int ww = 0; ww < w; ++ww) r += s_in_wave[ww][e];
      s_src[r] = i;
      if (writer) {
        pos[i] = r;
        src[r] = i;
      }
    }
    __syncthreads();
    s_base[tid] += s_in_wave[0][tid] + s_in_wave[1][tid] + s_in_wave[2][tid] + s_in_wave[3][tid];
  }
  __syncthreads();

  // 4. this workgroup's share of the rows: one wavefront per row, 16 bytes per lane per step
  for (int r = blockIdx.x * 4 + w; r < A; r += gridDim.x * 4) {
    const uint4* in = x + (size_t)(s_src[r] / k) * row_vecs;
    uint4* out = xp + (size_t)r * row_vecs;
    int c = lane;
    for (; c + 192 < row_vecs; c += 256) {  // four independent loads in flight per lane
      const uint4 q0 = in[c], q1 = in[c + 64], q2 = in[c + 128], q3 = in[c + 192];
      out[c] = q0;
      out[c + 64] = q1;
      out[c + 128] = q2;
      out[c + 192] = q3;
    }
    for (; c < row_vecs; c += 64) out[c] = in[c];
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


bool launch_route_dispatch_fused(const float* logits, const void* x, int T, int E, int k, int row_bytes,
                                 int32_t* topk_idx, float* topk_w, int32_t* counts, int32_t* offsets, void* xp,
                                 int32_t* pos, int32_t* src, hipStream_t stream) {
  const int A = T * k;
  if (T < 1 || T > kFusedMaxT || A > kFusedMaxA || T * E > kFusedMaxLogits) return false;
  const int L = E <= 8 ? 8 : E <= 16 ? 16 : E <= 32 ? 32 : 64;
  const dim3 grid((A + 3) / 4 < 256 ? (A + 3) / 4 : 256), block(256);
  const uint4* xv = static_cast<const uint4*>(x);
  uint4* xpv = static_cast<uint4*>(xp);
  const int rv = row_bytes / 16;
  switch (L) {
    case 8: hipLaunchKernelGGL((route_dispatch_small_kernel<8, 8>), grid, block, 0, stream, logits, xv, T, E, k, rv, topk_idx, topk_w, counts, offsets, xpv, pos, src); break;
    case 16: hipLaunchKernelGGL((route_dispatch_small_kernel<16, 16>), grid, block, 0, stream, logits, xv, T, E, k, rv, topk_idx, topk_w, counts, offsets, xpv, pos, src); break;
    case 32: hipLaunchKernelGGL((route_dispatch_small_kernel<32, 0>), grid, block, 0, stream, logits, xv, T, E, k, rv, topk_idx, topk_w, counts, offsets, xpv, pos, src); break;
    default: hipLaunchKernelGGL((route_dispatch_small_kernel<64, 0>), grid, block, 0, stream, logits, xv, T, E, k, rv, topk_idx, topk_w, counts, offsets, xpv, pos, src); break;
  }
  return true;
}

template <int TT, int EPT, int L>
static void launch_gate_topk(bool bf16, hipStream_t stream, const void* x, const float* wr, int T, int d, int E, int k,
                             float* logits, int32_t* topk_idx, float* topk_w) {
  const dim3 grid((T + TT - 1) / TT);
  if (bf16)
    hipLaunchKernelGGL((gate_topk_kernel<TT, EPT, L, true>), grid, dim3(256), 0, stream, x, wr, T, d, E, k, logits,
                       topk_idx, topk_w);
  else
    hipLaunchKernelGGL((gate_topk_kernel<TT, EPT, L, false>), grid, dim3(256), 0, stream, x, wr, T, d, E, k, logits,
                       topk_idx, topk_w);
}

hipError_t launch_gate_route(const void* x, const float* w_router, int T, int d, int E, int k, int dtype, float* logits,
                             int32_t* topk_idx, float* topk_w, int32_t* counts, int32_t* offsets, hipStream_t stream) {
  if (T > 0) {
    const bool bf16 = dtype == MOE_BF16;
    const dim3 wgrid((T + 3) / 4);
    if (E <= 8) {  // one wavefront per token
      if (bf16) hipLaunchKernelGGL((gate_topk_wave_kernel<8, true>), wgrid, dim3(256), 0, stream, x, w_router, T, d, E, k, logits, topk_idx, topk_w);
      else hipLaunchKernelGGL((gate_topk_wave_kernel<8, false>), wgrid, dim3(256), 0, stream, x, w_router, T, d, E, k, logits, topk_idx, topk_w);
    } else if (E <= 16) {
      if (bf16) hipLaunchKernelGGL((gate_topk_wave_kernel<16, true>), wgrid, dim3(256), 0, stream, x, w_router, T, d, E, k, logits, topk_idx, topk_w);
      else hipLaunchKernelGGL((gate_topk_wave_kernel<16, false>), wgrid, dim3(256), 0, stream, x, w_router, T, d, E, k, logits, topk_idx, topk_w);
    }
    // more experts: 16-token workgroups (16 expert groups of EPT) while E allows it
    else if (E <= 32) launch_gate_topk<16, 2, 32>(bf16, stream, x, w_router, T, d, E, k, logits, topk_idx, topk_w);
    else if (E <= 64) launch_gate_topk<16, 4, 64>(bf16, stream, x, w_router, T, d, E, k, logits, topk_idx, topk_w);
    else if (E <= 128) launch_gate_topk<32, 16, 64>(bf16, stream, x, w_router, T, d, E, k, logits, topk_idx, topk_w);
    else launch_gate_topk<32, 32, 64>(bf16, stream, x, w_router, T, d, E, k, logits, topk_idx, topk_w);
  }
  hipLaunchKernelGGL(route_count_kernel, dim3(1), dim3(1024), 0, stream, topk_idx, T * k, E, counts, offsets);
  return hipGetLastError();
}

}  // namespace moe
