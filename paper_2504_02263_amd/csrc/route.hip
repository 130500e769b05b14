// Routing kernels: top-k selection with softmax over the picks, then per-expert counts and
// offsets (paper Section 2.2 for the routing rule; Section 6 "Fused kernels" for the list of
// by-products: token counts per expert and normalised token weights).
#include <limits.h>
#include <type_traits>
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

typedef __bf16 gate_bf16x8 __attribute__((ext_vector_type(8)));
typedef float gate_floatx16 __attribute__((ext_vector_type(16)));
typedef unsigned int gate_u32x4 __attribute__((ext_vector_type(4)));

template <int I, int N, typename F>
__device__ __forceinline__ void gate_static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    gate_static_for<I + 1, N>(f);
  }
}

// Common end of the matrix-core gating kernels: add the four wavefronts' partial logits in the fixed
// order 0, 1, 2, 3 through LDS, write the logits if asked to, and run the top-k on the 32 x E tile.
template <int NT>
__device__ __forceinline__ void gate_finish(const gate_floatx16 (&acc)[NT], float (*lg)[33], int t0, int T, int E,
                                            int k, int L, float* __restrict__ logits,
                                            int32_t* __restrict__ topk_idx, float* __restrict__ topk_w) {
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int frow = lane & 31, fg = lane >> 5;
  // acc[i][r]: expert 32 i + 8 (r / 4) + 4 (lane / 32) + r % 4, token lane % 32
  for (int turn = 0; turn < 4; ++turn) {
    if (w == turn) {
#pragma unroll
      for (int i = 0; i < NT; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float* p = &lg[32 * i + 8 * (r >> 2) + 4 * fg + (r & 3)][frow];
          *p = turn == 0 ? acc[i][r] : *p + acc[i][r];
        }
    }
    __syncthreads();
  }
  if (logits) {
    for (int u = tid; u < 32 * E; u += 256) {
      const int r = u / E, e = u % E;
      if (t0 + r < T) logits[(size_t)(t0 + r) * E + e] = lg[e][r];
    }
  }
  auto topk_rows = [&](auto L_) {
    constexpr int LL = decltype(L_)::value;
    const int sl = tid % LL;
    for (int base = 0; base < 32; base += 256 / LL) {
      const int r = base + tid / LL;
      const bool valid = t0 + r < T;
      float v[kMaxPerLane];
#pragma unroll
      for (int i = 0; i < kMaxPerLane; ++i) {
        const int e = sl + i * LL;
        float q = -INFINITY;
        if (valid && e < E) {
          q = lg[e][r];
          if (q != q) q = -INFINITY;
        }
        v[i] = q;
      }
      int my_idx;
      float my_w;
      topk_group<LL>(v, sl, E, k, my_idx, my_w);
      if (valid && sl < k) {
        topk_idx[(size_t)(t0 + r) * k + sl] = my_idx;
        topk_w[(size_t)(t0 + r) * k + sl] = my_w;
      }
    }
  };
  if (L == 8) topk_rows(std::integral_constant<int, 8>{});
  else if (L == 16) topk_rows(std::integral_constant<int, 16>{});
  else if (L == 32) topk_rows(std::integral_constant<int, 32>{});
  else topk_rows(std::integral_constant<int, 64>{});
}

// Matrix-core gating for up to 64 experts (NT <= 2) without workgroup barriers in the main loop:
// each of the 4 wavefronts owns a quarter of the hidden dimension and stages its own 32-column
// chunks (token tile, and the w_router tile split into hi + lo bf16 terms as described below) in a
// private LDS region, reads them back in operand order and issues the MFMAs; LDS operations of one
// wavefront execute in order, so nothing but the data dependences has to be waited for, and loads,
// conversion and MFMAs of neighbouring chunks overlap. Rows of a chunk are 64 bytes (4 units of
// 16 B); unit index XOR ((row >> 2) & 3) keeps both the row-major stores and the operand-order
// reads free of bank conflicts.
template <int NT, int D>
__global__ __launch_bounds__(256) void gate_topk_mfma_wave_kernel(const uint16_t* __restrict__ x,
                                                                  const float* __restrict__ wr, int T, int d, int E,
                                                                  int k, int L, float* __restrict__ logits,
                                                                  int32_t* __restrict__ topk_idx,
                                                                  float* __restrict__ topk_w) {
  __shared__ gate_u32x4 xs[4][32 * 4];
  __shared__ gate_u32x4 whi[4][NT * 32 * 4];
  __shared__ gate_u32x4 wlo[4][NT * 32 * 4];
  __shared__ float lg[NT * 32][33];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int frow = lane & 31, fg = lane >> 5;
  const int t0 = blockIdx.x * 32;
  const int kq = d >> 2;  // columns of this wavefront: [w kq, (w + 1) kq); a multiple of 32
  // staging role: units lane and lane + 64 of a 32-row x 4-unit tile: row = u / 4, unit = u % 4
  int sdst[2];
  const uint16_t* xsrc[2];
  const float* wsrc[NT][2];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int u = lane + 64 * h, row = u >> 2, unit = u & 3;
    sdst[h] = row * 4 + (unit ^ ((row >> 2) & 3));
    xsrc[h] = x + (size_t)min(t0 + row, T - 1) * d + w * kq + 8 * unit;
#pragma unroll
    for (int q = 0; q < NT; ++q) wsrc[q][h] = wr + (size_t)min(32 * q + row, E - 1) * d + w * kq + 8 * unit;
  }
  int frd[2];  // this lane's fragment piece of k-step s of a chunk
#pragma unroll
  for (int s2 = 0; s2 < 2; ++s2) frd[s2] = frow * 4 + ((2 * s2 + fg) ^ ((frow >> 2) & 3));

  gate_floatx16 acc[NT];
#pragma unroll
  for (int i = 0; i < NT; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;

  gate_u32x4 xreg[D][2];
  float4 wreg[D][NT][2][2];
  auto fetch = [&](auto j_, int c) {
    constexpr int j = decltype(j_)::value;
    c = min(c, kq - 32);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      xreg[j][h] = *reinterpret_cast<const gate_u32x4*>(xsrc[h] + c);
#pragma unroll
      for (int q = 0; q < NT; ++q) {
        wreg[j][q][h][0] = *reinterpret_cast<const float4*>(wsrc[q][h] + c);
        wreg[j][q][h][1] = *reinterpret_cast<const float4*>(wsrc[q][h] + c + 4);
      }
    }
  };
  auto step = [&](auto j_, int c) {
    constexpr int j = decltype(j_)::value;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      xs[w][sdst[h]] = xreg[j][h];
#pragma unroll
      for (int q = 0; q < NT; ++q) {
        const float4 a0 = wreg[j][q][h][0], a1 = wreg[j][q][h][1];
        const float a[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
        gate_bf16x8 hi, lo;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          hi[i] = (__bf16)a[i];
          lo[i] = (__bf16)(a[i] - (float)hi[i]);
        }
        whi[w][q * 128 + sdst[h]] = __builtin_bit_cast(gate_u32x4, hi);
        wlo[w][q * 128 + sdst[h]] = __builtin_bit_cast(gate_u32x4, lo);
      }
    }
    fetch(j_, c + 32 * D);  // refill this ring slot (past the end: a harmless refetch of the last chunk)
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
      const gate_bf16x8 b = __builtin_bit_cast(gate_bf16x8, xs[w][frd[s2]]);
#pragma unroll
      for (int i = 0; i < NT; ++i)
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(gate_bf16x8, whi[w][i * 128 + frd[s2]]), b, acc[i], 0, 0, 0);
#pragma unroll
      for (int i = 0; i < NT; ++i)
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(gate_bf16x8, wlo[w][i * 128 + frd[s2]]), b, acc[i], 0, 0, 0);
    }
  };
  gate_static_for<0, D>([&](auto j_) { fetch(j_, 32 * decltype(j_)::value); });
  // kq / 32 is a multiple of D (the launcher picks D so), and no load sits under a branch: the loop
  // body is one basic block and every wait counts exactly the loads issued after the one it needs
  for (int c0 = 0; c0 < kq; c0 += 32 * D)
    gate_static_for<0, D>([&](auto j_) { step(j_, c0 + 32 * decltype(j_)::value); });
  __syncthreads();
  gate_finish<NT>(acc, lg, t0, T, E, k, L, logits, topk_idx, topk_w);
}

// Gating GEMM on the matrix cores, for more than 16 experts and bf16 activations (same fusion as
// above: the logits go straight into the top-k, Section 6 "Fused kernels"). A workgroup owns 32
// tokens and walks the hidden dimension in chunks of 64 columns. Per chunk its 256 threads load
// the token tile (32 x 64 bf16) and the w_router tile (32 NT x 64 float32) with row-contiguous
// 16-byte loads, D chunks ahead in a register ring (a chunk is only four MFMAs per expert tile, so
// one chunk of lead would leave the load latency exposed); the float32 gating weights are split into two bf16
// terms, w = hi + lo with |w - hi - lo| <= 2^-18 |w|, and all three tiles go to LDS in the
// swizzled [row][8 x 16 B] layout of the FFN kernels. Wavefront s then takes MFMA k-step s of the
// chunk (v_mfma_f32_32x32x16_bf16: w_router tile = A operand, token tile = B operand) and issues
// one MFMA per term and expert tile, so the logits keep float32-level accuracy (the activations
// are bf16 already). The four partial sums are added in wavefront order 0, 1, 2, 3 through LDS (a
// fixed order: the logits, and with them the routing, are reproducible), then the top-k runs on
// the 32 x E logits in LDS.
template <int NT, int D>  // NT = 32-expert tiles (E <= 32 NT); D = ring depth; L = lanes per token in the top-k
__global__ __launch_bounds__(256) void gate_topk_mfma_kernel(const uint16_t* __restrict__ x,
                                                             const float* __restrict__ wr, int T, int d, int E, int k,
                                                             int L, float* __restrict__ logits,
                                                             int32_t* __restrict__ topk_idx,
                                                             float* __restrict__ topk_w) {
  __shared__ gate_u32x4 xs[32 * 8];
  __shared__ gate_u32x4 whi[NT * 32 * 8];
  __shared__ gate_u32x4 wlo[NT * 32 * 8];
  __shared__ float lg[NT * 32][33];  // [expert][token], padded
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int frow = lane & 31, fg = lane >> 5;
  const int t0 = blockIdx.x * 32;
  // staging role: 16-byte unit (tid % 8) of row tid / 8 (+ 32 q for the w_router tile)
  const int srow = tid >> 3, sunit = tid & 7;
  const int sdst = srow * 8 + (sunit ^ ((srow >> 1) & 7));  // (row + 32 q) keeps the same swizzle term
  const uint16_t* xsrc = x + (size_t)min(t0 + srow, T - 1) * d + 8 * sunit;
  const float* wsrc[NT];
#pragma unroll
  for (int q = 0; q < NT; ++q) wsrc[q] = wr + (size_t)min(32 * q + srow, E - 1) * d + 8 * sunit;
  // MFMA role: fragment piece of k-step w
  const int frd = frow * 8 + ((2 * w + fg) ^ ((frow >> 1) & 7));

  gate_floatx16 acc[NT];
#pragma unroll
  for (int i = 0; i < NT; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;

  gate_u32x4 xreg[D];
  float4 wreg[D][NT][2];
#pragma unroll
  for (int j = 0; j < D; ++j) {
    const int c = min(64 * j, d - 64);
    xreg[j] = *reinterpret_cast<const gate_u32x4*>(xsrc + c);
#pragma unroll
    for (int q = 0; q < NT; ++q) {
      wreg[j][q][0] = *reinterpret_cast<const float4*>(wsrc[q] + c);
      wreg[j][q][1] = *reinterpret_cast<const float4*>(wsrc[q] + c + 4);
    }
  }
  for (int c0 = 0; c0 < d; c0 += 64 * D) {
#pragma unroll
    for (int j = 0; j < D; ++j) {
      const int c = c0 + 64 * j;
      {  // d / 64 is a multiple of D (the launcher picks D so): no load sits under a branch
        xs[sdst] = xreg[j];
#pragma unroll
        for (int q = 0; q < NT; ++q) {
          const float a[8] = {wreg[j][q][0].x, wreg[j][q][0].y, wreg[j][q][0].z, wreg[j][q][0].w,
                              wreg[j][q][1].x, wreg[j][q][1].y, wreg[j][q][1].z, wreg[j][q][1].w};
          gate_bf16x8 hi, lo;
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            hi[i] = (__bf16)a[i];
            lo[i] = (__bf16)(a[i] - (float)hi[i]);
          }
          whi[q * 256 + sdst] = __builtin_bit_cast(gate_u32x4, hi);
          wlo[q * 256 + sdst] = __builtin_bit_cast(gate_u32x4, lo);
        }
        {  // refill this ring slot with chunk c + 64 D (past the end: a harmless refetch of the last chunk)
          const int cn = min(c + 64 * D, d - 64);
          xreg[j] = *reinterpret_cast<const gate_u32x4*>(xsrc + cn);
#pragma unroll
          for (int q = 0; q < NT; ++q) {
            wreg[j][q][0] = *reinterpret_cast<const float4*>(wsrc[q] + cn);
            wreg[j][q][1] = *reinterpret_cast<const float4*>(wsrc[q] + cn + 4);
          }
        }
        __syncthreads();
        const gate_bf16x8 b = __builtin_bit_cast(gate_bf16x8, xs[frd]);
#pragma unroll
        for (int i = 0; i < NT; ++i)
          acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(gate_bf16x8, whi[i * 256 + frd]), b, acc[i], 0, 0, 0);
#pragma unroll
        for (int i = 0; i < NT; ++i)
          acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(gate_bf16x8, wlo[i * 256 + frd]), b, acc[i], 0, 0, 0);
        __syncthreads();
      }
    }
  }

  gate_finish<NT>(acc, lg, t0, T, E, k, L, logits, topk_idx, topk_w);
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
// FROM_IDX: the picks are given (topk_idx is an input, written by the fused gating kernel just before)
// and step 1 only stages them; logits and topk_w are not touched.
template <int L, int EM, bool FROM_IDX = false>
__global__ __launch_bounds__(256) void route_dispatch_small_kernel(
    const float* __restrict__ logits, const uint4* __restrict__ x, int T, int E, int k, int row_vecs,
    int32_t* __restrict__ topk_idx, float* __restrict__ topk_w, int32_t* __restrict__ counts,
    int32_t* __restrict__ offsets, uint4* __restrict__ xp, int32_t* __restrict__ pos, int32_t* __restrict__ src) {
  __shared__ float s_logits[FROM_IDX ? 1 : kFusedMaxLogits];  // the whole logits matrix: one round of independent loads
  __shared__ int s_idx[kFusedMaxA];            // expert of assignment i = t * k + j
  __shared__ int s_src[kFusedMaxA];            // assignment that owns row r
  __shared__ int s_base[kMaxExperts];          // counts, then the next free row of each expert
  __shared__ int s_in_wave[4][kMaxExperts];    // assignments of e in each wavefront of the current chunk
  __shared__ int s_wave_total[4];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const bool writer = blockIdx.x == 0;
  const int A = T * k;

  // 1. top-k of every token (256 / L tokens per pass)
  if constexpr (FROM_IDX) {
#pragma unroll 4
    for (int i = tid; i < A; i += 256) {
      const int e = topk_idx[i];
      s_idx[i] = (unsigned)e < (unsigned)E ? e : 0;  // the gating kernel only writes experts in range
    }
  } else {
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

// Lanes that share one token in topk_group: the smallest group with at most kMaxPerLane experts per
// lane and one lane per pick (fewer lanes per token = more tokens per wavefront pass).
static int topk_lanes(int E, int k) {
  int L = 8;
  while (L < 64 && (E > kMaxPerLane * L || k > L)) L *= 2;
  return L;
}

hipError_t launch_route(const float* logits, int T, int E, int k, int32_t* topk_idx, float* topk_w, int32_t* counts,
                        int32_t* offsets, hipStream_t stream) {
  if (T > 0) {
    const int L = topk_lanes(E, k);
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
  const int L = E <= 8 ? -8 : E <= 16 ? -16 : topk_lanes(E, k);  // negative: the lane-per-token variant
  const dim3 grid((A + 3) / 4 < 256 ? (A + 3) / 4 : 256), block(256);
  const uint4* xv = static_cast<const uint4*>(x);
  uint4* xpv = static_cast<uint4*>(xp);
  const int rv = row_bytes / 16;
  switch (L) {
    case -8: hipLaunchKernelGGL((route_dispatch_small_kernel<8, 8>), grid, block, 0, stream, logits, xv, T, E, k, rv, topk_idx, topk_w, counts, offsets, xpv, pos, src); break;
    case -16: hipLaunchKernelGGL((route_dispatch_small_kernel<16, 16>), grid, block, 0, stream, logits, xv, T, E, k, rv, topk_idx, topk_w, counts, offsets, xpv, pos, src); break;
    case 8: hipLaunchKernelGGL((route_dispatch_small_kernel<8, 0>), grid, block, 0, stream, logits, xv, T, E, k, rv, topk_idx, topk_w, counts, offsets, xpv, pos, src); break;
    case 16: hipLaunchKernelGGL((route_dispatch_small_kernel<16, 0>), grid, block, 0, stream, logits, xv, T, E, k, rv, topk_idx, topk_w, counts, offsets, xpv, pos, src); break;
    case 32: hipLaunchKernelGGL((route_dispatch_small_kernel<32, 0>), grid, block, 0, stream, logits, xv, T, E, k, rv, topk_idx, topk_w, counts, offsets, xpv, pos, src); break;
    default: hipLaunchKernelGGL((route_dispatch_small_kernel<64, 0>), grid, block, 0, stream, logits, xv, T, E, k, rv, topk_idx, topk_w, counts, offsets, xpv, pos, src); break;
  }
  return true;
}

// Counts, offsets and the dispatch pack from given picks in one launch (decode-sized batches); returns
// false (nothing launched) when the batch is too large for it.
bool launch_dispatch_from_picks_fused(const int32_t* topk_idx, const void* x, int T, int E, int k, int row_bytes,
                                      int32_t* counts, int32_t* offsets, void* xp, int32_t* pos, int32_t* src,
                                      hipStream_t stream) {
  const int A = T * k;
  if (T < 1 || T > kFusedMaxT || A > kFusedMaxA) return false;
  const dim3 grid((A + 3) / 4 < 256 ? (A + 3) / 4 : 256), block(256);
  hipLaunchKernelGGL((route_dispatch_small_kernel<8, 0, true>), grid, block, 0, stream, nullptr,
                     static_cast<const uint4*>(x), T, E, k, row_bytes / 16, const_cast<int32_t*>(topk_idx), nullptr,
                     counts, offsets, static_cast<uint4*>(xp), pos, src);
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
  launch_gate_topk_only(x, w_router, T, d, E, k, dtype, logits, topk_idx, topk_w, stream);
  hipLaunchKernelGGL(route_count_kernel, dim3(1), dim3(1024), 0, stream, topk_idx, T * k, E, counts, offsets);
  return hipGetLastError();
}

void launch_count(const int32_t* topk_idx, int T, int E, int k, int32_t* counts, int32_t* offsets, hipStream_t stream) {
  hipLaunchKernelGGL(route_count_kernel, dim3(1), dim3(1024), 0, stream, topk_idx, T * k, E, counts, offsets);
}

void launch_gate_topk_only(const void* x, const float* w_router, int T, int d, int E, int k, int dtype, float* logits,
                           int32_t* topk_idx, float* topk_w, hipStream_t stream) {
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
    // more experts, bf16 activations: the gating GEMM runs on the matrix cores
    else if (bf16) {
      const dim3 mgrid((T + 31) / 32);
      const uint16_t* xb = static_cast<const uint16_t*>(x);
      const int L = topk_lanes(E, k);
      // ring depth: must divide the chunk count (d / 128 per wavefront, d / 64 per workgroup)
#define MOE_GATE_LAUNCH(KERNEL) hipLaunchKernelGGL(KERNEL, mgrid, dim3(256), 0, stream, xb, w_router, T, d, E, k, L, logits, topk_idx, topk_w)
      if (E <= 64) {
        const int D = d % 512 == 0 ? 4 : d % 256 == 0 ? 2 : 1;
        if (E <= 32) {
          if (D == 4) MOE_GATE_LAUNCH((gate_topk_mfma_wave_kernel<1, 4>));
          else if (D == 2) MOE_GATE_LAUNCH((gate_topk_mfma_wave_kernel<1, 2>));
          else MOE_GATE_LAUNCH((gate_topk_mfma_wave_kernel<1, 1>));
        } else {
          if (D == 4) MOE_GATE_LAUNCH((gate_topk_mfma_wave_kernel<2, 4>));
          else if (D == 2) MOE_GATE_LAUNCH((gate_topk_mfma_wave_kernel<2, 2>));
          else MOE_GATE_LAUNCH((gate_topk_mfma_wave_kernel<2, 1>));
        }
      } else if (E <= 128) {
        if (d % 256 == 0) MOE_GATE_LAUNCH((gate_topk_mfma_kernel<4, 4>));
        else MOE_GATE_LAUNCH((gate_topk_mfma_kernel<4, 2>));
      } else {
        MOE_GATE_LAUNCH((gate_topk_mfma_kernel<8, 2>));
      }
#undef MOE_GATE_LAUNCH
    }
    // more experts, float32 activations: 16-token workgroups (16 expert groups of EPT) while E allows it
    else if (E <= 32) launch_gate_topk<16, 2, 32>(bf16, stream, x, w_router, T, d, E, k, logits, topk_idx, topk_w);
    else if (E <= 64) launch_gate_topk<16, 4, 64>(bf16, stream, x, w_router, T, d, E, k, logits, topk_idx, topk_w);
    else if (E <= 128) launch_gate_topk<32, 16, 64>(bf16, stream, x, w_router, T, d, E, k, logits, topk_idx, topk_w);
    else launch_gate_topk<32, 32, 64>(bf16, stream, x, w_router, T, d, E, k, logits, topk_idx, topk_w);
  }
}

}  // namespace moe
