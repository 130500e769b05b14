// Expert FFN as a grouped SwiGLU GEMM (paper Section 4.2, Table 3: "FFN Input" (b_e, h) x (h, h')
// and "FFN Output" (b_e, h') x (h', h); tensor-parallel degree 1), plus the one-time weight pre-pack.
//
// bf16 path. Both GEMMs are C[m, n] = sum_k X[m, k] * W[n, k] with K contiguous in X and W. The
// weights are pre-packed into matrix-core operand order: a "fragment" is the 32 (n) x 16 (k)
// operand of one v_mfma_f32_32x32x16_bf16, stored as 64 lanes x 16 bytes = 1 KiB where lane
// l = (n % 32) + 32 * g holds k = 16 * ks + 8 * g .. + 7. A wavefront owns one 32-row n-tile and
// streams its fragments from HBM straight into registers, 1 KiB fully contiguous per load, each
// weight byte read once per m-tile. Tokens (the other operand) are staged through LDS and shared
// by the four wavefronts of the workgroup. Per-expert row ranges come from `offsets` on the device.
#include <math.h>
#include <stdlib.h>
#include <type_traits>
#include "moe_internal.h"

namespace moe {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));  // one 16-byte unit

// Compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), so that
// register-array indices derived from the loop variable are constants.
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

struct TileLoc {
  int expert;   // -1: this workgroup has no tile
  int row0;     // first row of the m-tile
  int row_end;  // end of the expert's segment
};

// Map m-tile slot -> (expert, first row). Expert e owns ceil(c_e / BM) consecutive slots in
// expert order. All 256 threads of the workgroup must call this (thread i handles expert i).
__device__ __forceinline__ TileLoc locate_tile(const int32_t* __restrict__ offsets, int E, int BM, int slot) {
  __shared__ int s_wave_total[4];
  __shared__ int s_loc[3];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  int lo = 0, hi = 0;
  if (tid < E) {
    lo = offsets[tid];
    hi = offsets[tid + 1];
  }
  const int nt = (hi - lo + BM - 1) / BM;
  int incl = nt;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int o = __shfl_up(incl, off);
    if (lane >= off) incl += o;
  }
  if (lane == 63) s_wave_total[w] = incl;
  if (tid == 0) s_loc[0] = -1;
  __syncthreads();
  int excl = incl - nt;
  for (int ww = 0; ww < w; ++ww) excl += s_wave_total[ww];
  if (nt > 0 && slot >= excl && slot < excl + nt) {
    s_loc[0] = tid;
    s_loc[1] = lo + (slot - excl) * BM;
    s_loc[2] = hi;
  }
  __syncthreads();
  TileLoc t;
  t.expert = s_loc[0];
  t.row0 = s_loc[1];
  t.row_end = s_loc[2];
  return t;
}

__device__ __forceinline__ float silu(float g) { return g / (1.f + __expf(-g)); }

// ------------------------------------------------------------------------------------------
// bf16 weight pre-pack: canonical [E, N, K] (K contiguous) -> fragments
//   packed[(((e * NT + nt) * KS + ks) * NW + sel) * 64 + lane] (16-byte units),
//   NT = N / 32, KS = K / 16, NW = matrices interleaved per k-step (2 for gate|up, 1 for down).
__global__ __launch_bounds__(256) void pack_bf16_kernel(const uint4* __restrict__ w0, const uint4* __restrict__ w1,
                                                        int E, int N, int K, int NW, uint4* __restrict__ packed) {
  const size_t total = (size_t)E * N * (K / 8) * NW;
  const int NT = N / 32, KS = K / 16;
  for (size_t u = (size_t)blockIdx.x * 256 + threadIdx.x; u < total; u += (size_t)gridDim.x * 256) {
    size_t q = u;
    const int lane = q % 64; q /= 64;
    const int sel = q % NW;  q /= NW;
    const int ks = q % KS;   q /= KS;
    const int nt = q % NT;   q /= NT;
    const int e = (int)q;
    const int n = nt * 32 + (lane & 31);
    const int kv = ks * 2 + (lane >> 5);  // 16-byte unit along K
    const uint4* w = sel == 0 ? w0 : w1;
    packed[u] = w[((size_t)e * N + n) * (K / 8) + kv];
  }
}

// ------------------------------------------------------------------------------------------
// bf16 grouped GEMM on the matrix cores.
//   NW = 2: C = silu(X Wg^T) .* (X Wu^T)  (gate and up fragments interleaved per k-step)
//   NW = 1: C = X W^T
// Workgroup = 4 wavefronts; wavefront w owns n-tile nt = 4 * blockIdx.x + w (32 output columns)
// and all BM = 32 * MT rows of the m-tile. K is walked in chunks of 64 (4 MFMA k-steps).
//
// Pipeline. Global loads return in order, so one ring of NST chunks carries both operands:
// weights for chunk c + NST and the workgroup's share of the token slab for chunk c + NST + 1 are
// issued in iteration c, into registers. The token share for chunk c + 1 is written to LDS at
// the end of iteration c (double-buffered slab, one barrier per chunk). At every wait about
// NST - 1 chunks stay in flight.
//
// LDS slab: [BM rows][8 units of 16 B], unit index XOR (row % 8): the row-major writes and the
// operand-order reads (32 rows, same logical unit) are both bank-conflict free.
template <int MT, int NW, int NST>
__global__ __launch_bounds__(256) void ffn_bf16_kernel(const u32x4* __restrict__ X, const int32_t* __restrict__ offsets,
                                                       const u32x4* __restrict__ Wp, __bf16* __restrict__ C, int E,
                                                       int N, int K) {
  static_assert(NST % 2 == 0, "chunk parity must equal ring-slot parity");
  constexpr int BM = 32 * MT;
  __shared__ u32x4 slab[2][BM * 8];

  const TileLoc loc = locate_tile(offsets, E, BM, blockIdx.y);
  if (loc.expert < 0) return;

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int NT = N / 32, KS = K / 16, NC = K / 64, KV = K / 8;
  const int nt = blockIdx.x * 4 + w;
  const bool has_n = nt < NT;
  const int rows = min(loc.row_end - loc.row0, BM);

  // weights of this wavefront: chunk c, k-step s, matrix sel -> wbase[(c * 4 + s) * NW * 64 + sel * 64]
  const u32x4* wbase = Wp + ((size_t)loc.expert * NT + (has_n ? nt : 0)) * KS * NW * 64 + lane;
  // token slab share: per pass p thread loads row p * 32 + tid / 8, unit tid % 8
  const int trow = tid >> 3, tunit = tid & 7;
  const int swz_w = trow * 8 + (tunit ^ (trow & 7));  // + p * 256 (rows p*32.. keep row % 8)

  u32x4 wreg[NST][4 * NW];
  u32x4 treg[NST][MT];

  // Loads never branch: chunk indices past the end are clamped to the last chunk and rows past
  // the segment to its last row (what they fetch is never used), so the loop body is straight-line
  // code and the load counter waits stay exact.
  auto load_w = [&](auto st_, int c) {
    constexpr int st = decltype(st_)::value;
    c = min(c, NC - 1);
#pragma unroll
    for (int i = 0; i < 4 * NW; ++i)  // streamed once: non-temporal, so the weights do not evict the tokens from L2
      wreg[st][i] = __builtin_nontemporal_load(&wbase[(size_t)(c * 4 * NW + i) * 64]);
  };
  const u32x4* xrow[MT];  // this thread's source row in each pass
#pragma unroll
  for (int p = 0; p < MT; ++p) xrow[p] = X + (size_t)(loc.row0 + min(p * 32 + trow, rows - 1)) * KV + tunit;
  auto load_t = [&](auto st_, int c) {
    constexpr int st = decltype(st_)::value;
    c = min(c, NC - 1);
#pragma unroll
    for (int p = 0; p < MT; ++p) treg[st][p] = xrow[p][c * 8];
  };
  auto store_t = [&](auto st_, auto buf_) {
    constexpr int st = decltype(st_)::value;
    constexpr int buf = decltype(buf_)::value;
#pragma unroll
    for (int p = 0; p < MT; ++p) slab[buf][p * 256 + swz_w] = treg[st][p];
  };

  floatx16 acc[NW][MT];
#pragma unroll
  for (int s = 0; s < NW; ++s)
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[s][m][r] = 0.f;

  const int frow = lane & 31, fg = lane >> 5;
  // One pipeline stage for chunk c held in ring slot st (= c % NST); chunk parity == st parity.
  auto stage = [&](auto st_, int c) {
    constexpr int st = decltype(st_)::value;
    constexpr int buf = st & 1;
    constexpr int nxt = (st + 1) % NST;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
#pragma unroll
      for (int m = 0; m < MT; ++m) {
        if (m * 32 < rows) {  // uniform over the workgroup: 32-row groups past the segment cost nothing
          const int row = m * 32 + frow;
          const bf16x8 b = __builtin_bit_cast(bf16x8, slab[buf][row * 8 + ((2 * s + fg) ^ (row & 7))]);
#pragma unroll
          for (int sel = 0; sel < NW; ++sel)
            acc[sel][m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                __builtin_bit_cast(bf16x8, wreg[st][s * NW + sel]), b, acc[sel][m], 0, 0, 0);
        }
      }
    }
    load_w(st_, c + NST);
    store_t(std::integral_constant<int, nxt>{}, std::integral_constant<int, buf ^ 1>{});
    load_t(std::integral_constant<int, nxt>{}, c + 1 + NST);
    __syncthreads();
  };

  // prologue: chunk 0 tokens straight to LDS; then the steady-state issue order W[c], tokens[c + 1]
  load_t(std::integral_constant<int, 0>{}, 0);
  store_t(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
  static_for<0, NST>([&](auto st_) {
    constexpr int st = decltype(st_)::value;
    load_w(st_, st);
    load_t(std::integral_constant<int, (st + 1) % NST>{}, st + 1);
  });
  __syncthreads();

  // NC is a multiple of NST (the launcher picks NST so), so there is no remainder loop
  for (int c0 = 0; c0 < NC; c0 += NST) static_for<0, NST>([&](auto st_) { stage(st_, c0 + decltype(st_)::value); });

  if (!has_n) return;
  // acc[..][m][r] holds C[row = m * 32 + lane % 32][col = nt * 32 + 8 * (r / 4) + 4 * (lane / 32) + r % 4]
#pragma unroll
  for (int m = 0; m < MT; ++m) {
    const int row = m * 32 + frow;
    if (row < rows) {
      __bf16* crow = C + (size_t)(loc.row0 + row) * N + nt * 32 + 4 * fg;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        bf16x4 o;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float v = acc[0][m][q * 4 + i];
          if (NW == 2) v = silu(v) * acc[NW - 1][m][q * 4 + i];
          o[i] = (__bf16)v;
        }
        *reinterpret_cast<bf16x4*>(crow + 8 * q) = o;
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// f32 grouped GEMM, plain FMA: 32 (m) x 64 (n) tile per workgroup, K in chunks of 32 through LDS.
// Thread (tx = tid % 64, ty = tid / 64) computes rows ty * 8 .. + 7 of column tx.
template <int NW>
__global__ __launch_bounds__(256) void ffn_f32_kernel(const float* __restrict__ X, const int32_t* __restrict__ offsets,
                                                      const float* __restrict__ W0, const float* __restrict__ W1,
                                                      float* __restrict__ C, int E, int N, int K) {
  constexpr int BM = 32, BN = 64, BK = 32;
  __shared__ float xs[BM][BK + 1];
  __shared__ float ws[NW][BN][BK + 1];

  const TileLoc loc = locate_tile(offsets, E, BM, blockIdx.y);
  if (loc.expert < 0) return;
  const int tid = threadIdx.x, tx = tid & 63, ty = tid >> 6;
  const int rows = min(loc.row_end - loc.row0, BM);
  const int n0 = blockIdx.x * BN;

  float acc[NW][8];
#pragma unroll
  for (int s = 0; s < NW; ++s)
#pragma unroll
    for (int r = 0; r < 8; ++r) acc[s][r] = 0.f;

  const int xr = tid >> 3, xc = (tid & 7) * 4;   // x tile: 32 rows x 8 float4
  const int wr = tid >> 2, wc = (tid & 3) * 8;   // w tile: 64 rows x 4 x (2 float4)
  for (int k0 = 0; k0 < K; k0 += BK) {
    float4 xv = {0.f, 0.f, 0.f, 0.f};
    if (xr < rows) xv = *reinterpret_cast<const float4*>(X + (size_t)(loc.row0 + xr) * K + k0 + xc);
    xs[xr][xc + 0] = xv.x; xs[xr][xc + 1] = xv.y; xs[xr][xc + 2] = xv.z; xs[xr][xc + 3] = xv.w;
#pragma unroll
    for (int s = 0; s < NW; ++s) {
      const float* Wm = s == 0 ? W0 : W1;
      float4 a = {0.f, 0.f, 0.f, 0.f}, b = a;
      if (n0 + wr < N) {
        const float* p = Wm + ((size_t)loc.expert * N + n0 + wr) * K + k0 + wc;
        a = *reinterpret_cast<const float4*>(p);
        b = *reinterpret_cast<const float4*>(p + 4);
      }
      float* d = &ws[s][wr][wc];
      d[0] = a.x; d[1] = a.y; d[2] = a.z; d[3] = a.w; d[4] = b.x; d[5] = b.y; d[6] = b.z; d[7] = b.w;
    }
    __syncthreads();
#pragma unroll 8
    for (int kk = 0; kk < BK; ++kk) {
      float xv8[8];
#pragma unroll
      for (int r = 0; r < 8; ++r) xv8[r] = xs[ty * 8 + r][kk];
#pragma unroll
      for (int s = 0; s < NW; ++s) {
        const float wv = ws[s][tx][kk];
#pragma unroll
        for (int r = 0; r < 8; ++r) acc[s][r] = fmaf(xv8[r], wv, acc[s][r]);
      }
    }
    __syncthreads();
  }
  if (n0 + tx < N) {
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const int row = ty * 8 + r;
      if (row < rows) {
        float v = acc[0][r];
        if (NW == 2) v = (v / (1.f + expf(-v))) * acc[NW - 1][r];
        C[(size_t)(loc.row0 + row) * N + n0 + tx] = v;
      }
    }
  }
}

template <int MT, int NW>
void launch_bf16(const uint4* X, const int32_t* offsets, const uint4* Wp, __bf16* C, int A, int E, int N, int K,
                 hipStream_t stream) {
  constexpr int BM = 32 * MT;
  const int slots = A / BM + (E < A ? E : A);  // upper bound on sum_e ceil(c_e / BM)
  const dim3 grid((N / 32 + 3) / 4, slots), block(256);
  // ring depth: K / 64 chunks must be a multiple of it (K is a multiple of 128)
  static const char* env_nst = getenv("MOE_DBG_NST");
  const bool want4 = !(env_nst && atoi(env_nst) == 2);
  if constexpr (MT < 8) {
    if (K % 256 == 0 && want4) {
    hipLaunchKernelGGL((ffn_bf16_kernel<MT, NW, 4>), grid, block, 0, stream, reinterpret_cast<const u32x4*>(X), offsets,
                       reinterpret_cast<const u32x4*>(Wp), C, E, N, K);
      return;
    }
  }
    hipLaunchKernelGGL((ffn_bf16_kernel<MT, NW, 2>), grid, block, 0, stream, reinterpret_cast<const u32x4*>(X), offsets,
                       reinterpret_cast<const u32x4*>(Wp), C, E, N, K);
}

template <int NW>
void launch_bf16_mt(int MT, const uint4* X, const int32_t* offsets, const uint4* Wp, __bf16* C, int A, int E, int N,
                    int K, hipStream_t stream) {
  switch (MT) {
    case 1: launch_bf16<1, NW>(X, offsets, Wp, C, A, E, N, K, stream); break;
    case 2: launch_bf16<2, NW>(X, offsets, Wp, C, A, E, N, K, stream); break;
    case 4: launch_bf16<4, NW>(X, offsets, Wp, C, A, E, N, K, stream); break;
    default: launch_bf16<8, NW>(X, offsets, Wp, C, A, E, N, K, stream); break;
  }
}

}  // namespace

size_t packed_weight_bytes(const moe_config& cfg) {
  const size_t elem = cfg.dtype == MOE_BF16 ? 2 : 4;
  return (size_t)3 * cfg.E * cfg.d * cfg.f * elem;
}

hipError_t launch_pack_weights(const moe_config& cfg, const void* w_gate, const void* w_up, const void* w_down,
                               void* packed, hipStream_t stream) {
  const size_t one = (size_t)cfg.E * cfg.d * cfg.f;  // elements of one matrix set
  if (cfg.dtype == MOE_BF16) {
    uint4* p = static_cast<uint4*>(packed);
    hipLaunchKernelGGL(pack_bf16_kernel, dim3(4096), dim3(256), 0, stream, static_cast<const uint4*>(w_gate),
                       static_cast<const uint4*>(w_up), cfg.E, cfg.f, cfg.d, 2, p);
    hipLaunchKernelGGL(pack_bf16_kernel, dim3(4096), dim3(256), 0, stream, static_cast<const uint4*>(w_down),
                       static_cast<const uint4*>(w_down), cfg.E, cfg.d, cfg.f, 1, p + 2 * one / 8);
    return hipGetLastError();
  }
  float* p = static_cast<float*>(packed);
  hipError_t err = hipMemcpyAsync(p, w_gate, one * 4, hipMemcpyDeviceToDevice, stream);
  if (err == hipSuccess) err = hipMemcpyAsync(p + one, w_up, one * 4, hipMemcpyDeviceToDevice, stream);
  if (err == hipSuccess) err = hipMemcpyAsync(p + 2 * one, w_down, one * 4, hipMemcpyDeviceToDevice, stream);
  return err;
}

hipError_t launch_ffn_stage(const moe_config& cfg, int stage, int T, const void* in, const int32_t* offsets,
                            const void* packed, void* out, hipStream_t stream) {
  const int A = T * cfg.k;
  if (A == 0) return hipSuccess;
  const size_t one = (size_t)cfg.E * cfg.d * cfg.f;  // elements of one matrix set
  const int N = stage == 0 ? cfg.f : cfg.d, K = stage == 0 ? cfg.d : cfg.f;
  if (cfg.dtype == MOE_BF16) {
    // m-tile height from the mean rows per expert (the host never sees the real counts);
    // mean + 3 sqrt(mean) covers the spread of a near-uniform router, so most experts fit one m-tile
    const float mean = (float)A / cfg.E;
    const float want = mean + 3.f * sqrtf(mean);
    int MT = want <= 32.f ? 1 : want <= 64.f ? 2 : want <= 128.f ? 4 : 8;
    static const char* env_mt = getenv("MOE_DBG_MT");
    if (env_mt) MT = atoi(env_mt);
    const uint4* wp = static_cast<const uint4*>(packed);
    if (stage == 0)
      launch_bf16_mt<2>(MT, static_cast<const uint4*>(in), offsets, wp, static_cast<__bf16*>(out), A, cfg.E, N, K, stream);
    else
      launch_bf16_mt<1>(MT, static_cast<const uint4*>(in), offsets, wp + 2 * one / 8, static_cast<__bf16*>(out), A,
                        cfg.E, N, K, stream);
    return hipGetLastError();
  }
  const float* wp = static_cast<const float*>(packed);
  const dim3 grid((N + 63) / 64, A / 32 + (cfg.E < A ? cfg.E : A));
  if (stage == 0)
    hipLaunchKernelGGL((ffn_f32_kernel<2>), grid, dim3(256), 0, stream, static_cast<const float*>(in), offsets, wp,
                       wp + one, static_cast<float*>(out), cfg.E, N, K);
  else
    hipLaunchKernelGGL((ffn_f32_kernel<1>), grid, dim3(256), 0, stream, static_cast<const float*>(in), offsets,
                       wp + 2 * one, wp + 2 * one, static_cast<float*>(out), cfg.E, N, K);
  return hipGetLastError();
}

}  // namespace moe
