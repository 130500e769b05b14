// Expert FFN as a grouped SwiGLU GEMM (paper Section 4.2, Table 3: "FFN Input" (b_e, h) x (h, h')
// and "FFN Output" (b_e, h') x (h', h); tensor-parallel degree 1), plus the one-time weight pre-pack.
//
// bf16 path. Both GEMMs are C[m, n] = sum_k X[m, k] * W[n, k] with K contiguous in X and W. The
// weights are pre-packed into matrix-core operand order: a "fragment" is the 32 (n) x 16 (k)
// operand of one v_mfma_f32_32x32x16_bf16, stored as 64 lanes x 16 bytes = 1 KiB where lane
// l = (n % 32) + 32 * g holds k = 16 * ks + 8 * g .. + 7. Fragments come in pairs per k-step:
// (gate, up) of one 32-column tile for the input GEMM, two neighbouring 32-column tiles for the
// output GEMM. A wavefront streams its fragments from HBM straight into registers, 1 KiB fully
// contiguous per load. Tokens (the other operand) are staged through LDS and shared by the
// wavefronts of the workgroup. Row ranges stay on the device: every kernel works on a list of
// segments (rows [begin, end) to be multiplied with one expert's weights). For the plain layer
// segment e is expert e's rows, begin = offsets, end = offsets + 1; with several copies of a
// popular expert (Section 6, "Load balance") a copy is a segment holding part of that expert's rows.
#include <math.h>
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

struct Segs {
  const int32_t* begin;   // [count] first row of each segment
  const int32_t* end;     // [count] one past its last row
  const int32_t* expert;  // [count] whose weights the segment uses; nullptr: segment s uses expert s
  int count;              // segments, <= 256
  int experts;            // experts in the packed weights
  int rows_cap;           // rows the activation buffers hold; ranges are clipped to it
  int tall_first;         // large-batch kernel: order the segments by tile height (see locate_tile)
  int rows_above;         // this launch takes only the segments with rows_above < rows <= rows_upto:
  int rows_upto;          //   the counts stay on the device, so each kernel picks its own segments there
};

struct TileLoc {
  int expert;   // segment index; -1: this workgroup has no tile
  int row0;     // first row of the m-tile
  int rows;     // rows of the m-tile (<= BM)
  int within;   // position inside the expert's block of `per_tile`-sized groups (see locate_tile)
  int tiles;    // m-tiles of this expert
  int step;     // rows of the expert's full-height tiles (its last tile may hold fewer)
};

// Work items are ordered segment-major ("expert" below = segment). Expert e owns
// tiles_e * per_tile consecutive positions, tiles_e = ceil(c_e / BM). Position q inside an expert's
// block maps to m-tile q % tiles_e and `within` = q / tiles_e, so the m-tiles that share one group
// of weight columns are neighbours.
// Order of the segments: by index, or (TALL_FIRST and segs.tall_first) segments with taller tiles
// first, equal heights by index. A launch of only a few rounds of workgroups then ends with its
// shortest tiles instead of a late, lonely tall one (an expert that needs a second tile; skewed
// loads). Long launches keep index order: there the mix of tall (matrix-core-heavy) and short
// (memory-heavy) tiles running side by side is worth more than the shorter tail.
// BALANCED: the expert's rows are split evenly over its tiles in multiples of 32 rows (so
// 1072 rows with BM = 256 become 224 + 224 + 224 + 224 + 176, not 4 x 256 + 48).
// All threads of the workgroup (>= 256, one per expert) must call this.
template <bool BALANCED, bool TALL_FIRST = false>
__device__ __forceinline__ TileLoc locate_tile(const Segs& segs, int BM, int per_tile, int pos) {
  __shared__ int2 s_key[TALL_FIRST ? 256 : 1];  // (tile height, tiles) of every segment
  __shared__ int s_wave_total[8];
  __shared__ int s_loc[6];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  int lo = 0, hi = 0;
  if (tid < segs.count) {
    lo = max(0, min(segs.begin[tid], segs.rows_cap));
    hi = max(lo, min(segs.end[tid], segs.rows_cap));
  }
  int rows = hi - lo;
  if (rows <= segs.rows_above || rows > segs.rows_upto) rows = 0;  // another launch's segment
  int nt = (rows + BM - 1) / BM;
  int step = nt == 0 ? 0 : BM;  // rows per tile
  if (BALANCED && nt > 0) {
    // All tiles of an expert run the schedule of its tallest tile, so the split is chosen by the row
    // groups it schedules, tiles x ceil(groups / tiles): one tile more than necessary is taken when
    // that schedules fewer groups and the tiles stay at least 6 groups tall (29 groups: 5 x 6 = 30
    // instead of 4 x 8 = 32).
    const int G = (rows + 31) >> 5;
    int mu = (G + nt - 1) / nt;
    const int mu1 = (G + nt) / (nt + 1);
    if (mu1 >= 6 && (nt + 1) * mu1 < nt * mu) {
      ++nt;
      mu = mu1;
    }
    step = mu * 32;
  }
  const bool by_height = TALL_FIRST && segs.tall_first;  // uniform over the grid
  int excl;  // tiles of the segments ordered before this one
  if (by_height) {
    if (tid < 256) s_key[tid] = make_int2(step, nt);
    if (tid == 0) s_loc[0] = -1;
    __syncthreads();
    excl = 0;
    if (tid < segs.count && nt > 0) {
      for (int o0 = 0; o0 < segs.count; o0 += 8) {
        int2 key[8];  // eight broadcast reads in flight, then branch-free arithmetic (entries past count hold 0 tiles)
#pragma unroll
        for (int j = 0; j < 8; ++j) key[j] = s_key[min(o0 + j, 255)];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int before = (key[j].x > step) | ((key[j].x == step) & (o0 + j < tid));
          excl += key[j].y & -before;
        }
      }
    }
  } else {
    int incl = nt;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int o = __shfl_up(incl, off);
      if (lane >= off) incl += o;
    }
    if (lane == 63 && w < 8) s_wave_total[w] = incl;
    if (tid == 0) s_loc[0] = -1;
    __syncthreads();
    excl = incl - nt;
    for (int ww = 0; ww < w && ww < 4; ++ww) excl += s_wave_total[ww];  // experts live in the first 4 wavefronts
  }
  const int first = excl * per_tile;
  if (tid < segs.count && nt > 0 && pos >= first && pos < first + nt * per_tile) {
    const int q = pos - first;
    const int r0 = lo + (q % nt) * step;
    s_loc[0] = tid;
    s_loc[1] = r0;
    s_loc[2] = max(0, min(step, hi - r0));
    s_loc[3] = q / nt;
    s_loc[4] = nt;
    s_loc[5] = step;
  }
  __syncthreads();
  TileLoc t;
  t.expert = s_loc[0];
  t.row0 = s_loc[1];
  t.rows = s_loc[2];
  t.within = s_loc[3];
  t.tiles = s_loc[4];
  t.step = s_loc[5];
  return t;
}

// Expert whose weights segment `seg` uses; -1 if the list names none of the packed experts.
__device__ __forceinline__ int segment_expert(const Segs& segs, int seg) {
  const int e = segs.expert ? segs.expert[seg] : seg;
  return (unsigned)e < (unsigned)segs.experts ? e : -1;
}

// silu(g) = g / (1 + e^-g) for the bf16 path: hardware exponential and reciprocal (about 1 ulp each, far
// inside the bf16 rounding that follows) instead of an IEEE division, which costs a dozen instructions per
// element of an epilogue that computes 128 of them per lane. Every bf16 kernel uses this one function, so
// they still agree bit for bit.
__device__ __forceinline__ float silu(float g) { return g * __builtin_amdgcn_rcpf(1.f + __expf(-g)); }

// ------------------------------------------------------------------------------------------
// bf16 weight pre-pack: canonical [E, N, K] matrices (K contiguous) -> fragment pairs
//   packed[(((e * NP + p) * KS + ks) * 2 + sel) * 64 + lane]   (16-byte units), KS = K / 16.
// gate_up = true : NP = N / 32, fragment (p, sel) is rows 32 p .. of w0 (gate, sel 0) or w1 (up, sel 1)
// gate_up = false: NP = N / 64, fragment (p, sel) is rows 32 (2 p + sel) .. of w0
__global__ __launch_bounds__(256) void pack_bf16_kernel(const uint4* __restrict__ w0, const uint4* __restrict__ w1,
                                                        int E, int N, int K, int gate_up,
                                                        uint4* __restrict__ packed) {
  const int NP = gate_up ? N / 32 : N / 64, KS = K / 16;
  const size_t total = (size_t)E * NP * KS * 128;
  for (size_t u = (size_t)blockIdx.x * 256 + threadIdx.x; u < total; u += (size_t)gridDim.x * 256) {
    size_t q = u;
    const int lane = q % 64; q /= 64;
    const int sel = q % 2;   q /= 2;
    const int ks = q % KS;   q /= KS;
    const int p = q % NP;    q /= NP;
    const int e = (int)q;
    const int n = (gate_up ? p : 2 * p + sel) * 32 + (lane & 31);
    const int kv = ks * 2 + (lane >> 5);  // 16-byte unit along K
    const uint4* w = (gate_up && sel) ? w1 : w0;
    packed[u] = w[((size_t)e * N + n) * (K / 8) + kv];
  }
}

// ------------------------------------------------------------------------------------------
// bf16 grouped GEMM on the matrix cores.
//
// Workgroup = WN x WM wavefronts. Wavefront (wn, wm) owns weight unit `WN * group + wn` and the
// 32-row groups [wm * MTW, (wm + 1) * MTW) of an m-tile of BM = 32 * MTW * WM rows.
//   NW = 2: the unit is a fragment pair; GATEUP: C = silu(X Wg^T) .* (X Wu^T) on one 32-column
//           tile, applied to the accumulators in registers; otherwise two 32-column tiles of X W^T
//   NW = 1: the unit is one fragment of a pair (one 32-column tile; loads stride over its twin)
// K is walked in chunks of 64 (4 MFMA k-steps).
//
// Grid (1-D), made for 8 XCDs with one L2 each: workgroups are dealt to XCDs round-robin, so id % 8
// is the XCD and id / 8 the position in that XCD's queue. For expert e each XCD owns the weight-unit
// groups g = 8 * j + (xcd + e) % 8; its queue is expert-major, then j, then m-tile: the m-tiles of one expert that
// read the same weights run next to each other on one L2, and no weight line is wanted by two XCDs.
//
// Pipeline. Global loads return in order, so one register ring of NST chunks carries both
// operands: weights for chunk c + NST and the workgroup's share of the token slab for chunk
// c + NST + 1 are issued in stage c. The token share for chunk c + 1 is written to LDS at the end
// of stage c (double-buffered slab, one barrier per chunk). Loads never branch (indices past the
// end are clamped; what they fetch is unused), which keeps the s_waitcnt vmcnt counts exact: about
// NST - 1 chunks stay in flight across every wait. Weights that are read once are loaded non-temporally
// (worth +13 % of streaming bandwidth).
//
// LDS slab: [BM rows][8 units of 16 B], unit index XOR ((row >> 1) & 7): both the row-major
// writes and the operand-order reads (32 rows, same logical unit) are free of bank conflicts
// (measured with the LDS bank-conflict counter; XOR with row & 7 is not).
template <int MTW, int NW, int NST, int WN, int WM, bool GATEUP>
struct Gemm {
  static constexpr int THREADS = 64 * WN * WM;
  static constexpr int BM = 32 * MTW * WM;
  static constexpr int RPP = THREADS / 8;  // slab rows written per pass (8 threads per 128-byte row)
  static constexpr int PASSES = (BM + RPP - 1) / RPP;

  u32x4 (*slab)[BM * 8];
  const u32x4* wbase;
  const u32x4* xrow[PASSES];
  int NC, swz_w, trow, frow, fg, mbase;

  // MU = 32-row groups of this wavefront that hold real rows (the others are skipped entirely);
  // NTL: non-temporal weight loads (weights that no other tile reads).
  template <int MU, bool NTL>
  __device__ __forceinline__ void run(floatx16 (&acc)[NW][MTW]) {
    u32x4 wreg[NST][4 * NW];
    u32x4 treg[NST][PASSES];
    auto load_w = [&](auto st_, int c) {
      constexpr int st = decltype(st_)::value;
      c = min(c, NC - 1);
#pragma unroll
      for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int i = 0; i < NW; ++i) {
          const u32x4* p = wbase + (size_t)(c * 4 + s) * 128 + i * 64;
          wreg[st][s * NW + i] = NTL ? __builtin_nontemporal_load(p) : *p;
        }
    };
    auto load_t = [&](auto st_, int c) {
      constexpr int st = decltype(st_)::value;
      c = min(c, NC - 1);
#pragma unroll
      for (int p = 0; p < PASSES; ++p) treg[st][p] = xrow[p][c * 8];
    };
    auto store_t = [&](auto st_, auto buf_) {
      constexpr int st = decltype(st_)::value;
      constexpr int buf = decltype(buf_)::value;
#pragma unroll
      for (int p = 0; p < PASSES; ++p)
        if (BM % RPP == 0 || p * RPP + trow < BM) slab[buf][p * RPP * 8 + swz_w] = treg[st][p];
    };
    // One pipeline stage for chunk c held in ring slot st (= c % NST); chunk parity == st parity.
    auto stage = [&](auto st_, int c) {
      constexpr int st = decltype(st_)::value;
      constexpr int buf = st & 1;
      constexpr int nxt = (st + 1) % NST;
#pragma unroll
      for (int s = 0; s < 4; ++s) {
#pragma unroll
        for (int m = 0; m < MU; ++m) {
          const int row = (mbase + m) * 32 + frow;
          const bf16x8 b = __builtin_bit_cast(bf16x8, slab[buf][row * 8 + ((2 * s + fg) ^ ((row >> 1) & 7))]);
#pragma unroll
          for (int i = 0; i < NW; ++i)
            acc[i][m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wreg[st][s * NW + i]), b,
                                                                acc[i][m], 0, 0, 0);
        }
      }
      load_w(st_, c + NST);
      store_t(std::integral_constant<int, nxt>{}, std::integral_constant<int, buf ^ 1>{});
      load_t(std::integral_constant<int, nxt>{}, c + 1 + NST);
      __syncthreads();
    };

    // prologue: every first load goes out at once (chunk 0 tokens, then the steady-state issue order
    // W[c], tokens[c + 1]), so the workgroup pays one memory latency, not two, before its first MFMA
    u32x4 t0[PASSES];
#pragma unroll
    for (int p = 0; p < PASSES; ++p) t0[p] = xrow[p][0];
    static_for<0, NST>([&](auto st_) {
      constexpr int st = decltype(st_)::value;
      load_w(st_, st);
      load_t(std::integral_constant<int, (st + 1) % NST>{}, st + 1);
    });
#pragma unroll
    for (int p = 0; p < PASSES; ++p)
      if (BM % RPP == 0 || p * RPP + trow < BM) slab[0][p * RPP * 8 + swz_w] = t0[p];
    __syncthreads();
    // NC is a multiple of NST (K is a multiple of 128 and NST is 2), so there is no remainder loop
    for (int c0 = 0; c0 < NC; c0 += NST) static_for<0, NST>([&](auto st_) { stage(st_, c0 + decltype(st_)::value); });
  }
};

template <int MTW, int NW, int NST, int WN, int WM, bool GATEUP>
__global__ __launch_bounds__(64 * WN * WM) void ffn_bf16_kernel(const u32x4* __restrict__ X, const Segs segs,
                                                               const u32x4* __restrict__ Wp, __bf16* __restrict__ C,
                                                               int N, int K) {
  static_assert(NST % 2 == 0, "chunk parity must equal ring-slot parity");
  static_assert(WN * WM >= 4, "the tile locator needs one thread per expert (256)");
  static_assert(NW == 2 || !GATEUP, "gate and up fragments are consumed together");
  using G = Gemm<MTW, NW, NST, WN, WM, GATEUP>;
  constexpr int BM = G::BM;
  __shared__ u32x4 slab[2][BM * 8];

  const int NP = GATEUP ? N / 32 : N / 64;            // fragment pairs along N
  const int units = NW == 2 ? NP : 2 * NP;            // weight units (one per wavefront column)
  const int groups = (units + WN - 1) / WN;
  const int groups_per_xcd = (groups + 7) / 8;
  const int xcd = blockIdx.x & 7;
  const TileLoc loc = locate_tile<false>(segs, BM, groups_per_xcd, blockIdx.x >> 3);
  if (loc.expert < 0) return;
  const int group = loc.within * 8 + ((xcd + loc.expert) & 7);  // rotate per expert: evens out a group count that is not a multiple of 8
  const int wexp = segment_expert(segs, loc.expert);
  if (group >= groups || wexp < 0) return;

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int wn = w % WN, wm = w / WN;
  const int KS = K / 16, KV = K / 8;
  const int unit = group * WN + wn;
  const bool has_n = unit < units;
  const int rows = loc.rows;

  G g;
  g.slab = slab;
  g.NC = K / 64;
  {
    const int u = has_n ? unit : 0;
    const int pair = NW == 2 ? u : u >> 1, sel = NW == 2 ? 0 : u & 1;
    g.wbase = Wp + ((size_t)wexp * NP + pair) * KS * 128 + sel * 64 + lane;
  }
  g.trow = tid >> 3;
  const int tunit = tid & 7;
  g.swz_w = g.trow * 8 + (tunit ^ ((g.trow >> 1) & 7));
#pragma unroll
  for (int p = 0; p < G::PASSES; ++p)
    g.xrow[p] = X + (size_t)(loc.row0 + min(p * G::RPP + g.trow, rows - 1)) * KV + tunit;
  g.frow = lane & 31;
  g.fg = lane >> 5;
  g.mbase = wm * MTW;

  floatx16 acc[NW][MTW];
#pragma unroll
  for (int i = 0; i < NW; ++i)
#pragma unroll
    for (int m = 0; m < MTW; ++m)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][m][r] = 0.f;

  // 32-row groups of this wavefront that hold real rows; every wavefront runs the same number of
  // stages and barriers whatever its count is.
  int mu = (rows - g.mbase * 32 + 31) / 32;
  mu = __builtin_amdgcn_readfirstlane(max(0, min(mu, MTW)));
  // A segment of up to BM rows is one tile and its weights are read once: non-temporal loads (worth
  // +13 % of streaming bandwidth). The tiles of a taller segment sit next to each other in the queue
  // and read the same weights: cached loads, so that the second tile finds them in L2. Only the
  // gate|up kernel carries the second flavour of the K loop: with it the compiler schedules the
  // first flavour differently, which measured 1.5-2 % faster there and 4 % slower in the output GEMM.
  const bool once = loc.tiles == 1;
  static_for<0, MTW + 1>([&](auto mu_) {
    if (mu == decltype(mu_)::value) {
      if (once || !GATEUP) g.template run<decltype(mu_)::value, true>(acc);
      else g.template run<decltype(mu_)::value, false>(acc);
    }
  });

  if (!has_n) return;
  // acc[i][m][r] holds row (mbase + m) * 32 + lane % 32, column 8 * (r / 4) + 4 * (lane / 32) + r % 4 of its tile
#pragma unroll
  for (int m = 0; m < MTW; ++m) {
    const int row = (g.mbase + m) * 32 + g.frow;
    if (row < rows) {
      __bf16* crow = C + (size_t)(loc.row0 + row) * N + 4 * g.fg;
#pragma unroll
      for (int i = 0; i < (GATEUP ? 1 : NW); ++i) {
        const int tile = GATEUP ? unit : (NW == 2 ? 2 * unit + i : unit);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          bf16x4 o;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            float v = acc[i][m][q * 4 + j];
            if (GATEUP) v = silu(v) * acc[NW - 1][m][q * 4 + j];
            o[j] = (__bf16)v;
          }
          *reinterpret_cast<bf16x4*>(crow + tile * 32 + 8 * q) = o;
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// bf16 grouped GEMM for large per-expert batches (matrix-core bound).
//
// Workgroup = 4 wavefronts, one per SIMD with the whole 512-entry register file: wavefront w owns
// fragment pair `4 * group + w` and all rows of an m-tile of up to kWideBM = 256 rows (up to
// 2 x 8 accumulator tiles = 256 registers). An expert's rows are split evenly over its tiles in
// multiples of 32 (see locate_tile), so a tile runs MU = 1..8 32-row groups. Same weight layout and
// XCD mapping as above; the order of the experts in the queue is chosen per launch (locate_tile).
//
// With one wavefront per SIMD nothing hides LDS latency but the wavefront's own schedule, so the
// k-step loop is software-pipelined by hand: token fragments are read R - 1 (row group, k-step)
// items ahead of the two MFMAs that consume them, through a ring of R fragment registers (the
// compiler on its own sinks every ds_read next to its use); a scheduling barrier at every k-step
// boundary plus per-k-step group barriers pin that order. The slab is triple-buffered: stage c
// reads buffer c % 3, takes the first fragments of chunk c + 1 from buffer (c + 1) % 3 before the
// stage's barrier, and writes the tokens of chunk c + 2 into buffer (c + 2) % 3, so no MFMA waits
// on LDS right after a barrier.
// The tokens of chunk c + 2 are loaded from global memory TPF stages before the stage that stores
// them: one stage for tall tiles, two for tiles of up to kWideTpf2Max row groups, whose stages are
// shorter than an L2 round trip under load (and which have the registers for a second chunk in flight).
constexpr int kWideBM = 256;
constexpr int kWideTpf2Max = 5;

template <bool GATEUP, int MU, int NST, bool NTL, int TPF>
__device__ __forceinline__ void wide_tile(const u32x4* __restrict__ X, const u32x4* __restrict__ wbase,
                                          __bf16* __restrict__ C, u32x4* __restrict__ slab, int row0, int rows, int N,
                                          int K, int pair, bool has_n) {
  constexpr int BUF = kWideBM * 8;            // 16-byte units per slab buffer
  constexpr int R = (MU % 2 == 0) ? 8 : 4;    // fragment ring; divides the 4 * MU items of a stage
  constexpr int D = R - 1;                    // read-ahead distance in items
  constexpr int ITEMS = 4 * MU;
  const int tid = threadIdx.x, lane = tid & 63;
  const int NC = K / 64, KV = K / 8;
  const int trow = tid >> 3, tunit = tid & 7;
  const int swz_w = trow * 8 + (tunit ^ ((trow >> 1) & 7));
  const u32x4* xrow[MU];  // pass p covers rows 32 p .. 32 p + 31
#pragma unroll
  for (int p = 0; p < MU; ++p) xrow[p] = X + (size_t)(row0 + min(p * 32 + trow, rows - 1)) * KV + tunit;
  const int frow = lane & 31, fg = lane >> 5;
  int rd[4];  // slab unit of this lane's fragment piece in k-step s (row group 0)
#pragma unroll
  for (int s = 0; s < 4; ++s) rd[s] = frow * 8 + ((2 * s + fg) ^ ((frow >> 1) & 7));

  u32x4 wreg[NST][8];
  u32x4 treg[TPF][MU];  // token chunks in flight, loaded TPF stages before they go to LDS
  bf16x8 bfr[R];
  floatx16 acc[2][MU];

  auto load_t = [&](auto slot_, int c) {
    c = min(c, NC - 1);
#pragma unroll
    for (int p = 0; p < MU; ++p) treg[decltype(slot_)::value][p] = xrow[p][c * 8];
  };
  auto store_t = [&](auto slot_, int boff) {
#pragma unroll
    for (int p = 0; p < MU; ++p) slab[boff + p * 256 + swz_w] = treg[decltype(slot_)::value][p];
  };
  auto load_w_step = [&](auto st_, int c, int s) {
    constexpr int st = decltype(st_)::value;
    c = min(c, NC - 1);
    const u32x4* p = wbase + (size_t)(c * 4 + s) * 128;
    wreg[st][2 * s] = NTL ? __builtin_nontemporal_load(p) : p[0];
    wreg[st][2 * s + 1] = NTL ? __builtin_nontemporal_load(p + 64) : p[64];
  };
  // fragment of item it = s * MU + m of the chunk in buffer `boff`
  auto frag = [&](int boff, int it) {
    return __builtin_bit_cast(bf16x8, slab[boff + (it % MU) * 256 + rd[it / MU]]);
  };

  // prologue: all first loads go out at once (tokens of chunks 0 .. 1 + TPF, then the weights of the
  // first NST chunks), so the workgroup pays one memory latency before its first MFMA; chunks 0 and 1
  // go to LDS, chunk 2 (and 3) stay in registers for stage 0 (and 1)
  {
    u32x4 t0[MU], t1[MU];
#pragma unroll
    for (int p = 0; p < MU; ++p) t0[p] = xrow[p][0];
#pragma unroll
    for (int p = 0; p < MU; ++p) t1[p] = xrow[p][8];
#pragma unroll
    for (int p = 0; p < MU; ++p) treg[0][p] = xrow[p][16];  // K >= 256 (the launcher sees to it): chunks 1..3 exist
    if constexpr (TPF == 2) {
#pragma unroll
      for (int p = 0; p < MU; ++p) treg[1][p] = xrow[p][24];
    }
    static_for<0, NST>([&](auto st_) {
#pragma unroll
      for (int s = 0; s < 4; ++s) load_w_step(st_, decltype(st_)::value, s);
    });
#pragma unroll
    for (int p = 0; p < MU; ++p) slab[p * 256 + swz_w] = t0[p];
#pragma unroll
    for (int p = 0; p < MU; ++p) slab[BUF + p * 256 + swz_w] = t1[p];
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int m = 0; m < MU; ++m)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][m][r] = 0.f;
#pragma unroll
  for (int it = 0; it < D; ++it) bfr[it % R] = frag(0, it);  // D <= ITEMS for every MU >= 2; MU = 1: D = 3 < 4

  int cur = 0, nxt = BUF, wr = 2 * BUF;
  auto stage = [&](auto st_, int c) {
    constexpr int st = decltype(st_)::value;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
#pragma unroll
      for (int m = 0; m < MU; ++m) {
        const int it = s * MU + m;
        // read ahead: item it + D of this chunk, or of the next chunk's buffer past the end
        if (it + D < ITEMS) bfr[(it + D) % R] = frag(cur, it + D);
        else bfr[(it + D) % R] = frag(nxt, it + D - ITEMS);
        acc[0][m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wreg[st][2 * s]), bfr[it % R],
                                                            acc[0][m], 0, 0, 0);
        acc[1][m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wreg[st][2 * s + 1]),
                                                            bfr[it % R], acc[1][m], 0, 0, 0);
      }
      if (s == 0) {
        // token loads go out before this stage's weight loads: loads return in order, and waiting
        // for these tokens one stage from now must not wait for weights needed NST stages from now
        store_t(std::integral_constant<int, st % TPF>{}, wr);  // tokens of chunk c + 2
        load_t(std::integral_constant<int, st % TPF>{}, c + 2 + TPF);
      }
      load_w_step(st_, c + NST, s);  // this k-step's weight registers are free again
#pragma unroll
      for (int m = 0; m < MU; ++m) {
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // 1 LDS read
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);  // 2 MFMA
        if (s == 0) {
          __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);  // 1 LDS write
          __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);  // 1 global load
        }
      }
      __builtin_amdgcn_sched_group_barrier(0x020, 2, 0);  // the two weight loads
      __builtin_amdgcn_sched_barrier(0);                  // nothing moves across a k-step boundary
    }
    __syncthreads();
    const int t = cur;
    cur = nxt;
    nxt = wr;
    wr = t;
  };
  for (int c0 = 0; c0 < NC; c0 += NST) static_for<0, NST>([&](auto st_) { stage(st_, c0 + decltype(st_)::value); });

  // Epilogue. In the accumulators a lane holds 4 consecutive columns of one row per register quad, so
  // storing them directly writes 16-byte pieces of 32 different rows per instruction, and the time a
  // workgroup waits for those partial-line writes is pure overhead (up to a quarter of a short-K
  // tile). The results are instead transposed through the slab (idle now: the K loop ended with a
  // barrier) and leave as whole 16-byte units, consecutive lanes on consecutive units of a row.
  // 8-byte slot (unit u, half fg) of row r sits at r * SL + ((u ^ g(r)) << 1 | fg); g(r) spreads the
  // row-strided writes over the banks (2-way conflicts) and keeps the unit-strided reads conflict-free.
  // The lane arithmetic below restarts from the thread id behind an opaque asm: otherwise the compiler
  // computes the epilogue's addresses before the K loop and keeps them in registers across it, which
  // the 7- and 8-group tiles cannot afford.
  int etid = threadIdx.x;
  asm volatile("" : "+v"(etid));
  const int w = etid >> 6, elane = etid & 63, erow = elane & 31, eg = elane >> 5;
  if constexpr (GATEUP) {
    // Each wavefront owns 32 columns (64 bytes per row) but the four of a workgroup own 128
    // consecutive ones: all write into one [32 MU rows][256 bytes] image, one barrier, and every
    // store instruction then covers 4 full 256-byte row pieces.
    uint2* ep8 = reinterpret_cast<uint2*>(slab);
    if (has_n) {
#pragma unroll
      for (int m = 0; m < MU; ++m) {
        const int r = m * 32 + erow;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          bf16x4 o;
#pragma unroll
          for (int j = 0; j < 4; ++j) o[j] = (__bf16)(silu(acc[0][m][q * 4 + j]) * acc[1][m][q * 4 + j]);
          ep8[r * 32 + ((((w * 4 + q) ^ (r & 15)) << 1) | eg)] = __builtin_bit_cast(uint2, o);
        }
      }
    }
    __syncthreads();
    const int ru = elane & 15;
    const int col = (pair - w) * 32 + 8 * ru;      // columns of wavefronts past the last pair stay unwritten
    __bf16* cbase = C + (size_t)row0 * N + col;
#pragma unroll
    for (int t = 0; t < 2 * MU; ++t) {
      const int r = t * 16 + w * 4 + (elane >> 4);
      const u32x4 v = slab[r * 16 + (ru ^ (r & 15))];
      if (r < rows && col < N) *reinterpret_cast<u32x4*>(cbase + (size_t)r * N) = v;
    }
  } else {
    // Each wavefront owns 64 columns, a full 128-byte line per row: it transposes one 32-row group
    // at a time through a private 4 KiB piece of the slab. LDS operations of one wavefront execute
    // in order, so no barrier is needed.
    if (!has_n) return;
    uint2* ep8 = reinterpret_cast<uint2*>(slab) + w * 512;
    const u32x4* ep16 = slab + w * 256;
    const int ru = elane & 7;
    __bf16* cbase = C + (size_t)row0 * N + pair * 64 + 8 * ru;
#pragma unroll
    for (int m = 0; m < MU; ++m) {
#pragma unroll
      for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          bf16x4 o;
#pragma unroll
          for (int j = 0; j < 4; ++j) o[j] = (__bf16)acc[i][m][q * 4 + j];
          ep8[erow * 16 + ((((i * 4 + q) ^ ((erow >> 1) & 7)) << 1) | eg)] = __builtin_bit_cast(uint2, o);
        }
      }
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int r = t * 8 + (elane >> 3);         // row inside this 32-row group
        const u32x4 v = ep16[r * 8 + (ru ^ ((r >> 1) & 7))];
        if (m * 32 + r < rows) *reinterpret_cast<u32x4*>(cbase + (size_t)(m * 32 + r) * N) = v;
      }
    }
  }
}

template <bool GATEUP>
__global__ __launch_bounds__(256) void ffn_bf16_wide_kernel(const u32x4* __restrict__ X, const Segs segs,
                                                           const u32x4* __restrict__ Wp, __bf16* __restrict__ C,
                                                           int N, int K) {
  __shared__ u32x4 slab[3 * kWideBM * 8];
  const int NP = GATEUP ? N / 32 : N / 64;
  const int groups = (NP + 3) / 4;
  const int groups_per_xcd = (groups + 7) / 8;
  const int xcd = blockIdx.x & 7;
  const TileLoc loc = locate_tile<true, true>(segs, kWideBM, groups_per_xcd, blockIdx.x >> 3);
  if (loc.expert < 0) return;
  const int group = loc.within * 8 + ((xcd + loc.expert) & 7);  // rotate per expert: evens out a group count that is not a multiple of 8
  const int wexp = segment_expert(segs, loc.expert);
  if (group >= groups || loc.rows <= 0 || wexp < 0) return;
  const int pair = group * 4 + (threadIdx.x >> 6);
  const bool has_n = pair < NP;
  const int rows = loc.rows;
  const u32x4* wbase = Wp + ((size_t)wexp * NP + (has_n ? pair : 0)) * (K / 16) * 128 + (threadIdx.x & 63);
  // 32-row groups the tile runs, 1..8. The m-tiles of an expert share their weights through L2 only
  // while they sweep K side by side, so they must take the same time: an expert's shorter last tile
  // runs the schedule of its full-height tiles (its missing rows are clamped loads and skipped
  // stores; the split in locate_tile is chosen to keep that waste small).
  const int mu = __builtin_amdgcn_readfirstlane(loc.tiles > 1 ? loc.step / 32 : (rows + 31) / 32);
  // Tiles of up to 5 row groups have registers to spare for a deeper weight ring (K / 64 must divide
  // by it). An expert with a single m-tile reads its weights once: non-temporal loads, as in the
  // streaming kernel; otherwise cached loads, since the expert's m-tiles share the weights in L2.
  const bool deep = (K % 256) == 0;
  const bool once = loc.tiles == 1;
  static_for<1, kWideBM / 32 + 1>([&](auto mu_) {
    constexpr int MU = decltype(mu_)::value;
    constexpr int TPF = MU <= kWideTpf2Max ? 2 : 1;  // short stages: token loads go out two stages ahead
    if (mu == MU) {
      if (once) {
        if (MU <= 5 && deep) wide_tile<GATEUP, MU, 4, true, TPF>(X, wbase, C, slab, loc.row0, rows, N, K, pair, has_n);
        else wide_tile<GATEUP, MU, 2, true, TPF>(X, wbase, C, slab, loc.row0, rows, N, K, pair, has_n);
      } else {
        if (MU <= 5 && deep) wide_tile<GATEUP, MU, 4, false, TPF>(X, wbase, C, slab, loc.row0, rows, N, K, pair, has_n);
        else wide_tile<GATEUP, MU, 2, false, TPF>(X, wbase, C, slab, loc.row0, rows, N, K, pair, has_n);
      }
    }
  });
}

// ------------------------------------------------------------------------------------------
// f32 grouped GEMM, plain FMA: 32 (m) x 64 (n) tile per workgroup, K in chunks of 32 through LDS.
// Thread (tx = tid % 64, ty = tid / 64) computes rows ty * 8 .. + 7 of column tx.
template <int NW>
__global__ __launch_bounds__(256) void ffn_f32_kernel(const float* __restrict__ X, const Segs segs,
                                                      const float* __restrict__ W0, const float* __restrict__ W1,
                                                      float* __restrict__ C, int N, int K) {
  constexpr int BM = 32, BN = 64, BK = 32;
  __shared__ float xs[BM][BK + 1];
  __shared__ float ws[NW][BN][BK + 1];

  const TileLoc loc = locate_tile<false>(segs, BM, 1, blockIdx.x);  // m-tiles on grid.x: no 65535 limit
  if (loc.expert < 0) return;
  const int wexp = segment_expert(segs, loc.expert);
  if (wexp < 0) return;
  const int tid = threadIdx.x, tx = tid & 63, ty = tid >> 6;
  const int rows = loc.rows;
  const int n0 = blockIdx.y * BN;

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
        const float* p = Wm + ((size_t)wexp * N + n0 + wr) * K + k0 + wc;
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

// Upper bound on the m-tiles of S segments holding at most A rows: sum ceil(c / BM) <= A / BM + min(S, A);
// the balanced split of the large-batch kernel may take one more tile per segment.
inline int max_m_tiles(int A, int S, int BM, int extra = 0) { return A / BM + (1 + extra) * (S < A ? S : A); }

// `tiles` = upper bound on the m-tiles of the segments this launch takes (sizes the grid).
template <int MTW, int NW, int NST, int WN, int WM, bool GATEUP>
void launch_bf16(const void* X, const Segs& segs, const void* Wp, void* C, int tiles, int N, int K, hipStream_t stream) {
  const int NP = GATEUP ? N / 32 : N / 64;
  const int units = NW == 2 ? NP : 2 * NP;
  const int groups = (units + WN - 1) / WN;
  const int groups_per_xcd = (groups + 7) / 8;
  const dim3 grid(8 * groups_per_xcd * tiles), block(64 * WN * WM);
  hipLaunchKernelGGL((ffn_bf16_kernel<MTW, NW, NST, WN, WM, GATEUP>), grid, block, 0, stream,
                     static_cast<const u32x4*>(X), segs, static_cast<const u32x4*>(Wp), static_cast<__bf16*>(C), N, K);
}

// rows_expected = rows the launch is expected to process (only orders the tile queue).
template <bool GATEUP>
void launch_bf16_wide(const void* X, Segs segs, const void* Wp, void* C, int tiles, int rows_expected, int segs_expected,
                      int N, int K, hipStream_t stream) {
  const int NP = GATEUP ? N / 32 : N / 64;
  const int groups_per_xcd = ((NP + 3) / 4 + 7) / 8;
  // Expected workgroups with a tile: about rows / 256 + half a tile per segment, times the column
  // groups. Up to four rounds of 256 compute units the tail decides the time: tall tiles first. With at
  // most 16 segments, too, whatever the length of the launch: each expert's block of the queue is then
  // long (many column groups), index order ends the launch with whatever the last expert happens to
  // need and leaves a skewed load's heaviest expert in the middle (measured, tall-first against index
  // order: +3.5 % at 256 rows per expert on 8 experts, +3.7 % on 16 Zipf-loaded experts at 1024 mean
  // rows, neutral at 512 and 1024 uniform rows). With many segments the blocks are short, index order
  // already mixes the heights finely, and sorting would only separate the matrix-core-heavy tiles from
  // the memory-heavy ones (-3 ... -11 % on 32 and 64 experts).
  const float est = ((float)rows_expected / kWideBM + 0.5f * segs_expected) * ((NP + 3) / 4);
  segs.tall_first = est <= 4.f * 256.f || segs_expected <= 16;
  const dim3 grid(8 * groups_per_xcd * tiles), block(256);
  hipLaunchKernelGGL((ffn_bf16_wide_kernel<GATEUP>), grid, block, 0, stream, static_cast<const u32x4*>(X), segs,
                     static_cast<const u32x4*>(Wp), static_cast<__bf16*>(C), N, K);
}

// Copy r of R of expert e takes the r-th of R consecutive parts of [offsets[e], offsets[e + 1]).
__global__ void slot_segments_kernel(const int32_t* __restrict__ slot_expert, const int32_t* __restrict__ slot_copy,
                                     const int32_t* __restrict__ replicas, const int32_t* __restrict__ offsets,
                                     int n_slots, int E, int32_t* __restrict__ seg_begin,
                                     int32_t* __restrict__ seg_end) {
  const int s = blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= n_slots) return;
  const int e = slot_expert[s];
  int lo = 0, hi = 0;
  if ((unsigned)e < (unsigned)E) {
    const int R = replicas[e], r = slot_copy[s];
    if (R >= 1 && r >= 0 && r < R) {
      const long long base = offsets[e], c = offsets[e + 1] - base;
      lo = (int)(base + (r * c) / R);
      hi = (int)(base + ((r + 1) * c) / R);
    }
  }
  seg_begin[s] = lo;
  seg_end[s] = hi;
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
                       static_cast<const uint4*>(w_up), cfg.E, cfg.f, cfg.d, 1, p);
    hipLaunchKernelGGL(pack_bf16_kernel, dim3(4096), dim3(256), 0, stream, static_cast<const uint4*>(w_down),
                       static_cast<const uint4*>(w_down), cfg.E, cfg.d, cfg.f, 0, p + 2 * one / 8);
    return hipGetLastError();
  }
  float* p = static_cast<float*>(packed);
  hipError_t err = hipMemcpyAsync(p, w_gate, one * 4, hipMemcpyDeviceToDevice, stream);
  if (err == hipSuccess) err = hipMemcpyAsync(p + one, w_up, one * 4, hipMemcpyDeviceToDevice, stream);
  if (err == hipSuccess) err = hipMemcpyAsync(p + 2 * one, w_down, one * 4, hipMemcpyDeviceToDevice, stream);
  return err;
}

hipError_t launch_slot_segments(const int32_t* slot_expert, const int32_t* slot_copy, const int32_t* replicas,
                                const int32_t* offsets, int n_slots, int E, int32_t* seg_begin, int32_t* seg_end,
                                hipStream_t stream) {
  if (n_slots == 0) return hipSuccess;
  hipLaunchKernelGGL(slot_segments_kernel, dim3((n_slots + 255) / 256), dim3(256), 0, stream, slot_expert, slot_copy,
                     replicas, offsets, n_slots, E, seg_begin, seg_end);
  return hipGetLastError();
}

constexpr int kStreamRows = 128;  // rows of the streaming kernel's tile

bool ffn_picks_streaming(const moe_config& cfg, int stage, int n_segs, int rows_hint, int seg_rows_max) {
  const int K = stage == 0 ? cfg.d : cfg.f;
  const float mean = (cfg.load_skew >= 1.f ? cfg.load_skew : 1.f) * (float)rows_hint / (n_segs > 0 ? n_segs : 1);  // of a popular segment
  return K < 256 || seg_rows_max <= kStreamRows || mean + 2.f * sqrtf(mean) <= (float)kStreamRows;
}

hipError_t launch_ffn_segments(const moe_config& cfg, int stage, const int32_t* seg_begin, const int32_t* seg_end,
                               const int32_t* seg_expert, int n_segs, int rows_bound, int rows_hint, int rows_cap,
                               int seg_rows_max, const void* in, const void* packed, void* out, hipStream_t stream) {
  const int A = rows_bound;
  if (A == 0 || n_segs == 0) return hipSuccess;
  constexpr int kAll = 0x7fffffff;
  Segs segs{seg_begin, seg_end, seg_expert, n_segs, cfg.E, rows_cap, 0, 0, kAll};
  const size_t one = (size_t)cfg.E * cfg.d * cfg.f;  // elements of one matrix set
  const int N = stage == 0 ? cfg.f : cfg.d, K = stage == 0 ? cfg.d : cfg.f;
  if (cfg.dtype == MOE_BF16) {
    // Two kernels; everything that depends on a segment's row count is decided where the counts are, on
    // the device (tiles per segment, the 32-row groups a tile computes, cached or streaming weight loads,
    // ring depths). The host only picks the kernel for the launch, from what it knows: the shape and the
    // expected rows per segment.
    //  - Streaming kernel: 8 wavefronts side by side along N, 128-row tiles. A wavefront only computes the
    //    32-row groups that hold real rows, so at 8 rows per segment the tall tile costs nothing. A segment
    //    of up to 128 rows is one tile whose weights are read once; a taller one (a skewed router's popular
    //    expert) becomes several tiles that sit side by side in the queue and share the weights through L2.
    //  - Large-batch kernel: 256-row tiles, one wavefront per SIMD, tiles of every height (1..8 row groups);
    //    it needs K >= 256.
    // The streaming kernel runs when a popular segment is expected to stay within one of its tiles:
    // mean + 2 sigma <= 128 rows (mean = rows per segment x the caller's load_skew hint, sigma = sqrt(mean),
    // the spread of a near-uniform router), or when no segment can be taller (seg_rows_max: an expert gets
    // at most one row per token). Measured: at 104 and 112 mean rows it is
    // 3 % faster, at 120 mean rows the large-batch kernel wins by 9 %.
    const bool streaming = ffn_picks_streaming(cfg, stage, n_segs, rows_hint, seg_rows_max);
    const char* w = static_cast<const char*>(packed) + (stage == 0 ? 0 : 2 * one * 2);
    if (streaming) {
      const int tiles = max_m_tiles(A, n_segs, kStreamRows);
      if (stage == 0) launch_bf16<4, 2, 2, 8, 1, true>(in, segs, w, out, tiles, N, K, stream);
      else launch_bf16<4, 1, 2, 8, 1, false>(in, segs, w, out, tiles, N, K, stream);
    } else {
      const int tiles = max_m_tiles(A, n_segs, kWideBM, 1);
      if (stage == 0) launch_bf16_wide<true>(in, segs, w, out, tiles, rows_hint, n_segs, N, K, stream);
      else launch_bf16_wide<false>(in, segs, w, out, tiles, rows_hint, n_segs, N, K, stream);
    }
    return hipGetLastError();
  }
  const float* wp = static_cast<const float*>(packed);
  const dim3 grid(max_m_tiles(A, n_segs, 32), (N + 63) / 64);
  if (stage == 0)
    hipLaunchKernelGGL((ffn_f32_kernel<2>), grid, dim3(256), 0, stream, static_cast<const float*>(in), segs, wp,
                       wp + one, static_cast<float*>(out), N, K);
  else
    hipLaunchKernelGGL((ffn_f32_kernel<1>), grid, dim3(256), 0, stream, static_cast<const float*>(in), segs,
                       wp + 2 * one, wp + 2 * one, static_cast<float*>(out), N, K);
  return hipGetLastError();
}

// The plain layer: segment e = expert e's rows, offsets[e] .. offsets[e + 1].
hipError_t launch_ffn_stage(const moe_config& cfg, int stage, int T, const void* in, const int32_t* offsets,
                            const void* packed, void* out, hipStream_t stream) {
  const int A = T * cfg.k;
  // an expert gets at most one row per token: no segment of the plain layer holds more than T rows
  return launch_ffn_segments(cfg, stage, offsets, offsets + 1, nullptr, cfg.E, A, A, A, T, in, packed, out, stream);
}

}  // namespace moe
