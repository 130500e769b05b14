// Dispatch pack: a stable counting sort of the A = T*k assignments by expert, then a row gather
// into the expert-contiguous buffer (paper Section 2.2: tokens are sent to their experts;
// Section 6 "Fused kernels": the scatter step). All integer work; results are exact.
#include "moe_internal.h"

namespace moe {
namespace {

constexpr int kRankBlock = 256;  // assignments ranked per workgroup

constexpr int kRankMaxBlocks = 1024;  // workgroups of the ranking kernel, at most

// Workgroup b ranks the `chunks` consecutive 256-assignment chunks [b * chunks, (b + 1) * chunks).
// Row of assignment i with expert e:
//   offsets[e] + #{i' < i : idx[i'] == e}
// The count splits into (assignments of e before the workgroup's first chunk) + (in its earlier chunks)
// + (in earlier wavefronts of the chunk) + (in earlier lanes of the same wavefront). The first term is
// recounted here from topk_idx itself, so the kernel needs no state from any other launch; the launcher
// gives a workgroup one chunk while that keeps the grid within kRankMaxBlocks workgroups and more beyond,
// so the recount costs at most kRankMaxBlocks / 2 passes over topk_idx however large the batch is.
__global__ __launch_bounds__(kRankBlock) void dispatch_rank_kernel(const int32_t* __restrict__ topk_idx,
                                                                   const int32_t* __restrict__ offsets, int A, int E,
                                                                   int chunks, int32_t* __restrict__ pos,
                                                                   int32_t* __restrict__ src) {
  __shared__ int before[kMaxExperts];      // assignments of e before the current chunk
  __shared__ int in_wave[4][kMaxExperts];  // assignments of e in each wavefront of the current chunk
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  before[tid] = 0;
  __syncthreads();

  const long long first = (long long)blockIdx.x * chunks * kRankBlock;  // multiple of 4: int4 loads stay aligned
  if (first >= A) return;  // uniform over the workgroup
  const int start = (int)first;
  for (int i = tid * 4; i < start; i += kRankBlock * 4) {
    const int4 q = *reinterpret_cast<const int4*>(topk_idx + i);
    if ((unsigned)q.x < (unsigned)E) atomicAdd(&before[q.x], 1);
    if ((unsigned)q.y < (unsigned)E) atomicAdd(&before[q.y], 1);
    if ((unsigned)q.z < (unsigned)E) atomicAdd(&before[q.z], 1);
    if ((unsigned)q.w < (unsigned)E) atomicAdd(&before[q.w], 1);
  }
  const unsigned long long below = (1ull << lane) - 1ull;
  for (int c = 0; c < chunks && start + c * kRankBlock < A; ++c) {
#pragma unroll
    for (int i = 0; i < 4; ++i) in_wave[i][tid] = 0;
    __syncthreads();  // also orders the updates of `before` (the recount, or the previous chunk) before the reads below
    const int i = start + c * kRankBlock + tid;
    int e = -1;
    if (i < A) {
      e = topk_idx[i];
      if ((unsigned)e >= (unsigned)E) e = -1;
    }
    // Rank among equal experts inside the wavefront, lanes in ascending order: peel one expert
    // value per round (the one held by the lowest lane still waiting).
    int rank = 0;
    unsigned long long todo = __ballot(e >= 0);
    while (todo) {
      const int leader = __ffsll((long long)todo) - 1;
      const int le = __shfl(e, leader);
      const unsigned long long same = __ballot(e == le);
      if (e == le) {
        rank = __popcll(same & below);
        if (lane == leader) in_wave[w][le] = __popcll(same);
      }
      todo &= ~same;
    }
    __syncthreads();
    if (e >= 0) {
      int r = offsets[e] + before[e] + rank;
      for (int ww = 0; ww < w; ++ww) r += in_wave[ww][e];
      if ((unsigned)r < (unsigned)A) {
        pos[i] = r;
        src[r] = i;
      }
    }
    __syncthreads();
    before[tid] += in_wave[0][tid] + in_wave[1][tid] + in_wave[2][tid] + in_wave[3][tid];
  }
}

// One wavefront per output row: xp[r, :] = x[src[r] / k, :], 16 bytes per lane per step.
__global__ __launch_bounds__(256) void dispatch_copy_kernel(const uint4* __restrict__ x,
                                                            const int32_t* __restrict__ src, int A, int T, int k,
                                                            int row_vecs, uint4* __restrict__ xp) {
  const int lane = threadIdx.x & 63;
  const int waves = gridDim.x * 4;
  for (int r = blockIdx.x * 4 + (threadIdx.x >> 6); r < A; r += waves) {
    const int t = src[r] / k;
    if ((unsigned)t >= (unsigned)T) continue;
    const uint4* in = x + (size_t)t * row_vecs;
    uint4* out = xp + (size_t)r * row_vecs;
    for (int c = lane; c < row_vecs; c += 64) out[c] = in[c];
  }
}

}  // namespace

hipError_t launch_dispatch(const void* x, const int32_t* topk_idx, const int32_t* offsets, int T, int E, int k,
                           int row_bytes, void* xp, int32_t* pos, int32_t* src, hipStream_t stream) {
  const int A = T * k;
  if (A == 0) return hipSuccess;
  const int n_chunks = (A + kRankBlock - 1) / kRankBlock;
  const int chunks = (n_chunks + kRankMaxBlocks - 1) / kRankMaxBlocks;  // per workgroup
  hipLaunchKernelGGL(dispatch_rank_kernel, dim3((n_chunks + chunks - 1) / chunks), dim3(kRankBlock), 0, stream,
                     topk_idx, offsets, A, E, chunks, pos, src);
  int blocks = (A + 3) / 4;
  if (blocks > 16384) blocks = 16384;
  hipLaunchKernelGGL(dispatch_copy_kernel, dim3(blocks), dim3(256), 0, stream, static_cast<const uint4*>(x), src, A,
                     T, k, row_bytes / 16, static_cast<uint4*>(xp));
  return hipGetLastError();
}

}  // namespace moe
