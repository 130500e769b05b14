// Internal declarations shared by the translation units of the MoE library (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "moe.h"

struct moe_ctx {
  moe_config cfg;
  char err[256];
};

namespace moe {

constexpr int kMaxExperts = 256;   // experts held one per thread of a 256-thread workgroup
constexpr int kMaxTopK = 64;       // one wavefront lane per pick

// Each launcher enqueues its kernels on `stream` and returns hipGetLastError().
hipError_t launch_route(const float* logits, int T, int E, int k, int32_t* topk_idx, float* topk_w,
                        int32_t* counts, int32_t* offsets, hipStream_t stream);
hipError_t launch_gate_route(const void* x, const float* w_router, int T, int d, int E, int k, int dtype, float* logits,
                             int32_t* topk_idx, float* topk_w, int32_t* counts, int32_t* offsets, hipStream_t stream);
// The gating GEMM with the top-k and the weights alone (one launch; T = 0: nothing), and the counting launch alone.
void launch_gate_topk_only(const void* x, const float* w_router, int T, int d, int E, int k, int dtype, float* logits,
                           int32_t* topk_idx, float* topk_w, hipStream_t stream);
void launch_count(const int32_t* topk_idx, int T, int E, int k, int32_t* counts, int32_t* offsets, hipStream_t stream);
// Counts, offsets and the dispatch pack from given picks in one launch when the batch is small enough
// (false: nothing launched).
bool launch_dispatch_from_picks_fused(const int32_t* topk_idx, const void* x, int T, int E, int k, int row_bytes,
                                      int32_t* counts, int32_t* offsets, void* xp, int32_t* pos, int32_t* src,
                                      hipStream_t stream);
// Routing + dispatch pack in one launch when the batch is small enough; returns false (nothing
// launched) when it is not, and the caller runs launch_route then launch_dispatch instead.
bool launch_route_dispatch_fused(const float* logits, const void* x, int T, int E, int k, int row_bytes,
                                 int32_t* topk_idx, float* topk_w, int32_t* counts, int32_t* offsets, void* xp,
                                 int32_t* pos, int32_t* src, hipStream_t stream);
hipError_t launch_dispatch(const void* x, const int32_t* topk_idx, const int32_t* offsets, int T, int E, int k,
                           int row_bytes, void* xp, int32_t* pos, int32_t* src, hipStream_t stream);
hipError_t launch_combine(const void* y, const int32_t* pos, const float* topk_w, int T, int k, int d,
                          int dtype, void* out, hipStream_t stream);
hipError_t launch_pack_weights(const moe_config& cfg, const void* w_gate, const void* w_up, const void* w_down,
                               void* packed, hipStream_t stream);
// stage 0: h = silu(xp Wg^T) .* (xp Wu^T)   (in = xp, out = h);  stage 1: y = h Wd^T   (in = h, out = y)
hipError_t launch_ffn_stage(const moe_config& cfg, int stage, int T, const void* in, const int32_t* offsets,
                            const void* packed, void* out, hipStream_t stream);
// The same two stages over explicit row segments: rows [seg_begin[s], seg_end[s]) use the weights of
// expert seg_expert[s] (nullptr: expert s). rows_bound >= the rows of all segments together (sizes the
// grid), rows_hint = their expected number, rows_cap = rows in `in` and `out`, seg_rows_max >= the rows of
// the largest segment (a launch whose segments cannot exceed 128 rows needs one kernel only).
hipError_t launch_ffn_segments(const moe_config& cfg, int stage, const int32_t* seg_begin, const int32_t* seg_end,
                               const int32_t* seg_expert, int n_segs, int rows_bound, int rows_hint, int rows_cap,
                               int seg_rows_max, const void* in, const void* packed, void* out, hipStream_t stream);
// Which bf16 GEMM kernel a launch of `stage` over n_segs segments runs (see launch_ffn_segments): true = streaming.
bool ffn_picks_streaming(const moe_config& cfg, int stage, int n_segs, int rows_hint, int seg_rows_max);
hipError_t launch_slot_segments(const int32_t* slot_expert, const int32_t* slot_copy, const int32_t* replicas,
                                const int32_t* offsets, int n_slots, int E, int32_t* seg_begin, int32_t* seg_end,
                                hipStream_t stream);
size_t packed_weight_bytes(const moe_config& cfg);
// Roofline probes: a streaming read of `bytes` (rounded down to whole loads: probe_stream_read_bytes) and
// `iters` x 16 MFMAs per wavefront from registers on `workgroups` x 4 wavefronts.
hipError_t launch_probe_stream_read(const void* buf, size_t bytes, void* sink, hipStream_t stream);
size_t probe_stream_read_bytes(size_t bytes);
hipError_t launch_probe_mfma(const void* operands, int iters, int workgroups, void* sink, hipStream_t stream);

}  // namespace moe
