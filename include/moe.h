/*
 * moe.h: C ABI of the expert-side hot path of one Mixture-of-Experts layer on one MI355X (gfx950).
 *
 * The four hot calls follow the paper's statement of the MoE layer (Section 2.2: gating scores,
 * top-k routing, expert FFNs, weighted sum of the selected experts' outputs), the steps its
 * implementation section lists for the fused gating kernel (Section 6 "Fused kernels": top-k
 * selection, number of tokens per expert, normalised token weights, scatter to experts) and the
 * two expert GEMMs of its GEMM table (Section 4.2, Table 3: "FFN Input", "FFN Output"):
 *
 *     moe_route -> moe_dispatch -> moe_expert_ffn -> moe_combine
 *
 * Conventions for every call below
 *   - Notation: T tokens, d hidden size (paper: h), f expert intermediate size (paper: h'),
 *     E experts, k experts per token (paper: K), A = T*k assignments.
 *   - Every tensor pointer is a DEVICE pointer owned by the caller, row-major and contiguous,
 *     16-byte aligned (the exceptions say so: moe_plan_experts is a host function, and the two
 *     probes return a scalar through a host pointer). The library allocates no device memory and keeps no device state: each
 *     call is a pure function of its arguments, so calls on different streams never share
 *     anything but their arguments.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream). All work is enqueued
 *     on it; no call synchronises the device or copies anything to the host. The per-expert
 *     sizes stay on the device (`offsets` is read by the kernels).
 *   - x, xp, h, y, out and the expert weights share cfg.dtype (float32 or bfloat16). Router
 *     logits and token weights are always float32; index arrays are int32.
 *   - Errors: argument errors (null pointer, T < 0, T > T_max, misaligned pointer) are detected
 *     on the host before anything is launched and leave the outputs untouched; a failed launch
 *     returns MOE_ERR_HIP. moe_last_error() gives a message for the last failure on that ctx.
 *     T == 0 is MOE_OK; moe_route then still writes counts = 0 and offsets = 0.
 *   - A moe_ctx is not thread-safe; use one per host thread.
 */
#ifndef MOE_H
#define MOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct moe_ctx moe_ctx; /* opaque; host memory only */

typedef enum {
  MOE_OK = 0,
  MOE_ERR_INVALID_ARG = 1,
  MOE_ERR_UNSUPPORTED = 2, /* shape or dtype outside what the kernels are built for */
  MOE_ERR_HIP = 3          /* a HIP call or launch failed */
} moe_status;

typedef enum { MOE_F32 = 0, MOE_BF16 = 1 } moe_dtype;

typedef struct {
  int32_t T_max; /* largest T any call will be given; T_max * k <= 2^22 */
  int32_t d;     /* hidden size; multiple of 128 */
  int32_t f;     /* expert intermediate size; multiple of 128 */
  int32_t E;     /* experts, 1..256 */
  int32_t k;     /* experts per token, 1..min(E, 64) */
  int32_t dtype; /* moe_dtype */
  /* Optional hint, 0 = unknown (treated as 1): how many times the mean number of rows the most popular
   * experts are expected to get (a serving engine that tracks expert popularity, as the paper's load
   * balancer does, Section 6 "Load balance", knows this; per-batch counts never leave the device). It only
   * helps pick the GEMM kernel for a launch; results never depend on it. Must be 0 or a finite value >= 1. */
  float load_skew;
} moe_config;

/* Validate cfg and build a context (host memory only). MOE_ERR_INVALID_ARG for a null
 * pointer or non-positive sizes, MOE_ERR_UNSUPPORTED for sizes outside the limits above. */
moe_status moe_create(const moe_config* cfg, moe_ctx** out);
void moe_destroy(moe_ctx* ctx);
/* Message of the last failed call on ctx ("" if none). Valid until the next call on ctx. */
const char* moe_last_error(const moe_ctx* ctx);
const char* moe_status_string(moe_status s);

/* Name of the GEMM kernel moe_ffn_input (stage 0) or moe_ffn_output (stage 1) launches for a batch of T tokens on
 * this context: "streaming" (128-row tiles, weights read once, for decode-sized per-expert batches; Section 2.3's
 * memory-bound side), "large-batch" (256-row tiles, matrix-core bound side) or "f32". A host-side query for
 * reports; "" for bad arguments. */
const char* moe_ffn_kernel_name(const moe_ctx* ctx, int32_t T, int32_t stage);

/* Bytes of the packed expert-weight buffer moe_pack_weights writes (0 if cfg is invalid). */
size_t moe_packed_weight_bytes(const moe_config* cfg);

/*
 * One-time weight pre-pack (expert weights are static while serving). Canonical layout in:
 *   w_gate[E, f, d], w_up[E, f, d], w_down[E, d, f]     (each expert's matrix is [out, in],
 * so Table 3's (h, h') "FFN Input" parameter is used as x * W^T). Out: `packed`, the layout the
 * FFN kernels stream (bf16: tiles in matrix-core operand order; f32: plain concatenation).
 * `packed` must hold moe_packed_weight_bytes(cfg) bytes and must not overlap the inputs.
 */
moe_status moe_pack_weights(moe_ctx* ctx, const void* w_gate, const void* w_up, const void* w_down,
                            void* packed, void* stream);

/*
 * Routing (Section 2.2; Section 6 "Fused kernels"). In: logits[T, E] float32.
 * Out: topk_idx[T, k]  the k experts with the largest logits, largest first; equal logits are
 *                      ordered by ascending expert index (so ties go to the lower index)
 *      topk_w[T, k]    softmax over those k logits (float32)
 *      counts[E]       assignments per expert
 *      offsets[E + 1]  exclusive prefix sum of counts; offsets[E] = T*k
 * NaN logits rank as -inf. Indices, counts and offsets are exact integers.
 */
moe_status moe_route(moe_ctx* ctx, int32_t T, const float* logits, int32_t* topk_idx, float* topk_w,
                     int32_t* counts, int32_t* offsets, void* stream);

/*
 * Gating GEMM fused with the routing (Section 2.2: the gate scores are a matrix multiplication of
 * each token's embedding with the gating parameters; Section 6 "Fused kernels": the paper fuses the
 * top-k, the per-expert counts and the normalised weights with the gating computation).
 * In: x[T, d] (cfg.dtype), w_router[E, d] float32.
 *     logits[t, e] = sum_c x[t, c] * w_router[e, c], accumulated in float32
 * Out: logits[T, E] float32 (may be NULL: then the scores never leave the chip), and topk_idx,
 * topk_w, counts, offsets exactly as moe_route would give on those logits. Two launches instead
 * of the three of a separate gate GEMM followed by moe_route.
 */
moe_status moe_gate_route(moe_ctx* ctx, int32_t T, const void* x, const float* w_router, float* logits,
                          int32_t* topk_idx, float* topk_w, int32_t* counts, int32_t* offsets, void* stream);

/*
 * Dispatch pack (Section 2.2: each token goes to the experts its routing picked; Section 6 "Fused
 * kernels": the scatter step): stable counting sort of the A assignments by expert.
 * In: x[T, d], topk_idx[T, k], offsets[E + 1] (as written by moe_route).
 * Out: xp[A, d]   expert-contiguous copy of the tokens: rows offsets[e]..offsets[e+1]-1 belong
 *                 to expert e, in ascending flat assignment order t*k + j
 *      pos[T, k]  row of assignment (t, j)
 *      src[A]     flat assignment index t*k + j that owns row r  (pos and src are inverse
 *                 permutations of each other)
 * Entries of topk_idx outside [0, E) are skipped (their pos/src/xp entries stay unwritten).
 */
moe_status moe_dispatch(moe_ctx* ctx, int32_t T, const void* x, const int32_t* topk_idx,
                        const int32_t* offsets, void* xp, int32_t* pos, int32_t* src, void* stream);

/*
 * moe_route followed by moe_dispatch as one call (Section 6 "Fused kernels": the paper fuses the
 * top-k, the per-expert counts, the normalised weights and the scatter because each is a small
 * memory-bound step). Same arguments, same outputs bit for bit as the two calls. For decode-sized
 * batches (T <= 512, T*k <= 2048 and T*E <= 8192) everything runs in a single launch; larger
 * batches run the four kernels of the two calls.
 */
moe_status moe_route_dispatch(moe_ctx* ctx, int32_t T, const float* logits, const void* x, int32_t* topk_idx,
                              float* topk_w, int32_t* counts, int32_t* offsets, void* xp, int32_t* pos, int32_t* src,
                              void* stream);

/*
 * The whole step in front of the experts as one call, from the token embeddings to the packed rows:
 * gating GEMM, top-k, normalised weights, per-expert counts and the scatter (Section 6 "Fused kernels" lists
 * exactly these as one fused kernel). Arguments and outputs as moe_gate_route followed by moe_dispatch, bit
 * for bit. Two launches for decode-sized batches (T <= 512 and T*k <= 2048): the gating kernel (GEMM + top-k
 * + weights, one workgroup per block of tokens), then one kernel that counts, scans, ranks and copies the
 * rows. A single launch would have every workgroup read all of x for the gating GEMM (there is no grid-wide
 * barrier to share its result), which costs more than the second launch; the picks it hands over are
 * T*k integers that stay in L2. Larger batches run the four kernels of the two calls.
 */
moe_status moe_gate_route_dispatch(moe_ctx* ctx, int32_t T, const void* x, const float* w_router, float* logits,
                                   int32_t* topk_idx, float* topk_w, int32_t* counts, int32_t* offsets, void* xp,
                                   int32_t* pos, int32_t* src, void* stream);

/*
 * Expert FFN as a grouped SwiGLU GEMM (Section 4.2, Table 3; tensor-parallel degree 1):
 * for every expert e and row r in [offsets[e], offsets[e+1]):
 *     h[r, :] = silu(xp[r, :] * W_gate_e^T) .* (xp[r, :] * W_up_e^T)      ("FFN Input", fused)
 *     y[r, :] = h[r, :] * W_down_e^T                                       ("FFN Output")
 * In: xp[A, d], offsets[E + 1], packed weights from moe_pack_weights.
 * Workspace: h_ws[A, f] in cfg.dtype (caller-owned; holds h afterwards). Out: y[A, d].
 * bf16: products accumulate in float32; h and y are rounded to bf16 (nearest-even) when stored.
 * Experts with no rows cost nothing (their weights are not read).
 */
moe_status moe_expert_ffn(moe_ctx* ctx, int32_t T, const void* xp, const int32_t* offsets,
                          const void* packed_w, void* h_ws, void* y, void* stream);

/*
 * moe_expert_ffn without a caller-provided workspace, for callers that cannot allocate device
 * memory: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc. The
 * intermediate h[T*k, f] lives in a static array of MOE_STATIC_SCRATCH_BYTES inside the library's
 * device image (every GPU the library runs on holds its own copy until the process ends); the call
 * allocates and frees nothing. Same kernels and the same y, bit for bit, as moe_expert_ffn.
 * MOE_ERR_UNSUPPORTED (nothing launched, y untouched) if T*k*f*sizeof(element) exceeds
 * MOE_STATIC_SCRATCH_BYTES. All calls on one GPU share that GPU's array: calls that overlap in time
 * on one GPU (different streams, or different contexts) race on h; issue them on one stream or
 * order them with events. Nothing in the array has to start at zero (every row of h that is read
 * was written by the same call before).
 */
#define MOE_STATIC_SCRATCH_BYTES (64u << 20)
moe_status moe_expert_ffn_static(moe_ctx* ctx, int32_t T, const void* xp, const int32_t* offsets,
                                 const void* packed_w, void* y, void* stream);

/*
 * The two GEMM stages of moe_expert_ffn as separate calls, named as in Table 3 (same kernels,
 * same results; moe_expert_ffn is moe_ffn_input followed by moe_ffn_output):
 *   moe_ffn_input :  h[A, f] = silu(xp * W_gate^T) .* (xp * W_up^T)     reads xp[A, d]
 *   moe_ffn_output:  y[A, d] = h * W_down^T                              reads h[A, f]
 * Both take the same packed weight buffer and offsets[E + 1].
 */
moe_status moe_ffn_input(moe_ctx* ctx, int32_t T, const void* xp, const int32_t* offsets,
                         const void* packed_w, void* h, void* stream);
moe_status moe_ffn_output(moe_ctx* ctx, int32_t T, const void* h, const int32_t* offsets,
                          const void* packed_w, void* y, void* stream);

/*
 * Expert plan with on-device redundancy (Section 6, "Load balance"). HOST function: every pointer
 * is host memory, nothing touches the GPU. Spread M experts over N expert nodes, each with room
 * for S expert copies (N*S >= M), so that the largest node cost
 *     C_j = sum_i x[i][j] * max(a[i], K)        (x[i][j] = fraction of expert i served by node j)
 * is small: a[i] = cost of computing expert i's active tokens over the last period, K = lowest
 * cost a cold expert can have. The paper solves this greedily and gives no steps (Section 6 "Load balance"); the steps
 * taken are: (1) while spare slots remain, the expert with the largest per-copy share
 * max(a[i], K) / replicas[i] gets one more copy (at most one per node), unless that share is already
 * no more than the mean node cost; (2) the copies of an expert split it equally (x = 1 / replicas[i]);
 * (3) copies, largest share first, go to the cheapest node that has a free slot and no copy of that
 * expert. Ties go to the lower expert / copy / node index; arithmetic is IEEE double, left to right.
 * In:  a[M], K.   Out: replicas[M]; slot_expert[N*S] and slot_copy[N*S] (node j owns entries
 *      j*S .. j*S+S-1, filled in placement order, slot_expert = -1 for an empty slot); node_cost[N].
 * MOE_ERR_INVALID_ARG for null pointers, sizes < 1, N*S < M or a NaN cost; MOE_ERR_UNSUPPORTED if
 * the placement runs out of nodes that lack the expert (outputs are then unspecified).
 */
moe_status moe_plan_experts(int32_t M, int32_t N, int32_t S, const double* a, double K, int32_t* replicas,
                            int32_t* slot_expert, int32_t* slot_copy, double* node_cost);

/*
 * Row ranges of expert copies (Section 6, "Load balance": a popular expert's tokens are shared
 * between its copies). Copy r of the R = replicas[e] copies of expert e takes the r-th of R
 * consecutive parts of expert e's rows in the expert-contiguous layout:
 *     seg_begin[s] = offsets[e] + floor(r * c / R),  seg_end[s] = offsets[e] + floor((r + 1) * c / R),
 *     e = slot_expert[s], r = slot_copy[s], c = offsets[e + 1] - offsets[e].
 * In (device): slot_expert[n_slots], slot_copy[n_slots], replicas[E], offsets[E + 1]; n_slots <= 256.
 * Out (device): seg_begin[n_slots], seg_end[n_slots]. A slot naming no expert in [0, E), or a copy
 * number outside [0, R), gets the empty range [0, 0).
 */
moe_status moe_slot_segments(moe_ctx* ctx, int32_t n_slots, const int32_t* slot_expert, const int32_t* slot_copy,
                             const int32_t* replicas, const int32_t* offsets, int32_t* seg_begin, int32_t* seg_end,
                             void* stream);

/*
 * moe_expert_ffn over explicit row segments: what one expert node runs under an expert plan
 * (Section 6, "Load balance"; the GEMMs are those of Section 4.2, Table 3). For every segment s and
 * row r in [seg_begin[s], seg_end[s]), with e = seg_expert[s]:
 *     h[r, :] = silu(xp[r, :] * W_gate_e^T) .* (xp[r, :] * W_up_e^T),   y[r, :] = h[r, :] * W_down_e^T
 * Rows outside every segment are not touched. Each row's result is the same bits moe_expert_ffn
 * gives that row, however the rows are cut into segments.
 * In (device): xp[T*k, d], seg_begin / seg_end / seg_expert[n_segs] (n_segs <= 256), packed weights.
 * T is the token count of the batch the rows come from: ranges are clipped to [0, T*k) and the
 * segments must be disjoint (together they then hold at most T*k rows). rows_hint = expected rows in
 * all segments together (only picks the tile shape; <= 0: T*k). A segment whose expert is outside
 * [0, E) is skipped. Workspace h_ws[T*k, f]; out y[T*k, d].
 */
moe_status moe_expert_ffn_segments(moe_ctx* ctx, int32_t T, int32_t n_segs, int32_t rows_hint, const void* xp,
                                   const int32_t* seg_begin, const int32_t* seg_end, const int32_t* seg_expert,
                                   const void* packed_w, void* h_ws, void* y, void* stream);

/*
 * Combine (Section 2.2: the layer output is the weighted sum of the selected experts' outputs):
 *     out[t, :] = sum_{j = 0..k-1} topk_w[t, j] * y[pos[t, j], :]     (float32 sum, j ascending)
 * In: y[A, d], pos[T, k], topk_w[T, k]. Out: out[T, d] in cfg.dtype.
 * Entries of pos outside [0, A) contribute nothing.
 */
moe_status moe_combine(moe_ctx* ctx, int32_t T, const void* y, const int32_t* pos, const float* topk_w,
                       void* out, void* stream);

/*
 * Probes for the roofline's two denominators (Section 2.3: a GEMM is memory-bound below the ridge batch
 * F / B and compute-bound above it; B = memory bandwidth, F = peak compute). They compute no part of
 * the layer: a benchmark times them next to the layer's kernels to state what this chip reaches.
 *   moe_probe_stream_read: every wavefront reads its own contiguous share of buf[bytes] (device) with
 *     the non-temporal 16-byte loads of the weight stream; *bytes_read (host, may be NULL) receives
 *     the bytes actually read (bytes rounded down to whole loads per wavefront).
 *   moe_probe_mfma: `workgroups` x 4 wavefronts each issue iters x 16 v_mfma_f32_32x32x16_bf16 from
 *     registers; the operands are the first 2 KiB of `operands` (device; pass real weights: the
 *     matrix cores' clock under load depends on the bit patterns multiplied); *flops (host, may be
 *     NULL) receives the floating-point operations of the launch.
 * `sink` is 16 bytes of device memory the kernels may write. Both return after enqueueing.
 */
moe_status moe_probe_stream_read(moe_ctx* ctx, const void* buf, size_t bytes, void* sink, size_t* bytes_read,
                                 void* stream);
moe_status moe_probe_mfma(moe_ctx* ctx, const void* operands, int32_t iters, int32_t workgroups, void* sink,
                          double* flops, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_H */
