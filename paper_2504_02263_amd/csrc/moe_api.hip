// C ABI entry points: argument validation on the host, then the kernel launchers.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>
#include <mutex>
#include <new>
#include "moe_internal.h"

// Workspace of moe_expert_ffn_static: the intermediate h[A, f] of the two-stage expert FFN, held in
// the library's own device image so that the call allocates nothing. Every GPU the library runs on
// holds its own copy of this array, at its own address, until the process ends. In host code the
// name below is only a handle for hipGetSymbolAddress; kernels are given the address it returns.
static __device__ __align__(256) unsigned char scratch[MOE_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on each GPU, once resolved

// Device address of `scratch` on the current device (resolved once per device, with that device
// current). Allocates nothing: the array is part of the loaded code object.
hipError_t static_scratch(void** out) {
  int dev = -1;
  hipError_t err = hipGetDevice(&dev);
  if (err != hipSuccess) return err;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (err != hipSuccess) return err;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

moe_status fail(moe_ctx* ctx, moe_status s, const char* fmt, ...) {
  if (ctx) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
    va_end(ap);
  }
  return s;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

moe_status check_config(const moe_config* c, const char** why) {
  *why = "";
  if (c->T_max < 0 || c->d <= 0 || c->f <= 0 || c->E <= 0 || c->k <= 0) {
    *why = "T_max, d, f, E, k must be positive (T_max may be 0)";
    return MOE_ERR_INVALID_ARG;
  }
  if (c->k > c->E) { *why = "k > E"; return MOE_ERR_INVALID_ARG; }
  if (c->dtype != MOE_F32 && c->dtype != MOE_BF16) { *why = "unknown dtype"; return MOE_ERR_INVALID_ARG; }
  if (!(c->load_skew == 0.f || (c->load_skew >= 1.f && c->load_skew <= 1e6f))) {
    *why = "load_skew must be 0 (unknown) or a finite value >= 1";
    return MOE_ERR_INVALID_ARG;
  }
  if (c->E > moe::kMaxExperts) { *why = "E > 256"; return MOE_ERR_UNSUPPORTED; }
  if (c->k > moe::kMaxTopK) { *why = "k > 64"; return MOE_ERR_UNSUPPORTED; }
  if (c->d % 128 || c->f % 128) { *why = "d and f must be multiples of 128"; return MOE_ERR_UNSUPPORTED; }
  // Assignments per call. Counting (one workgroup) and ranking (at most 1024 workgroups, each recounting what
  // lies before its share) are linear in T*k; beyond 4 M assignments a batch should be split by the caller.
  if ((int64_t)c->T_max * c->k > (int64_t)1 << 22) { *why = "T_max * k > 2^22"; return MOE_ERR_UNSUPPORTED; }
  if ((int64_t)c->E * c->d * c->f > (int64_t)1 << 36) { *why = "E*d*f too large"; return MOE_ERR_UNSUPPORTED; }
  return MOE_OK;
}

// Common per-call checks; `ptrs` are all the tensor pointers of the call.
moe_status check_call(moe_ctx* ctx, const char* fn, int32_t T, const void* const* ptrs, int n) {
  if (!ctx) return MOE_ERR_INVALID_ARG;
  ctx->err[0] = 0;
  if (T < 0 || T > ctx->cfg.T_max)
    return fail(ctx, MOE_ERR_INVALID_ARG, "%s: T = %d outside [0, T_max = %d]", fn, T, ctx->cfg.T_max);
  for (int i = 0; i < n; ++i) {
    if (!ptrs[i]) return fail(ctx, MOE_ERR_INVALID_ARG, "%s: tensor pointer %d is null", fn, i);
    if (!aligned16(ptrs[i])) return fail(ctx, MOE_ERR_INVALID_ARG, "%s: tensor pointer %d is not 16-byte aligned", fn, i);
  }
  return MOE_OK;
}

moe_status finish(moe_ctx* ctx, const char* fn, hipError_t err) {
  if (err == hipSuccess) return MOE_OK;
  return fail(ctx, MOE_ERR_HIP, "%s: %s", fn, hipGetErrorString(err));
}

int elem_bytes(const moe_ctx* ctx) { return ctx->cfg.dtype == MOE_BF16 ? 2 : 4; }

}  // namespace

extern "C" {

moe_status moe_create(const moe_config* cfg, moe_ctx** out) {
  if (!cfg || !out) return MOE_ERR_INVALID_ARG;
  *out = nullptr;
  const char* why;
  const moe_status s = check_config(cfg, &why);
  if (s != MOE_OK) return s;
  moe_ctx* ctx = new (std::nothrow) moe_ctx;
  if (!ctx) return MOE_ERR_INVALID_ARG;
  ctx->cfg = *cfg;
  ctx->err[0] = 0;
  // Where a GPU is present, find the static workspace of moe_expert_ffn_static on the current device
  // now, so that the hot call has nothing left to set up. Best effort: a host without a GPU can still
  // create contexts (argument checks, the planner), and the hot call resolves it on first use otherwise.
  int n_dev = 0;
  if (hipGetDeviceCount(&n_dev) == hipSuccess && n_dev > 0) {
    void* p = nullptr;
    (void)static_scratch(&p);
  }
  (void)hipGetLastError();
  *out = ctx;
  return MOE_OK;
}

void moe_destroy(moe_ctx* ctx) { delete ctx; }

const char* moe_last_error(const moe_ctx* ctx) { return ctx ? ctx->err : "null context"; }

const char* moe_status_string(moe_status s) {
  switch (s) {
    case MOE_OK: return "MOE_OK";
    case MOE_ERR_INVALID_ARG: return "MOE_ERR_INVALID_ARG";
    case MOE_ERR_UNSUPPORTED: return "MOE_ERR_UNSUPPORTED";
    case MOE_ERR_HIP: return "MOE_ERR_HIP";
  }
  return "unknown moe_status";
}

const char* moe_ffn_kernel_name(const moe_ctx* ctx, int32_t T, int32_t stage) {
  if (!ctx || T < 0 || (stage != 0 && stage != 1)) return "";
  if (ctx->cfg.dtype != MOE_BF16) return "f32";
  const int A = T * ctx->cfg.k;
  return moe::ffn_picks_streaming(ctx->cfg, stage, ctx->cfg.E, A, T) ? "streaming" : "large-batch";
}

size_t moe_packed_weight_bytes(const moe_config* cfg) {
  const char* why;
  if (!cfg || check_config(cfg, &why) != MOE_OK) return 0;
  return moe::packed_weight_bytes(*cfg);
}

moe_status moe_pack_weights(moe_ctx* ctx, const void* w_gate, const void* w_up, const void* w_down, void* packed,
                            void* stream) {
  const void* ptrs[] = {w_gate, w_up, w_down, packed};
  const moe_status s = check_call(ctx, "moe_pack_weights", 0, ptrs, 4);
  if (s != MOE_OK) return s;
  return finish(ctx, "moe_pack_weights",
                moe::launch_pack_weights(ctx->cfg, w_gate, w_up, w_down, packed, static_cast<hipStream_t>(stream)));
}

moe_status moe_route(moe_ctx* ctx, int32_t T, const float* logits, int32_t* topk_idx, float* topk_w, int32_t* counts,
                     int32_t* offsets, void* stream) {
  const void* ptrs[] = {logits, topk_idx, topk_w, counts, offsets};
  const moe_status s = check_call(ctx, "moe_route", T, ptrs, 5);
  if (s != MOE_OK) return s;
  return finish(ctx, "moe_route",
                moe::launch_route(logits, T, ctx->cfg.E, ctx->cfg.k, topk_idx, topk_w, counts, offsets,
                                  static_cast<hipStream_t>(stream)));
}

moe_status moe_gate_route(moe_ctx* ctx, int32_t T, const void* x, const float* w_router, float* logits,
                          int32_t* topk_idx, float* topk_w, int32_t* counts, int32_t* offsets, void* stream) {
  const void* ptrs[] = {x, w_router, topk_idx, topk_w, counts, offsets};
  const moe_status s = check_call(ctx, "moe_gate_route", T, ptrs, 6);
  if (s != MOE_OK) return s;
  if (logits && !aligned16(logits)) return fail(ctx, MOE_ERR_INVALID_ARG, "moe_gate_route: logits is not 16-byte aligned");
  return finish(ctx, "moe_gate_route",
                moe::launch_gate_route(x, w_router, T, ctx->cfg.d, ctx->cfg.E, ctx->cfg.k, ctx->cfg.dtype, logits,
                                       topk_idx, topk_w, counts, offsets, static_cast<hipStream_t>(stream)));
}

moe_status moe_dispatch(moe_ctx* ctx, int32_t T, const void* x, const int32_t* topk_idx, const int32_t* offsets,
                        void* xp, int32_t* pos, int32_t* src, void* stream) {
  const void* ptrs[] = {x, topk_idx, offsets, xp, pos, src};
  const moe_status s = check_call(ctx, "moe_dispatch", T, ptrs, 6);
  if (s != MOE_OK) return s;
  return finish(ctx, "moe_dispatch",
                moe::launch_dispatch(x, topk_idx, offsets, T, ctx->cfg.E, ctx->cfg.k, ctx->cfg.d * elem_bytes(ctx), xp,
                                     pos, src, static_cast<hipStream_t>(stream)));
}

moe_status moe_route_dispatch(moe_ctx* ctx, int32_t T, const float* logits, const void* x, int32_t* topk_idx,
                              float* topk_w, int32_t* counts, int32_t* offsets, void* xp, int32_t* pos, int32_t* src,
                              void* stream) {
  const void* ptrs[] = {logits, x, topk_idx, topk_w, counts, offsets, xp, pos, src};
  const moe_status s = check_call(ctx, "moe_route_dispatch", T, ptrs, 9);
  if (s != MOE_OK) return s;
  const moe_config& c = ctx->cfg;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (moe::launch_route_dispatch_fused(logits, x, T, c.E, c.k, c.d * elem_bytes(ctx), topk_idx, topk_w, counts, offsets,
                                       xp, pos, src, st))
    return finish(ctx, "moe_route_dispatch", hipGetLastError());
  hipError_t err = moe::launch_route(logits, T, c.E, c.k, topk_idx, topk_w, counts, offsets, st);
  if (err == hipSuccess)
    err = moe::launch_dispatch(x, topk_idx, offsets, T, c.E, c.k, c.d * elem_bytes(ctx), xp, pos, src, st);
  return finish(ctx, "moe_route_dispatch", err);
}

moe_status moe_gate_route_dispatch(moe_ctx* ctx, int32_t T, const void* x, const float* w_router, float* logits,
                                   int32_t* topk_idx, float* topk_w, int32_t* counts, int32_t* offsets, void* xp,
                                   int32_t* pos, int32_t* src, void* stream) {
  const void* ptrs[] = {x, w_router, topk_idx, topk_w, counts, offsets, xp, pos, src};
  const moe_status s = check_call(ctx, "moe_gate_route_dispatch", T, ptrs, 9);
  if (s != MOE_OK) return s;
  if (logits && !aligned16(logits))
    return fail(ctx, MOE_ERR_INVALID_ARG, "moe_gate_route_dispatch: logits is not 16-byte aligned");
  const moe_config& c = ctx->cfg;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int row_bytes = c.d * elem_bytes(ctx);
  moe::launch_gate_topk_only(x, w_router, T, c.d, c.E, c.k, c.dtype, logits, topk_idx, topk_w, st);
  hipError_t err = hipGetLastError();
  if (err == hipSuccess &&
      !moe::launch_dispatch_from_picks_fused(topk_idx, x, T, c.E, c.k, row_bytes, counts, offsets, xp, pos, src, st)) {
    moe::launch_count(topk_idx, T, c.E, c.k, counts, offsets, st);
    err = moe::launch_dispatch(x, topk_idx, offsets, T, c.E, c.k, row_bytes, xp, pos, src, st);
  }
  if (err == hipSuccess) err = hipGetLastError();
  return finish(ctx, "moe_gate_route_dispatch", err);
}

moe_status moe_ffn_input(moe_ctx* ctx, int32_t T, const void* xp, const int32_t* offsets, const void* packed_w, void* h,
                         void* stream) {
  const void* ptrs[] = {xp, offsets, packed_w, h};
  const moe_status s = check_call(ctx, "moe_ffn_input", T, ptrs, 4);
  if (s != MOE_OK) return s;
  return finish(ctx, "moe_ffn_input",
                moe::launch_ffn_stage(ctx->cfg, 0, T, xp, offsets, packed_w, h, static_cast<hipStream_t>(stream)));
}

moe_status moe_ffn_output(moe_ctx* ctx, int32_t T, const void* h, const int32_t* offsets, const void* packed_w, void* y,
                          void* stream) {
  const void* ptrs[] = {h, offsets, packed_w, y};
  const moe_status s = check_call(ctx, "moe_ffn_output", T, ptrs, 4);
  if (s != MOE_OK) return s;
  return finish(ctx, "moe_ffn_output",
                moe::launch_ffn_stage(ctx->cfg, 1, T, h, offsets, packed_w, y, static_cast<hipStream_t>(stream)));
}

moe_status moe_expert_ffn(moe_ctx* ctx, int32_t T, const void* xp, const int32_t* offsets, const void* packed_w,
                          void* h_ws, void* y, void* stream) {
  const void* ptrs[] = {xp, offsets, packed_w, h_ws, y};
  const moe_status s = check_call(ctx, "moe_expert_ffn", T, ptrs, 5);
  if (s != MOE_OK) return s;
  hipError_t err = moe::launch_ffn_stage(ctx->cfg, 0, T, xp, offsets, packed_w, h_ws, static_cast<hipStream_t>(stream));
  if (err == hipSuccess)
    err = moe::launch_ffn_stage(ctx->cfg, 1, T, h_ws, offsets, packed_w, y, static_cast<hipStream_t>(stream));
  return finish(ctx, "moe_expert_ffn", err);
}

moe_status moe_expert_ffn_static(moe_ctx* ctx, int32_t T, const void* xp, const int32_t* offsets, const void* packed_w,
                                 void* y, void* stream) {
  const void* ptrs[] = {xp, offsets, packed_w, y};
  const moe_status s = check_call(ctx, "moe_expert_ffn_static", T, ptrs, 4);
  if (s != MOE_OK) return s;
  const size_t need = (size_t)T * ctx->cfg.k * ctx->cfg.f * elem_bytes(ctx);
  if (need > (size_t)MOE_STATIC_SCRATCH_BYTES)
    return fail(ctx, MOE_ERR_UNSUPPORTED,
                "moe_expert_ffn_static: h[T*k, f] needs %zu bytes, the static workspace holds %zu; use moe_expert_ffn",
                need, (size_t)MOE_STATIC_SCRATCH_BYTES);
  if (T == 0) return MOE_OK;
  void* h_ws = nullptr;
  hipError_t err = static_scratch(&h_ws);
  if (err == hipSuccess)
    err = moe::launch_ffn_stage(ctx->cfg, 0, T, xp, offsets, packed_w, h_ws, static_cast<hipStream_t>(stream));
  if (err == hipSuccess)
    err = moe::launch_ffn_stage(ctx->cfg, 1, T, h_ws, offsets, packed_w, y, static_cast<hipStream_t>(stream));
  return finish(ctx, "moe_expert_ffn_static", err);
}

moe_status moe_slot_segments(moe_ctx* ctx, int32_t n_slots, const int32_t* slot_expert, const int32_t* slot_copy,
                             const int32_t* replicas, const int32_t* offsets, int32_t* seg_begin, int32_t* seg_end,
                             void* stream) {
  const void* ptrs[] = {slot_expert, slot_copy, replicas, offsets, seg_begin, seg_end};
  const moe_status s = check_call(ctx, "moe_slot_segments", 0, ptrs, 6);
  if (s != MOE_OK) return s;
  if (n_slots < 0 || n_slots > moe::kMaxExperts)
    return fail(ctx, MOE_ERR_INVALID_ARG, "moe_slot_segments: n_slots = %d outside [0, %d]", n_slots, moe::kMaxExperts);
  return finish(ctx, "moe_slot_segments",
                moe::launch_slot_segments(slot_expert, slot_copy, replicas, offsets, n_slots, ctx->cfg.E, seg_begin,
                                          seg_end, static_cast<hipStream_t>(stream)));
}

moe_status moe_expert_ffn_segments(moe_ctx* ctx, int32_t T, int32_t n_segs, int32_t rows_hint, const void* xp,
                                   const int32_t* seg_begin, const int32_t* seg_end, const int32_t* seg_expert,
                                   const void* packed_w, void* h_ws, void* y, void* stream) {
  const void* ptrs[] = {xp, seg_begin, seg_end, seg_expert, packed_w, h_ws, y};
  const moe_status s = check_call(ctx, "moe_expert_ffn_segments", T, ptrs, 7);
  if (s != MOE_OK) return s;
  if (n_segs < 0 || n_segs > moe::kMaxExperts)
    return fail(ctx, MOE_ERR_INVALID_ARG, "moe_expert_ffn_segments: n_segs = %d outside [0, %d]", n_segs,
                moe::kMaxExperts);
  const int A = T * ctx->cfg.k;
  const int hint = rows_hint > 0 ? (rows_hint < A ? rows_hint : A) : A;
  hipError_t err = moe::launch_ffn_segments(ctx->cfg, 0, seg_begin, seg_end, seg_expert, n_segs, A, hint, A, A, xp,
                                            packed_w, h_ws, static_cast<hipStream_t>(stream));
  if (err == hipSuccess)
    err = moe::launch_ffn_segments(ctx->cfg, 1, seg_begin, seg_end, seg_expert, n_segs, A, hint, A, A, h_ws, packed_w,
                                   y, static_cast<hipStream_t>(stream));
  return finish(ctx, "moe_expert_ffn_segments", err);
}

moe_status moe_probe_stream_read(moe_ctx* ctx, const void* buf, size_t bytes, void* sink, size_t* bytes_read,
                                 void* stream) {
  const void* ptrs[] = {buf, sink};
  const moe_status s = check_call(ctx, "moe_probe_stream_read", 0, ptrs, 2);
  if (s != MOE_OK) return s;
  if (bytes_read) *bytes_read = moe::probe_stream_read_bytes(bytes);
  return finish(ctx, "moe_probe_stream_read",
                moe::launch_probe_stream_read(buf, bytes, sink, static_cast<hipStream_t>(stream)));
}

moe_status moe_probe_mfma(moe_ctx* ctx, const void* operands, int32_t iters, int32_t workgroups, void* sink,
                          double* flops, void* stream) {
  const void* ptrs[] = {operands, sink};
  const moe_status s = check_call(ctx, "moe_probe_mfma", 0, ptrs, 2);
  if (s != MOE_OK) return s;
  if (iters < 0 || iters > (1 << 24) || workgroups < 0 || workgroups > (1 << 20))
    return fail(ctx, MOE_ERR_INVALID_ARG, "moe_probe_mfma: iters = %d or workgroups = %d out of range", iters, workgroups);
  if (flops) *flops = (double)workgroups * 4.0 * iters * 16.0 * (2.0 * 32 * 32 * 16);
  return finish(ctx, "moe_probe_mfma",
                moe::launch_probe_mfma(operands, iters, workgroups, sink, static_cast<hipStream_t>(stream)));
}

moe_status moe_combine(moe_ctx* ctx, int32_t T, const void* y, const int32_t* pos, const float* topk_w, void* out,
                       void* stream) {
  const void* ptrs[] = {y, pos, topk_w, out};
  const moe_status s = check_call(ctx, "moe_combine", T, ptrs, 4);
  if (s != MOE_OK) return s;
  return finish(ctx, "moe_combine",
                moe::launch_combine(y, pos, topk_w, T, ctx->cfg.k, ctx->cfg.d, ctx->cfg.dtype, out,
                                    static_cast<hipStream_t>(stream)));
}

}  // extern "C"
