// Driver for the sanitizer build of the library's host code (tests/test_host_sanitizers.py): the planner on
// seeded instances and every entry point's argument checks, which return before anything is launched.
// Needs no GPU. Prints "host checks done" and exits 0 when every call returned what it should.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>
#include "moe_internal.h"

// The kernels are not part of this build: the checks under test return before any launcher is reached, and
// these stand-ins make the link complete (reaching one would be a test failure of its own).
namespace moe {
static hipError_t reached(const char* what) { printf("FAILED: launcher %s reached\n", what); return hipErrorUnknown; }
hipError_t launch_route(const float*, int, int, int, int32_t*, float*, int32_t*, int32_t*, hipStream_t) { return reached("route"); }
hipError_t launch_gate_route(const void*, const float*, int, int, int, int, int, float*, int32_t*, float*, int32_t*, int32_t*, hipStream_t) { return reached("gate_route"); }
void launch_gate_topk_only(const void*, const float*, int, int, int, int, int, float*, int32_t*, float*, hipStream_t) { reached("gate_topk"); }
void launch_count(const int32_t*, int, int, int, int32_t*, int32_t*, hipStream_t) { reached("count"); }
bool launch_dispatch_from_picks_fused(const int32_t*, const void*, int, int, int, int, int32_t*, int32_t*, void*, int32_t*, int32_t*, hipStream_t) { reached("dispatch_from_picks"); return true; }
bool launch_route_dispatch_fused(const float*, const void*, int, int, int, int, int32_t*, float*, int32_t*, int32_t*, void*, int32_t*, int32_t*, hipStream_t) { reached("route_dispatch"); return true; }
hipError_t launch_dispatch(const void*, const int32_t*, const int32_t*, int, int, int, int, void*, int32_t*, int32_t*, hipStream_t) { return reached("dispatch"); }
hipError_t launch_combine(const void*, const int32_t*, const float*, int, int, int, int, void*, hipStream_t) { return reached("combine"); }
hipError_t launch_pack_weights(const moe_config&, const void*, const void*, const void*, void*, hipStream_t) { return reached("pack"); }
hipError_t launch_ffn_stage(const moe_config&, int, int, const void*, const int32_t*, const void*, void*, hipStream_t) { return reached("ffn_stage"); }
hipError_t launch_ffn_segments(const moe_config&, int, const int32_t*, const int32_t*, const int32_t*, int, int, int, int, int, const void*, const void*, void*, hipStream_t) { return reached("ffn_segments"); }
bool ffn_picks_streaming(const moe_config& cfg, int, int n_segs, int rows_hint, int seg_rows_max) { return seg_rows_max <= 128 || rows_hint / (n_segs > 0 ? n_segs : 1) < 100; }
hipError_t launch_slot_segments(const int32_t*, const int32_t*, const int32_t*, const int32_t*, int, int, int32_t*, int32_t*, hipStream_t) { return reached("slot_segments"); }
size_t packed_weight_bytes(const moe_config& cfg) { return (size_t)3 * cfg.E * cfg.d * cfg.f * (cfg.dtype == MOE_BF16 ? 2 : 4); }
hipError_t launch_probe_stream_read(const void*, size_t, void*, hipStream_t) { return reached("probe_stream_read"); }
size_t probe_stream_read_bytes(size_t bytes) { return bytes; }
hipError_t launch_probe_mfma(const void*, int, int, void*, hipStream_t) { return reached("probe_mfma"); }
}  // namespace moe

static int failures = 0;
#define EXPECT(cond) do { if (!(cond)) { printf("FAILED line %d: %s\n", __LINE__, #cond); ++failures; } } while (0)

int main() {
  // planner: random instances shaped like the tests' (every output array exactly as large as documented)
  unsigned s = 12345;
  auto rnd = [&]() { s = s * 1664525u + 1013904223u; return (s >> 8) & 0xffffff; };
  int planned = 0;
  for (int it = 0; it < 3000; ++it) {
    const int M = 1 + rnd() % 48, N = 1 + rnd() % 12, S = (M + N - 1) / N + rnd() % 3;
    std::vector<double> a(M), cost(N);
    for (auto& v : a) v = (it % 3 == 0) ? double(1 + rnd() % 4) : (rnd() % 100000) / 100.0;
    std::vector<int32_t> rep(M), se((size_t)N * S), sc((size_t)N * S);
    const moe_status st = moe_plan_experts(M, N, S, a.data(), 2.0, rep.data(), se.data(), sc.data(), cost.data());
    if (st == MOE_OK) {
      ++planned;
      int copies = 0;
      for (int i = 0; i < M; ++i) copies += rep[i];
      int placed = 0;
      for (size_t q = 0; q < se.size(); ++q) placed += se[q] >= 0;
      EXPECT(copies == placed);
    }
  }
  EXPECT(planned > 2000);
  double one = 1.0, c1 = 0.0;
  int32_t r1 = 0, e1 = 0, k1 = 0;
  EXPECT(moe_plan_experts(0, 1, 1, &one, 1.0, &r1, &e1, &k1, &c1) == MOE_ERR_INVALID_ARG);
  EXPECT(moe_plan_experts(3, 1, 2, &one, 1.0, &r1, &e1, &k1, &c1) == MOE_ERR_INVALID_ARG);   // N * S < M
  EXPECT(moe_plan_experts(1, 1, 1, nullptr, 1.0, &r1, &e1, &k1, &c1) == MOE_ERR_INVALID_ARG);
  EXPECT(moe_plan_experts(1, 1, 1, &one, 1.0, &r1, &e1, &k1, &c1) == MOE_OK && r1 == 1 && e1 == 0);

  // contexts and argument checks
  moe_config good{64, 256, 512, 8, 2, MOE_BF16, 0.f};
  moe_ctx* ctx = nullptr;
  EXPECT(moe_create(&good, &ctx) == MOE_OK && ctx);
  moe_config bad = good;
  bad.k = 9;
  moe_ctx* none = nullptr;
  EXPECT(moe_create(&bad, &none) == MOE_ERR_INVALID_ARG && !none);
  bad = good; bad.d = 250;
  EXPECT(moe_create(&bad, &none) == MOE_ERR_UNSUPPORTED);
  bad = good; bad.load_skew = 0.5f;
  EXPECT(moe_create(&bad, &none) == MOE_ERR_INVALID_ARG);
  bad = good; bad.T_max = (1 << 22) / 2 + 1;
  EXPECT(moe_create(&bad, &none) == MOE_ERR_UNSUPPORTED);
  EXPECT(moe_create(nullptr, &none) == MOE_ERR_INVALID_ARG);
  EXPECT(moe_packed_weight_bytes(&good) == (size_t)3 * 8 * 256 * 512 * 2);
  EXPECT(moe_packed_weight_bytes(nullptr) == 0);
  EXPECT(std::strcmp(moe_ffn_kernel_name(ctx, 32, 0), "streaming") == 0);
  EXPECT(std::strcmp(moe_ffn_kernel_name(ctx, 64, 7), "") == 0);
  EXPECT(std::strcmp(moe_status_string(MOE_ERR_HIP), "MOE_ERR_HIP") == 0);

  void* ok = reinterpret_cast<void*>(0x1000);   // aligned, non-null, never dereferenced: the checks fail first
  void* odd = reinterpret_cast<void*>(0x1004);
  float* okf = static_cast<float*>(ok);
  int32_t* oki = static_cast<int32_t*>(ok);
  EXPECT(moe_route(ctx, 4, nullptr, oki, okf, oki, oki, nullptr) == MOE_ERR_INVALID_ARG);
  EXPECT(std::strstr(moe_last_error(ctx), "null") != nullptr);
  EXPECT(moe_route(ctx, 65, okf, oki, okf, oki, oki, nullptr) == MOE_ERR_INVALID_ARG);
  EXPECT(moe_route(nullptr, 4, okf, oki, okf, oki, oki, nullptr) == MOE_ERR_INVALID_ARG);
  EXPECT(moe_gate_route(ctx, 4, ok, okf, static_cast<float*>(odd), oki, okf, oki, oki, nullptr) == MOE_ERR_INVALID_ARG);
  EXPECT(moe_gate_route_dispatch(ctx, -1, ok, okf, nullptr, oki, okf, oki, oki, ok, oki, oki, nullptr) == MOE_ERR_INVALID_ARG);
  EXPECT(moe_dispatch(ctx, 4, ok, oki, oki, odd, oki, oki, nullptr) == MOE_ERR_INVALID_ARG);
  EXPECT(std::strstr(moe_last_error(ctx), "aligned") != nullptr);
  EXPECT(moe_route_dispatch(ctx, 4, okf, ok, oki, okf, oki, oki, nullptr, oki, oki, nullptr) == MOE_ERR_INVALID_ARG);
  EXPECT(moe_expert_ffn(ctx, 4, ok, oki, nullptr, ok, ok, nullptr) == MOE_ERR_INVALID_ARG);
  EXPECT(moe_expert_ffn_static(ctx, 4, ok, oki, ok, nullptr, nullptr) == MOE_ERR_INVALID_ARG);
  EXPECT(moe_ffn_input(ctx, 4, ok, oki, ok, odd, nullptr) == MOE_ERR_INVALID_ARG);
  EXPECT(moe_ffn_output(ctx, 99, ok, oki, ok, ok, nullptr) == MOE_ERR_INVALID_ARG);
  EXPECT(moe_combine(ctx, 4, ok, oki, nullptr, ok, nullptr) == MOE_ERR_INVALID_ARG);
  EXPECT(moe_pack_weights(ctx, ok, ok, ok, nullptr, nullptr) == MOE_ERR_INVALID_ARG);
  EXPECT(moe_slot_segments(ctx, 257, oki, oki, oki, oki, oki, oki, nullptr) == MOE_ERR_INVALID_ARG);
  EXPECT(moe_expert_ffn_segments(ctx, 4, -1, 0, ok, oki, oki, oki, ok, ok, ok, nullptr) == MOE_ERR_INVALID_ARG);
  EXPECT(moe_probe_mfma(ctx, ok, -1, 8, ok, nullptr, nullptr) == MOE_ERR_INVALID_ARG);
  EXPECT(moe_probe_stream_read(ctx, nullptr, 1024, ok, nullptr, nullptr) == MOE_ERR_INVALID_ARG);
  // a batch whose intermediate does not fit the static workspace is refused before anything else happens
  moe_config big{1 << 16, 128, 16384, 8, 2, MOE_BF16, 0.f};
  moe_ctx* bctx = nullptr;
  EXPECT(moe_create(&big, &bctx) == MOE_OK);
  EXPECT(moe_expert_ffn_static(bctx, 1 << 16, ok, oki, ok, ok, nullptr) == MOE_ERR_UNSUPPORTED);
  EXPECT(std::strstr(moe_last_error(bctx), "static workspace") != nullptr);
  moe_destroy(bctx);
  moe_destroy(ctx);
  moe_destroy(nullptr);
  if (failures) return 1;
  printf("host checks done\n");
  return 0;
}
