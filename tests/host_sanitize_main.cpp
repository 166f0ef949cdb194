// Host-side exercise of the C ABI for the sanitizer build (tests/test_host_sanitizers.py): every entry point is
// called in ways that end on the host (argument errors, size queries, the pipeline-degree routine), so the run
// needs no GPU.  Built with AddressSanitizer and UndefinedBehaviorSanitizer on the host code of the library.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../include/moe_mi355x.h"

static int g_fail = 0;
#define EXPECT(cond)                                                        \
  do {                                                                      \
    if (!(cond)) { printf("FAILED line %d: %s\n", __LINE__, #cond); ++g_fail; } \
  } while (0)

static uint64_t g_s = 0x9E3779B97F4A7C15ull;
static double rnd() {
  g_s ^= g_s << 13; g_s ^= g_s >> 7; g_s ^= g_s << 17;
  return (double)(g_s >> 11) / 9007199254740992.0;
}

int main() {
  // ---- capacity and size queries over many configurations, valid and invalid
  EXPECT(moe_capacity(256, 4, 1, 1.25) == 80 && moe_capacity(0, 4, 1, 1.0) == -1);
  const int Ns[] = {1, 63, 64, 1000, 16384, 65536}, Ms[] = {8, 64, 200, 768, 4096, 9216}, Es[] = {1, 4, 8, 12, 48, 64, 130, 256};
  for (int N : Ns) for (int M : Ms) for (int E : Es) for (int k : {1, 2, 6, 8}) for (int dt : {0, 1}) for (int gate : {0, 1, 2, 3}) {
    moe_config_t c = {N, M, E, 64, k, gate == 3 ? 16 : 0, dt, dt ? MOE_ACT_SWIGLU : MOE_ACT_RELU, gate, 0, 0};
    if (gate == 3) c.top_k = E;
    size_t ws = 0, sv = 0;
    const moe_status_t st = moe_workspace_bytes(&c, &ws, &sv);
    const bool ok = c.top_k <= E && c.top_k <= 8 && E <= 256 && M % (dt ? 8 : 4) == 0;
    EXPECT((st == MOE_OK) == ok);
    if (st == MOE_OK) {
      EXPECT(ws > 0 && sv > 0);
      size_t end = 0;
      for (int w = 0; w < MOE_SAVED_N_; ++w) {
        size_t off = 0, n = 0;
        EXPECT(moe_saved_offset(&c, w, &off, &n) == MOE_OK && off >= end);
        end = off + n;
      }
      EXPECT(end <= sv);
      size_t xw = 0;
      if (gate != 3) EXPECT(moe_route_xmoe_workspace_bytes(&c, 32, &xw) == MOE_OK && xw > 0);
      EXPECT(moe_route_xmoe_workspace_bytes(&c, 6, &xw) != MOE_OK);
    } else {
      EXPECT(std::strlen(moe_last_error()) > 0);
    }
  }
  // ---- every launching entry point, stopped by its argument checks
  {
    moe_config_t c = {64, 64, 4, 128, 2, 0, MOE_F32, MOE_ACT_RELU, 0, 0, 0};
    void* null = nullptr;
    void* fake = reinterpret_cast<void*>(4096);
    void* odd = reinterpret_cast<void*>(4100);
    float* ff = reinterpret_cast<float*>(fake);
    int32_t* fi = reinterpret_cast<int32_t*>(fake);
    EXPECT(moe_dispatch(&c, null, fi, fake, null) == MOE_ERR_INVALID_ARG);
    EXPECT(moe_dispatch(&c, odd, fi, fake, null) == MOE_ERR_INVALID_ARG);
    EXPECT(moe_dispatch_bwd(&c, null, fi, null, fake, null) == MOE_ERR_INVALID_ARG);
    EXPECT(moe_combine(&c, null, ff, fi, null, fake, null) == MOE_ERR_INVALID_ARG);
    EXPECT(moe_combine_bwd(&c, fake, null, ff, fi, fake, ff, null) == MOE_ERR_INVALID_ARG);
    EXPECT(moe_route(&c, fake, fake, null ? ff : nullptr, ff, ff, fi, ff, fi, fi, fi, fi, fi, fake, 16, null) == MOE_ERR_WORKSPACE);
    EXPECT(moe_route(nullptr, fake, fake, nullptr, ff, ff, fi, ff, fi, fi, fi, fi, fi, fake, 16, null) == MOE_ERR_INVALID_ARG);
    EXPECT(moe_route_bwd(&c, fake, fake, ff, fi, fi, ff, fake, nullptr, fake, fake, 16, null) == MOE_ERR_WORKSPACE);
    EXPECT(moe_route_noisy(&c, fake, fake, nullptr, null, ff, ff, ff, ff, fi, ff, fi, fi, fi, fi, fi, fake, 1u << 30, null) == MOE_ERR_INVALID_ARG);
    EXPECT(moe_route_noisy_bwd(&c, fake, fake, fake, ff, ff, ff, fi, fi, ff, fake, nullptr, null, fake, fake, 1u << 30, null) == MOE_ERR_INVALID_ARG);
    EXPECT(moe_route_xmoe(&c, fake, fake, fake, 7, ff, ff, ff, fi, ff, fi, fi, fi, fi, fi, fake, 1u << 30, null) == MOE_ERR_UNSUPPORTED);
    EXPECT(moe_route_xmoe_bwd(&c, fake, fake, fake, 32, ff, ff, fi, fi, ff, fake, fake, fake, fake, 8, null) == MOE_ERR_WORKSPACE);
    EXPECT(moe_expert_ffn_fwd(&c, fake, fi, null, null, fake, fake, fake, null, fake, null, 0, null) == MOE_ERR_INVALID_ARG);
    EXPECT(moe_expert_ffn_bwd(&c, fake, fake, fi, fake, null, fake, fake, null, fake, fake, fake, null, fake, fake, 16, null) == MOE_ERR_WORKSPACE);
    EXPECT(moe_layer_fwd(&c, fake, fake, nullptr, fake, null, fake, fake, fake, 16, fake, 1u << 30, null) == MOE_ERR_WORKSPACE);
    EXPECT(moe_layer_bwd(&c, fake, fake, fake, fake, null, fake, fake, 1u << 30, fake, fake, nullptr, fake, null, fake, fake, 16, null) == MOE_ERR_WORKSPACE);
    EXPECT(moe_layer_fwd_chunked(&c, fake, fake, nullptr, fake, null, fake, fake, fake, 1u << 30, fake, 1u << 30, 99, null, null) == MOE_ERR_INVALID_ARG);
    EXPECT(moe_layer_bwd_chunked(&c, fake, fake, fake, fake, null, fake, fake, 1u << 30, fake, fake, nullptr, fake, null, fake, fake, 1u << 30, 0, null) == MOE_ERR_INVALID_ARG);
    EXPECT(moe_layer_fwd_routed(&c, fake, fake, null, fake, fake, fake, 1u << 30, fake, 1u << 30, 17, null, null) == MOE_ERR_INVALID_ARG);
    EXPECT(moe_layer_bwd_routed(&c, fake, fake, null, fake, fake, 1u << 30, fake, fake, null, fake, nullptr, fake, 1u << 30, 1, null) == MOE_ERR_INVALID_ARG);
    moe_config_t big = {1 << 20, 64, 64, 64, 8, 0, MOE_BF16, MOE_ACT_RELU, 0, 0, 0};
    EXPECT(moe_route_static(&big, fake, fake, nullptr, ff, ff, fi, ff, fi, fi, fi, fi, fi, null) == MOE_ERR_WORKSPACE);
    EXPECT(moe_route_static(&c, null, fake, nullptr, ff, ff, fi, ff, fi, fi, fi, fi, fi, null) == MOE_ERR_INVALID_ARG);
  }
  // ---- pipeline degree (Sec. 4): random models, the arg-min against every degree tried
  for (int it = 0; it < 2000; ++it) {
    moe_pipeline_model_t m;
    double* f = reinterpret_cast<double*>(&m);
    for (int i = 0; i < 13; ++i) f[i] = rnd() < 0.15 ? 0.0 : std::pow(10.0, 4 * rnd() - 3);
    int32_t r = 0, which = 0;
    double t = 0;
    EXPECT(moe_find_pipeline_degree(&m, 32, &r, &t, &which) == MOE_OK && r >= 1 && r <= 32 && which >= 1 && which <= 4);
    double best = INFINITY;
    for (int q = 1; q <= 32; ++q) {
      int32_t w = 0;
      const double tq = moe_pipeline_time(&m, q, &w);
      EXPECT(std::isfinite(tq) && w >= 1 && w <= 4);
      if (tq < best) best = tq;
    }
    EXPECT(std::fabs(t - best) <= 1e-12 * std::fabs(best));
  }
  {
    moe_pipeline_model_t bad;
    std::memset(&bad, 0, sizeof(bad));
    bad.alpha_exp = -1.0;
    int32_t r = 0;
    EXPECT(moe_find_pipeline_degree(&bad, 8, &r, nullptr, nullptr) == MOE_ERR_INVALID_ARG);
    EXPECT(moe_find_pipeline_degree(nullptr, 8, &r, nullptr, nullptr) == MOE_ERR_INVALID_ARG);
    EXPECT(std::isnan(moe_pipeline_time(&bad, 2.0, nullptr)));
  }
  printf(g_fail ? "host sanitizer driver: %d expectation(s) failed\n" : "host sanitizer driver: ok\n", g_fail);
  return g_fail ? 1 : 0;
}
