// Host-only driver for the sanitizer build of the C ABI's argument validation (tests/test_sanitizers.py):
// links the library's host code (moesd_api.cpp, closed_forms.cpp) with launch stubs that enqueue
// nothing, and calls every entry point with bad and with well-formed arguments.  No GPU is touched:
// every well-formed call is refused by the stubbed runtime query before a kernel would start.
#include <cmath>
#include <cstdio>
#include <cstring>

#include "../../paper_2505_19645_amd/csrc/common.h"

// ---- stubs for the kernels' launch functions (never reached with valid device pointers) ----
hipError_t launch_router_logits(const uint16_t *, const uint16_t *, const float *, const uint16_t *, int, int, int,
                                double *, hipStream_t) { return hipErrorNoDevice; }
hipError_t launch_topk(const double *, int, int, int, int, int, float, int, int, int32_t *, float *, float *,
                       hipStream_t) { return hipErrorNoDevice; }
hipError_t launch_permute(const int32_t *, int64_t, int, int, int32_t *, int32_t *, int32_t *, int32_t *, int32_t *,
                          int32_t *, int32_t *, int, hipStream_t) { return hipErrorNoDevice; }
hipError_t launch_topk_permute(const double *, int, int, int, int, int, float, int, int, int32_t *, float *, float *,
                               int32_t *, int32_t *, int32_t *, int32_t *, int32_t *, int32_t *, int32_t *, int,
                               hipStream_t) { return hipErrorNoDevice; }
hipError_t launch_gate_up(const StreamArgs &, hipStream_t) { return hipErrorNoDevice; }
hipError_t launch_down(const StreamArgs &, hipStream_t) { return hipErrorNoDevice; }
size_t tiled_partials_bytes() { return (size_t)128 << 20; }
int shared_expert_streams(int, int, int, int, int, int, int) { return 1; }
hipError_t launch_gate_up_tiled(const StreamArgs &, float *, hipStream_t) { return hipErrorNoDevice; }
hipError_t launch_down_tiled(const StreamArgs &, float *, hipStream_t) { return hipErrorNoDevice; }
hipError_t launch_combine(const float *, const float *, int, const float *, const float *, const int32_t *, int, int,
                          int, uint16_t *, float *, hipStream_t) { return hipErrorNoDevice; }

static int failures = 0;
#define EXPECT(cond)                                            \
  do {                                                          \
    if (!(cond)) {                                              \
      std::printf("FAILED line %d: %s\n", __LINE__, #cond);     \
      ++failures;                                               \
    }                                                           \
  } while (0)

int main() {
  moesd_layer_desc d{};
  d.d = 256; d.E = 8; d.top_k = 2; d.inter = 512; d.renormalize = 1; d.routed_scale = 1.0f;
  void *p = reinterpret_cast<void *>(0x1000);  // never dereferenced
  moesd_weights w{};
  w.w_router = w.w_gate = w.w_up = w.w_down = p;
  // closed forms
  EXPECT(std::fabs(moesd_expected_active_experts(8, 2, 1) - 2.0) < 1e-12);
  EXPECT(std::isnan(moesd_expected_active_experts(0, 0, 1)));
  EXPECT(moesd_token_threshold(60, 4, 0.95) == 44);
  double pe[4] = {0.5, 0.5, 0.5, 0.5};
  EXPECT(std::fabs(moesd_expected_active_experts_p(pe, 4, 1) - 2.0) < 1e-12);
  EXPECT(moesd_expected_tokens_per_expert(8, 2, 0) == 0.0);
  // workspace sizes: valid, invalid, the largest shapes (no overflow of the size arithmetic)
  EXPECT(moesd_workspace_bytes(&d, 16) > 0 && moesd_workspace_bytes(&d, 16) % 256 == 0);
  EXPECT(moesd_workspace_bytes(&d, -1) == 0 && moesd_workspace_bytes(nullptr, 4) == 0);
  moesd_layer_desc big = d;
  big.d = 7168; big.E = 1024; big.top_k = 32; big.inter = 20480; big.shared_inter = 20480;
  EXPECT(moesd_workspace_bytes(&big, 200000) > ((size_t)1 << 36));
  EXPECT(moesd_workspace_bytes(&big, 300000) == 0);  // T * d * 2 >= 2^32
  // forward: every kind of refusal, then a well-formed call that stops at the (absent) runtime
  EXPECT(moesd_moe_forward(&d, &w, p, -1, p, nullptr, p, 1 << 20, 0, 0, 0, 0, 0, 0, 0, nullptr) == MOESD_INVALID_ARG);
  EXPECT(moesd_moe_forward(&d, &w, p, 16, p, nullptr, p, 16, 0, 0, 0, 0, 0, 0, 0, nullptr) == MOESD_WORKSPACE_TOO_SMALL);
  EXPECT(moesd_moe_forward(&d, &w, p, 16, p, nullptr, reinterpret_cast<void *>(0x1010), 1 << 20, 0, 0, 0, 0, 0, 0, 0,
                           nullptr) == MOESD_INVALID_ARG);
  EXPECT(moesd_moe_forward(&d, nullptr, p, 16, p, nullptr, p, 1 << 20, 0, 0, 0, 0, 0, 0, 0, nullptr) == MOESD_INVALID_ARG);
  EXPECT(moesd_moe_forward(&d, &w, nullptr, 16, p, nullptr, p, 1 << 20, 0, 0, 0, 0, 0, 0, 0, nullptr) == MOESD_INVALID_ARG);
  moesd_layer_desc bad = d;
  bad.top_k = 9;
  EXPECT(moesd_moe_forward(&bad, &w, p, 16, p, nullptr, p, 1 << 20, 0, 0, 0, 0, 0, 0, 0, nullptr) == MOESD_INVALID_ARG);
  bad = d; bad.E = 2048;
  EXPECT(moesd_moe_forward(&bad, &w, p, 16, p, nullptr, p, 1 << 20, 0, 0, 0, 0, 0, 0, 0, nullptr) == MOESD_UNSUPPORTED);
  bad = d; bad.weight_format = MOESD_WEIGHTS_FP8_E4M3;  // scales missing
  EXPECT(moesd_moe_forward(&bad, &w, p, 16, p, nullptr, p, 1 << 30, 0, 0, 0, 0, 0, 0, 0, nullptr) == MOESD_INVALID_ARG);
  bad = d; bad.n_group = 3; bad.topk_group = 1;
  EXPECT(moesd_moe_forward(&bad, &w, p, 16, p, nullptr, p, 1 << 20, 0, 0, 0, 0, 0, 0, 0, nullptr) == MOESD_INVALID_ARG);
  EXPECT(moesd_moe_forward_static(&d, &w, p, 200000, p, nullptr, 0, 0, 0, 0, 0, 0, 0, nullptr) == MOESD_WORKSPACE_TOO_SMALL);
  EXPECT(moesd_moe_forward_static(&d, &w, nullptr, 16, p, nullptr, 0, 0, 0, 0, 0, 0, 0, nullptr) == MOESD_INVALID_ARG);
  EXPECT(moesd_permute(8, 9, 4, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == MOESD_INVALID_ARG);
  EXPECT(moesd_route(&d, nullptr, p, nullptr, 4, nullptr, nullptr, p, 1 << 20, nullptr) == MOESD_INVALID_ARG);
  EXPECT(moesd_moe_forward(&d, &w, p, 0, p, nullptr, nullptr, 0, 0, 0, 0, 0, 0, 0, 0, nullptr) == MOESD_OK);  // T = 0
  // well-formed: the runtime query or the first (stubbed) launch reports an error, nothing else happens
  EXPECT(moesd_moe_forward(&d, &w, p, 16, p, nullptr, p, 1 << 20, 0, 0, 0, 0, 0, 0, 0, nullptr) == MOESD_HIP_ERROR);
  EXPECT(moesd_last_hip_error() != 0);
  EXPECT(std::strcmp(moesd_status_string(MOESD_WORKSPACE_TOO_SMALL), "workspace too small") == 0);
  std::printf(failures ? "abi_args: %d FAILED\n" : "abi_args: ok\n", failures);
  return failures ? 1 : 0;
}
