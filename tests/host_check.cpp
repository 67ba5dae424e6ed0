// Host-only checks of the C ABI, built with AddressSanitizer and UndefinedBehaviorSanitizer by
// tests/test_sanitizers.py: the planner and every argument / threshold validation that returns
// before the first GPU call (Section 4.2: 0 < c_low < c_high; tensor lists per Appendix A.1).
// Linked with gac_api.cpp and stand-ins for the kernel launchers (below), so no GPU code and
// no GPU is involved; reaching a launcher is a failure.
#include <hip/hip_runtime_api.h>

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "gac_internal.h"

static int g_failures = 0;
#define EXPECT(cond)                                                          \
  do {                                                                        \
    if (!(cond)) {                                                            \
      std::printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond);           \
      ++g_failures;                                                           \
    }                                                                         \
  } while (0)

// ---- stand-ins for gac_kernels.hip: none of them may be reached
namespace gac {
static hipError_t reached(const char* what) {
  std::printf("FAILED: launcher %s reached in a host-only check\n", what);
  ++g_failures;
  return hipErrorUnknown;
}
int adamw_blocks_per_cu(int) { return 1; }
hipError_t launch_reduce(int, const Seg*, int64_t, int, double*, unsigned int*, int, double*, gac_result*,
                         gac_result*, DecideParams, int, hipStream_t) { return reached("reduce"); }
hipError_t launch_snap_reduce(int, const Seg*, int64_t, int, const SnapBuffers&, int, double*, gac_result*,
                              gac_result*, DecideParams, int, int64_t, hipStream_t) { return reached("snap_reduce"); }
int64_t snap_group_count(int64_t n) { return (n + 255) / 256; }
hipError_t launch_finalize(const double*, double*, gac_result*, gac_result*, DecideParams, hipStream_t) { return reached("finalize"); }
hipError_t launch_apply(int, const Seg*, int, int64_t, int, const gac_result*, unsigned long long*, int, hipStream_t) { return reached("apply"); }
hipError_t launch_diag(const double*, const int32_t*, int, int64_t, int64_t, double, gac_diag*, gac_diag*, hipStream_t) { return reached("diag"); }
hipError_t launch_exchange(int, const Seg*, int, int64_t, int, const gac_result*, unsigned long long*, int, hipStream_t) { return reached("exchange"); }
hipError_t launch_snap_apply(int, const Seg*, int, int64_t, int, const gac_result*, unsigned long long*, int32_t*, int64_t, int, hipStream_t) { return reached("snap_apply"); }
hipError_t launch_apply_probe(int, const Seg*, int, int64_t, int, unsigned long long*, int, hipStream_t) { return reached("apply_probe"); }
hipError_t launch_apply_adamw(int, const Seg*, const AdamSeg*, int, int64_t, int, const gac_result*, unsigned long long*, AdamScalars, int, hipStream_t) { return reached("apply_adamw"); }
hipError_t launch_sweep(const double*, const int32_t*, int, int64_t, int64_t, const SweepPairs&, int, int32_t*, hipStream_t) { return reached("sweep"); }
hipError_t launch_set_step(int64_t*, int64_t, hipStream_t) { return reached("set_step"); }
hipError_t launch_set_word(uint32_t*, uint32_t, hipStream_t) { return reached("set_word"); }
hipError_t launch_state_op(int, int, const Seg*, int64_t, int, int, hipStream_t) { return reached("state_op"); }
hipError_t static_scratch(int, StaticScratch*) { return reached("static_scratch"); }
size_t static_scratch_bytes() { return 0; }
hipError_t launch_fill_segs(Seg*, const SegBatch&, unsigned int*, hipStream_t) { return reached("fill_segs"); }
}  // namespace gac

static void plan_checks() {
  int64_t chunks = -1, total = -1;
  // bf16: 32768 elements per chunk; fp32: 16384.  No chunk straddles two tensors.
  const int64_t a[] = {1, 32768, 32769, 0, 65536, 5};
  EXPECT(gac_plan_query(a, 6, GAC_BF16, 0, &chunks, &total) == GAC_OK);
  EXPECT(chunks == 1 + 1 + 2 + 0 + 2 + 1 && total == 1 + 32768 + 32769 + 65536 + 5);
  EXPECT(gac_plan_query(a, 6, GAC_F32, 0, &chunks, &total) == GAC_OK);
  EXPECT(chunks == 1 + 2 + 3 + 0 + 4 + 1);
  EXPECT(gac_plan_query(a, 6, GAC_F32, 2048, &chunks, nullptr) == GAC_OK);
  EXPECT(chunks == 1 + 16 + 17 + 0 + 32 + 1);
  EXPECT(gac_plan_query(nullptr, 0, GAC_F32, 0, &chunks, &total) == GAC_OK && chunks == 0 && total == 0);
  EXPECT(gac_plan_query(a, 6, GAC_F32, 0, nullptr, nullptr) == GAC_OK);
  const int64_t huge[] = {(int64_t{1} << 40) + 3, 7};
  EXPECT(gac_plan_query(huge, 2, GAC_BF16, 0, &chunks, &total) == GAC_OK);
  EXPECT(chunks == (int64_t{1} << 25) + 1 + 1 && total == (int64_t{1} << 40) + 10);
  const int64_t neg[] = {4, -1};
  EXPECT(gac_plan_query(neg, 2, GAC_F32, 0, &chunks, &total) == GAC_ERR_INVALID_ARG);
  EXPECT(gac_plan_query(a, -1, GAC_F32, 0, &chunks, &total) == GAC_ERR_INVALID_ARG);
  EXPECT(gac_plan_query(nullptr, 2, GAC_F32, 0, &chunks, &total) == GAC_ERR_INVALID_ARG);
  EXPECT(gac_plan_query(a, 6, 7, 0, &chunks, &total) == GAC_ERR_INVALID_ARG);
  EXPECT(gac_plan_query(a, 6, GAC_F32, 1000, &chunks, &total) == GAC_ERR_INVALID_ARG);
  EXPECT(gac_plan_query(a, 6, GAC_F32, -2048, &chunks, &total) == GAC_ERR_INVALID_ARG);
  // many tensors: the planner's table grows with the list
  std::vector<int64_t> many(100000);
  for (size_t j = 0; j < many.size(); ++j) many[j] = static_cast<int64_t>(j % 97);
  EXPECT(gac_plan_query(many.data(), static_cast<int32_t>(many.size()), GAC_BF16, 0, &chunks, &total) == GAC_OK);
  int64_t want_chunks = 0, want_total = 0;
  for (int64_t n : many) { want_chunks += n > 0; want_total += n; }
  EXPECT(chunks == want_chunks && total == want_total);
}

static void init_checks() {
  gac_config cfg;
  gac_default_config(&cfg);
  EXPECT(cfg.c_low == 0.05 && cfg.c_high == 0.3 && cfg.eps == 1e-8 && cfg.beta == 1.0);
  EXPECT(cfg.dtype == GAC_BF16 && cfg.n_tensors == 0 && cfg.device == -1 && cfg.flags == 0);
  gac_default_config(nullptr);
  const int64_t numel[] = {16, 0, 40000};
  cfg.n_tensors = 3;
  cfg.numel = numel;
  gac_ctx* ctx = reinterpret_cast<gac_ctx*>(0x1);
  EXPECT(gac_init(nullptr, &cfg) == GAC_ERR_INVALID_ARG);
  EXPECT(gac_init(&ctx, nullptr) == GAC_ERR_INVALID_ARG && ctx == nullptr);
  auto bad = [&](auto change, int want) {
    gac_config c = cfg;
    change(c);
    gac_ctx* out = reinterpret_cast<gac_ctx*>(0x1);
    EXPECT(gac_init(&out, &c) == want);
    EXPECT(out == nullptr);
  };
  const double nan = std::nan("");
  // Section 4.2: 0 < c_low < c_high
  bad([](gac_config& c) { c.c_low = 0.0; }, GAC_ERR_BAD_THRESHOLDS);
  bad([](gac_config& c) { c.c_low = -0.1; }, GAC_ERR_BAD_THRESHOLDS);
  bad([](gac_config& c) { c.c_low = 0.3; }, GAC_ERR_BAD_THRESHOLDS);
  bad([](gac_config& c) { c.c_high = 0.01; }, GAC_ERR_BAD_THRESHOLDS);
  bad([&](gac_config& c) { c.c_low = nan; }, GAC_ERR_BAD_THRESHOLDS);
  bad([&](gac_config& c) { c.c_high = nan; }, GAC_ERR_BAD_THRESHOLDS);
  bad([&](gac_config& c) { c.c_low = INFINITY; c.c_high = INFINITY; }, GAC_ERR_BAD_THRESHOLDS);
  bad([](gac_config& c) { c.eps = -1e-9; }, GAC_ERR_BAD_THRESHOLDS);
  bad([&](gac_config& c) { c.eps = nan; }, GAC_ERR_BAD_THRESHOLDS);
  bad([](gac_config& c) { c.beta = -1.0; }, GAC_ERR_BAD_THRESHOLDS);
  bad([](gac_config& c) { c.beta = INFINITY; }, GAC_ERR_BAD_THRESHOLDS);
  bad([](gac_config& c) { c.max_grad_norm = -1.0; }, GAC_ERR_BAD_THRESHOLDS);
  bad([&](gac_config& c) { c.max_grad_norm = nan; }, GAC_ERR_BAD_THRESHOLDS);
  bad([](gac_config& c) { c.n_tensors = -1; }, GAC_ERR_INVALID_ARG);
  bad([](gac_config& c) { c.numel = nullptr; }, GAC_ERR_INVALID_ARG);
  bad([](gac_config& c) { c.flags = 2; }, GAC_ERR_INVALID_ARG);
  bad([](gac_config& c) { c.flags = 0x80000000u; }, GAC_ERR_INVALID_ARG);
  bad([](gac_config& c) { c.dtype = 2; }, GAC_ERR_INVALID_ARG);
  bad([](gac_config& c) { c.chunk_elems = 100; }, GAC_ERR_INVALID_ARG);
  bad([](gac_config& c) { c.chunk_elems = -2048; }, GAC_ERR_INVALID_ARG);
  bad([](gac_config& c) { c.grid_blocks = -1; }, GAC_ERR_INVALID_ARG);
  bad([](gac_config& c) { c.grid_blocks = (1 << 16) + 1; }, GAC_ERR_INVALID_ARG);
  bad([](gac_config& c) { c.apply_blocks = -1; }, GAC_ERR_INVALID_ARG);
  bad([](gac_config& c) { c.history_capacity = 4097; }, GAC_ERR_INVALID_ARG);
  bad([](gac_config& c) { c.history_capacity = -1; }, GAC_ERR_INVALID_ARG);
  bad([](gac_config& c) { c.reserved = 1; }, GAC_ERR_INVALID_ARG);
  const int64_t negative[] = {16, -2, 3};
  bad([&](gac_config& c) { c.numel = negative; }, GAC_ERR_INVALID_ARG);
  // caller-provided state: a missing buffer for a non-empty tensor; the snapshot form needs
  // buffers of the library's own
  void* two_of_three[] = {reinterpret_cast<void*>(0x1000), nullptr, nullptr};
  bad([&](gac_config& c) { c.state_ptrs = two_of_three; }, GAC_ERR_INVALID_ARG);
  void* all_three[] = {reinterpret_cast<void*>(0x1000), nullptr, reinterpret_cast<void*>(0x2000)};
  bad([&](gac_config& c) { c.state_ptrs = all_three; c.flags = GAC_FLAG_SNAPSHOT_IN_REDUCE; }, GAC_ERR_INVALID_ARG);
}

static void null_context_checks() {
  gac_result res;
  double sums[3];
  int64_t n = 0, first = 0;
  gac_diag diag;
  gac_placement rep;
  int32_t counts[3];
  const double lo[] = {0.05}, hi[] = {0.3};
  void* p[] = {nullptr};
  float* fp[] = {nullptr};
  gac_adamw_hyper h = {1e-6, 0.9, 0.999, 1e-8, 1e-2, 1};
  EXPECT(gac_step(nullptr, p, nullptr, &res) == GAC_ERR_INVALID_ARG);
  EXPECT(gac_step_exchange(nullptr, p, nullptr, &res) == GAC_ERR_INVALID_ARG);
  EXPECT(gac_reduce_local(nullptr, p, nullptr, sums) == GAC_ERR_INVALID_ARG);
  EXPECT(gac_apply(nullptr, p, sums, nullptr, &res) == GAC_ERR_INVALID_ARG);
  EXPECT(gac_step_adamw(nullptr, p, fp, fp, fp, nullptr, &h, nullptr, &res) == GAC_ERR_INVALID_ARG);
  EXPECT(gac_result_device(nullptr, nullptr) == GAC_ERR_INVALID_ARG);
  EXPECT(gac_state_export(nullptr, p, &n, nullptr) == GAC_ERR_INVALID_ARG);
  EXPECT(gac_state_import(nullptr, p, 0, nullptr) == GAC_ERR_INVALID_ARG);
  EXPECT(gac_reset(nullptr, nullptr) == GAC_ERR_INVALID_ARG);
  EXPECT(gac_place_state(nullptr, p, 1, 0, nullptr, &rep) == GAC_ERR_INVALID_ARG);
  EXPECT(gac_set_thresholds(nullptr, 0.05, 0.3) == GAC_ERR_INVALID_ARG);
  EXPECT(gac_history_read(nullptr, 1, sums, counts, &n, &first, nullptr) == GAC_ERR_INVALID_ARG);
  EXPECT(gac_diag_summary(nullptr, 0, &diag, nullptr) == GAC_ERR_INVALID_ARG);
  EXPECT(gac_threshold_sweep(nullptr, 0, 1, lo, hi, counts, nullptr) == GAC_ERR_INVALID_ARG);
  EXPECT(gac_profile_enable(nullptr, 1) == GAC_ERR_INVALID_ARG);
  EXPECT(gac_profile_read(nullptr, sums, sums, sums, counts) == GAC_ERR_INVALID_ARG);
  gac_destroy(nullptr);
  for (int code = 1; code >= -9; --code) {
    const char* s = gac_strerror(code);
    EXPECT(s != nullptr && std::strlen(s) > 0);
  }
  EXPECT(std::strstr(gac_strerror(GAC_ERR_BAD_THRESHOLDS), "c_low") != nullptr);
  EXPECT(std::strstr(gac_strerror(GAC_ERR_TOO_LARGE), "capacity") != nullptr);
  EXPECT(std::strlen(gac_last_hip_error(nullptr)) == 0);
  EXPECT(std::strncmp(gac_version(), "gac-mi355x", 10) == 0);
  EXPECT(gac_source_hash() != nullptr);
}

static void static_step_checks() {
  // everything gac_step_static refuses before it touches the GPU
  gac_config cfg;
  gac_default_config(&cfg);
  cfg.dtype = GAC_F32;
  const int64_t numel[] = {8, 0};
  void* state[] = {reinterpret_cast<void*>(0x1000), nullptr};
  void* grads[] = {reinterpret_cast<void*>(0x2000), nullptr};
  cfg.n_tensors = 2;
  cfg.numel = numel;
  cfg.state_ptrs = state;
  auto bad = [&](auto change, void* const* g, int64_t step, int want) {
    gac_config c = cfg;
    change(c);
    EXPECT(gac_step_static(&c, g, step, nullptr, nullptr) == want);
  };
  EXPECT(gac_step_static(nullptr, grads, 1, nullptr, nullptr) == GAC_ERR_INVALID_ARG);
  bad([](gac_config& c) { c.state_ptrs = nullptr; }, grads, 1, GAC_ERR_INVALID_ARG);
  bad([](gac_config&) {}, nullptr, 1, GAC_ERR_INVALID_ARG);
  bad([](gac_config&) {}, grads, -1, GAC_ERR_INVALID_ARG);
  bad([](gac_config& c) { c.flags = GAC_FLAG_SNAPSHOT_IN_REDUCE; }, grads, 1, GAC_ERR_INVALID_ARG);
  bad([](gac_config& c) { c.history_capacity = 16; }, grads, 1, GAC_ERR_INVALID_ARG);
  bad([](gac_config& c) { c.c_low = 0.5; }, grads, 1, GAC_ERR_BAD_THRESHOLDS);
  bad([](gac_config& c) { c.eps = -1.0; }, grads, 1, GAC_ERR_BAD_THRESHOLDS);
  bad([](gac_config& c) { c.chunk_elems = 100; }, grads, 1, GAC_ERR_INVALID_ARG);
  bad([](gac_config& c) { c.grid_blocks = 1025; }, grads, 1, GAC_ERR_TOO_LARGE);
  bad([](gac_config&) {}, state, 1, GAC_ERR_INVALID_ARG);  // the gradient buffer IS the state buffer
  void* misaligned[] = {reinterpret_cast<void*>(0x2002), nullptr};
  bad([](gac_config&) {}, misaligned, 1, GAC_ERR_INVALID_ARG);
  void* missing[] = {nullptr, nullptr};
  bad([](gac_config&) {}, missing, 1, GAC_ERR_INVALID_ARG);
  const int64_t negative[] = {8, -1};
  bad([&](gac_config& c) { c.numel = negative; }, grads, 1, GAC_ERR_INVALID_ARG);
  // one tensor more than the static table holds
  const int n = GAC_STATIC_MAX_TENSORS + 1;
  std::vector<int64_t> many_numel(n, 8);
  std::vector<void*> many_state(n, reinterpret_cast<void*>(0x1000)), many_grads(n, reinterpret_cast<void*>(0x2000));
  gac_config big = cfg;
  big.n_tensors = n;
  big.numel = many_numel.data();
  big.state_ptrs = many_state.data();
  EXPECT(gac_step_static(&big, many_grads.data(), 1, nullptr, nullptr) == GAC_ERR_TOO_LARGE);
}

int main() {
  plan_checks();
  init_checks();
  null_context_checks();
  static_step_checks();
  if (g_failures == 0) std::printf("host checks ok\n");
  return g_failures == 0 ? 0 : 1;
}
