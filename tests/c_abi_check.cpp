// Plain C++ caller of the C ABI (no Python, no PyTorch): runs one GAC step on a short vector
// given on the command line and prints what the library returned, one "key: values" line each.
// The GPU test that drives it compares the output with the hand-worked cases in
// tests/golden/gac_len8_cases.txt (derived from Eq. 1 / Appendix A.1, Section 4.2 and Eq. 4).
//
//   c_abi_check <f32|bf16>[:step|:static|:snapshot] <eps> <c_low> <c_high> <n> d_1..d_n g_1..g_n
//
// The suffix picks the entry point: gac_step on a context with caller-owned state (default),
// gac_step_static (no context, nothing allocated), or gac_step on a snapshot-form context
// (library-owned state, imported and exported).
#include <hip/hip_runtime_api.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "gac.h"

#define CHECK_HIP(x)                                                              \
  do {                                                                            \
    hipError_t e_ = (x);                                                          \
    if (e_ != hipSuccess) {                                                       \
      std::printf("error: %s -> %s\n", #x, hipGetErrorString(e_));                \
      return 2;                                                                   \
    }                                                                             \
  } while (0)
#define CHECK_GAC(x)                                                              \
  do {                                                                            \
    int rc_ = (x);                                                                \
    if (rc_ != GAC_OK) {                                                          \
      std::printf("error: %s -> %d %s (%s)\n", #x, rc_, gac_strerror(rc_), gac_last_hip_error(nullptr)); \
      return 3;                                                                   \
    }                                                                             \
  } while (0)

// The inputs of the hand-worked cases are small integers: exact in bf16, so truncation is a
// faithful conversion here.
static uint16_t to_bf16(float f) {
  uint32_t u;
  std::memcpy(&u, &f, 4);
  return static_cast<uint16_t>(u >> 16);
}
static float from_bf16(uint16_t h) {
  uint32_t u = static_cast<uint32_t>(h) << 16;
  float f;
  std::memcpy(&f, &u, 4);
  return f;
}

int main(int argc, char** argv) {
  if (argc < 6) return 1;
  const bool bf16 = std::strncmp(argv[1], "bf16", 4) == 0;
  const char* colon = std::strchr(argv[1], ':');
  const char* entry = colon ? colon + 1 : "step";
  const double eps = std::atof(argv[2]), c_low = std::atof(argv[3]), c_high = std::atof(argv[4]);
  const int n = std::atoi(argv[5]);
  if (argc != 6 + 2 * n) return 1;
  std::vector<float> d(n), g(n);
  for (int i = 0; i < n; ++i) d[i] = static_cast<float>(std::atof(argv[6 + i]));
  for (int i = 0; i < n; ++i) g[i] = static_cast<float>(std::atof(argv[6 + n + i]));
  const size_t es = bf16 ? 2 : 4;
  std::vector<unsigned char> hd(n * es), hg(n * es);
  for (int i = 0; i < n; ++i) {
    if (bf16) {
      reinterpret_cast<uint16_t*>(hd.data())[i] = to_bf16(d[i]);
      reinterpret_cast<uint16_t*>(hg.data())[i] = to_bf16(g[i]);
    } else {
      reinterpret_cast<float*>(hd.data())[i] = d[i];
      reinterpret_cast<float*>(hg.data())[i] = g[i];
    }
  }
  void *dev_g, *dev_state, *dev_ref;
  CHECK_HIP(hipMalloc(&dev_g, n * es));
  CHECK_HIP(hipMalloc(&dev_state, n * es));
  CHECK_HIP(hipMalloc(&dev_ref, n * es));
  CHECK_HIP(hipMemcpy(dev_g, hg.data(), n * es, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(dev_ref, hd.data(), n * es, hipMemcpyHostToDevice));

  gac_config cfg;
  gac_default_config(&cfg);
  cfg.c_low = c_low;
  cfg.c_high = c_high;
  cfg.eps = eps;
  cfg.dtype = bf16 ? GAC_BF16 : GAC_F32;
  const int64_t numel = n;
  cfg.n_tensors = 1;
  cfg.numel = &numel;
  void* state_list[1] = {dev_state};
  cfg.state_ptrs = state_list;
  void* ref_list[1] = {dev_ref};
  void* grad_list[1] = {dev_g};
  gac_result r;
  gac_ctx* ctx = nullptr;
  if (std::strcmp(entry, "static") == 0) {
    // no context: the caller's state buffer holds d, the result record lands in device memory
    CHECK_HIP(hipMemcpy(dev_state, hd.data(), n * es, hipMemcpyHostToDevice));
    gac_result* dev_r = nullptr;
    CHECK_HIP(hipMalloc(reinterpret_cast<void**>(&dev_r), sizeof(gac_result)));
    CHECK_GAC(gac_step_static(&cfg, grad_list, 1, nullptr, dev_r));
    CHECK_HIP(hipDeviceSynchronize());
    CHECK_HIP(hipMemcpy(&r, dev_r, sizeof(r), hipMemcpyDeviceToHost));
    (void)hipFree(dev_r);
  } else if (std::strcmp(entry, "snapshot") == 0) {
    cfg.state_ptrs = nullptr;  // the library owns two state buffers
    cfg.flags = GAC_FLAG_SNAPSHOT_IN_REDUCE;
    CHECK_GAC(gac_init(&ctx, &cfg));
    CHECK_GAC(gac_state_import(ctx, ref_list, 0, nullptr));
    CHECK_GAC(gac_step(ctx, grad_list, nullptr, &r));
    void* out_list[1] = {dev_state};
    CHECK_GAC(gac_state_export(ctx, out_list, nullptr, nullptr));
  } else {
    CHECK_GAC(gac_init(&ctx, &cfg));
    CHECK_GAC(gac_state_import(ctx, ref_list, 0, nullptr));  // the reference direction d
    CHECK_GAC(gac_step(ctx, grad_list, nullptr, &r));
  }
  CHECK_HIP(hipDeviceSynchronize());
  std::vector<unsigned char> og(n * es), os(n * es);
  CHECK_HIP(hipMemcpy(og.data(), dev_g, n * es, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(os.data(), dev_state, n * es, hipMemcpyDeviceToHost));
  std::printf("sums: %.17g %.17g %.17g\n", r.dot, r.gg, r.dd);
  std::printf("c: %.17g\nalpha: %.17g\ncoef: %.17g\nregime: %d\nstep: %lld\n", r.c, r.alpha, r.coef,
              r.regime, static_cast<long long>(r.step));
  std::printf("gprime:");
  for (int i = 0; i < n; ++i)
    std::printf(" %.9g", bf16 ? from_bf16(reinterpret_cast<uint16_t*>(og.data())[i])
                              : reinterpret_cast<float*>(og.data())[i]);
  std::printf("\nstate:");
  for (int i = 0; i < n; ++i)
    std::printf(" %.9g", bf16 ? from_bf16(reinterpret_cast<uint16_t*>(os.data())[i])
                              : reinterpret_cast<float*>(os.data())[i]);
  std::printf("\n");
  gac_destroy(ctx);
  (void)hipFree(dev_g);
  (void)hipFree(dev_state);
  (void)hipFree(dev_ref);
  return 0;
}
