// Stand-alone check of the C ABI without PyTorch: device memory from hipMalloc
// (or, with a non-zero third argument, from co2_buffer_set_create), libco2.so
// called directly, results compared element by element with the CPU oracle
// (linked in from oracle/co2_oracle.cpp -- this program is a test).
//
//   co2_selftest [n] [K] [buffer_set] [mode]   exit code 0 = every element within 1e-5 relative
//   mode 0: co2_outer_step;  1: co2_outer_step_static (no workspace argument);
//        2: co2_outer_step with all three variant switches (current-round mean, anchor pull,
//           clipping by norm rescale) against the oracle's variant function
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "co2.h"
#include "co2_layout.h"

extern "C" int co2_oracle_outer_step_f32(int64_t n, int32_t S, const int64_t* seg_off, int32_t K,
                                         float alpha, float beta, float phi, float c, int32_t tau,
                                         int64_t step, float* x, const float* a_in, float* a_out,
                                         float* m, const float* const* d, float* dout,
                                         const float* first_step_norm, float* lambda_out,
                                         double* M2_out, double* T_out, int64_t* nclipped);
extern "C" int co2_oracle_outer_step_variant_f32(int64_t n, int32_t S, const int64_t* seg_off, int32_t K,
                                                 float alpha, float beta, float phi, float c, int32_t tau,
                                                 int64_t step, int32_t nonstale, int32_t norm_clip,
                                                 float pull_rho, float* x, const float* a_in, float* a_out,
                                                 float* m, const float* const* d, float* dout,
                                                 const float* first_step_norm, float* lambda_out,
                                                 float* scale_out, int64_t* nclipped);

#define HIP_OK(call)                                                                      \
  do {                                                                                    \
    hipError_t e_ = (call);                                                               \
    if (e_ != hipSuccess) {                                                               \
      std::fprintf(stderr, "HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); \
      return 2;                                                                           \
    }                                                                                     \
  } while (0)

// splitmix64 -> uniform in (-1, 1): a tiny counter-based source of test data
static float unit(uint64_t key) {
  uint64_t z = key + 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  z ^= z >> 31;
  return static_cast<float>(static_cast<double>(z >> 11) / 4503599627370496.0 - 1.0);
}

static bool close(const std::vector<float>& got, const std::vector<float>& want, const char* what) {
  for (size_t j = 0; j < got.size(); ++j) {
    const double g = got[j], w = want[j];
    if (std::fabs(g - w) > 1e-5 * std::fabs(w)) {
      std::fprintf(stderr, "%s[%zu]: got %.9g want %.9g\n", what, j, g, w);
      return false;
    }
  }
  return true;
}

int main(int argc, char** argv) {
  const int64_t n = argc > 1 ? std::atoll(argv[1]) : 100003;
  const int32_t K = argc > 2 ? std::atoi(argv[2]) : 3;
  const bool use_set = argc > 3 && std::atoi(argv[3]) != 0;   // buffers from co2_buffer_set_create
  const int mode = argc > 4 ? std::atoi(argv[4]) : 0;
  const bool variant = mode == 2;
  if (n < 8 || K < 1 || K > CO2_MAX_K || mode < 0 || mode > 2) { std::fprintf(stderr, "bad arguments\n"); return 2; }
  const std::vector<int64_t> seg = {0, 5, 5, n / 3 + 1, n - 2, n};
  const int32_t S = static_cast<int32_t>(seg.size()) - 1;
  const float alpha = 0.9f, beta = 0.9f, phi = variant ? 2e-2f : 2e-3f, c = 1.0f, rho = 0.5f;
  const int32_t tau = 4;
  std::vector<float> fsn(S);
  for (int32_t s = 0; s < S; ++s) fsn[s] = 1e-3f * (1.0f + 0.25f * static_cast<float>(s));

  std::vector<float> a(n), x(n), m(n, 0.0f), dout(n), lam(S);
  std::vector<std::vector<float>> d(K, std::vector<float>(n, 0.0f));
  for (int64_t j = 0; j < n; ++j) a[j] = 0.02f * unit(j);

  float *da, *dx, *dm, *ddout[2], *dlam;
  int64_t* dseg;
  std::vector<float*> dd(K);
  void* ws;
  const size_t nb = sizeof(float) * static_cast<size_t>(n);
  const size_t wsb = co2_workspace_bytes(n, S, K);
  co2_buffer_set* set = nullptr;
  if (use_set) {
    // the flat vectors out of one piece-major buffer set (2 MiB pieces: several per buffer)
    const int32_t count = 5 + (K - 1);
    std::vector<size_t> sizes(count, nb);
    std::vector<void*> ptr(count, nullptr);
    const int rc = co2_buffer_set_create(count, sizes.data(), size_t(2) << 20, ptr.data(), &set);
    if (rc != CO2_OK) {
      std::fprintf(stderr, "co2_buffer_set_create: %s (hip %d)\n", co2_strerror(rc), co2_last_hip_error());
      return 1;
    }
    da = static_cast<float*>(ptr[0]); dx = static_cast<float*>(ptr[1]); dm = static_cast<float*>(ptr[2]);
    ddout[0] = static_cast<float*>(ptr[3]); ddout[1] = static_cast<float*>(ptr[4]);
    for (int k = 1; k < K; ++k) dd[k] = static_cast<float*>(ptr[4 + k]);
  } else {
    HIP_OK(hipMalloc(&da, nb)); HIP_OK(hipMalloc(&dx, nb)); HIP_OK(hipMalloc(&dm, nb));
    HIP_OK(hipMalloc(&ddout[0], nb)); HIP_OK(hipMalloc(&ddout[1], nb));
    for (int k = 1; k < K; ++k) HIP_OK(hipMalloc(&dd[k], nb));
  }
  float* dfsn;
  HIP_OK(hipMalloc(&dfsn, sizeof(float) * S));
  HIP_OK(hipMemcpy(dfsn, fsn.data(), sizeof(float) * S, hipMemcpyHostToDevice));
  HIP_OK(hipMalloc(&dlam, sizeof(float) * S)); HIP_OK(hipMalloc(&dseg, sizeof(int64_t) * (S + 1)));
  HIP_OK(hipMalloc(&ws, wsb));
  HIP_OK(hipMemcpy(da, a.data(), nb, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(dm, m.data(), nb, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(dseg, seg.data(), sizeof(int64_t) * (S + 1), hipMemcpyHostToDevice));
  HIP_OK(hipMemset(ddout[1], 0, nb));

  std::vector<float> got(n);
  for (int64_t t = 0; t < 4; ++t) {
    // inner loop stand-in: local params drift from the anchor; peers' deltas arrive
    // (with the anchor pull the local parameters carry over instead of restarting from the anchor)
    for (int64_t j = 0; j < n; ++j)
      x[j] = ((variant && t > 0) ? x[j] : a[j]) + 1e-3f * unit((uint64_t(t + 1) << 40) + j);
    for (int k = 1; k < K; ++k)
      for (int64_t j = 0; j < n; ++j) d[k][j] = 1e-3f * unit((uint64_t(100 + k) << 48) + (uint64_t(t) << 40) + j);
    HIP_OK(hipMemcpy(dx, x.data(), nb, hipMemcpyHostToDevice));
    for (int k = 1; k < K; ++k) HIP_OK(hipMemcpy(dd[k], d[k].data(), nb, hipMemcpyHostToDevice));
    dd[0] = ddout[(t + 1) % 2];                 // own pseudo-gradient of the previous round

    co2_params p = {};
    p.n = n; p.S = S; p.K = K; p.seg_off = seg.data(); p.seg_off_dev = dseg;
    p.alpha = alpha; p.beta = beta; p.clip_phi = phi; p.penalty_c = c; p.tau = tau;
    p.flags = t >= 2 ? CO2_FLAG_CARRIED_NORMS : CO2_FLAG_NONE; p.step = t;
    int rc;
    if (mode == 1) {
      rc = co2_outer_step_static(&p, dx, da, da, dm, dd.data(), ddout[t % 2], nullptr, dlam, nullptr);
    } else if (variant) {
      p.flags = (t >= 1 ? CO2_FLAG_CARRIED_NORMS : CO2_FLAG_NONE) | CO2_FLAG_CURRENT_ROUND |
                CO2_FLAG_ANCHOR_PULL | CO2_FLAG_NORM_CLIP;
      p.pull_rho = rho;
      dd[0] = nullptr;                          // not read in the current-round order
      rc = co2_outer_step(&p, dx, da, da, dm, dd.data(), ddout[t % 2], dfsn, dlam, ws, wsb, nullptr);
    } else {
      rc = co2_outer_step(&p, dx, da, da, dm, dd.data(), ddout[t % 2], nullptr, dlam, ws, wsb, nullptr);
    }
    if (rc != CO2_OK) { std::fprintf(stderr, "co2_outer_step: %s\n", co2_strerror(rc)); return 1; }
    HIP_OK(hipDeviceSynchronize());

    // the oracle carries its own state: a, x, m, d[0] (its own previous delta_out)
    std::vector<const float*> dp(K);
    for (int k = 0; k < K; ++k) dp[k] = d[k].data();
    const int orc = variant
        ? co2_oracle_outer_step_variant_f32(n, S, seg.data(), K, alpha, beta, phi, c, tau, t, 1, 1, rho,
                                            x.data(), a.data(), a.data(), m.data(), dp.data(), dout.data(),
                                            fsn.data(), lam.data(), nullptr, nullptr)
        : co2_oracle_outer_step_f32(n, S, seg.data(), K, alpha, beta, phi, c, tau, t, x.data(), a.data(),
                                    a.data(), m.data(), t ? dp.data() : nullptr, dout.data(), nullptr,
                                    lam.data(), nullptr, nullptr, nullptr);
    if (orc != 0) {
      std::fprintf(stderr, "oracle rejected its arguments\n");
      return 1;
    }
    bool ok = true;
    HIP_OK(hipMemcpy(got.data(), dx, nb, hipMemcpyDeviceToHost)); ok = ok && close(got, x, "params");
    HIP_OK(hipMemcpy(got.data(), da, nb, hipMemcpyDeviceToHost)); ok = ok && close(got, a, "anchor");
    HIP_OK(hipMemcpy(got.data(), dm, nb, hipMemcpyDeviceToHost)); ok = ok && close(got, m, "momentum");
    HIP_OK(hipMemcpy(got.data(), ddout[t % 2], nb, hipMemcpyDeviceToHost)); ok = ok && close(got, dout, "delta_out");
    if (t >= 1 || variant) {
      std::vector<float> glam(S);
      HIP_OK(hipMemcpy(glam.data(), dlam, sizeof(float) * S, hipMemcpyDeviceToHost));
      ok = ok && close(glam, lam, "Lambda");
    }
    if (!ok) { std::fprintf(stderr, "round %lld: mismatch\n", static_cast<long long>(t)); return 1; }
    d[0] = dout;
    std::printf("round %lld ok\n", static_cast<long long>(t));
    std::fflush(stdout);
  }
  // argument errors come back as codes, nothing is launched
  co2_params bad = {};
  if (co2_outer_step(&bad, dx, da, da, dm, dd.data(), ddout[0], nullptr, nullptr, ws, wsb, nullptr) != CO2_EINVAL) return 1;
  if (set) {
    HIP_OK(hipDeviceSynchronize());
    if (co2_buffer_set_destroy(set) != CO2_OK) { std::fprintf(stderr, "co2_buffer_set_destroy failed\n"); return 1; }
  }
  std::printf("PASS n=%lld K=%d buffers=%s entry=%s\n", static_cast<long long>(n), K,
              use_set ? "buffer set" : "hipMalloc",
              mode == 1 ? "co2_outer_step_static" : variant ? "co2_outer_step, variant switches" : "co2_outer_step");
  return 0;
}
