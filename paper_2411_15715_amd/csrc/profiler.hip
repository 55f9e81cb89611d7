// Profiler half of the Profiler & Solver (Section III-D; measurements as in Section V-B / Table I):
// times GPU GEMMs, CPU GEMMs, host->device copies and kernel launches on this machine over a range
// of sizes and fits the linear models of Eq. 3.  GEMM times are taken from the library's own layer
// (a fully resident and a fully host-side dense layer of growing hidden size), so the fitted
// coefficients describe exactly the kernels and workers that the sliced layer will run.
#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstring>
#include <thread>
#include <vector>

#include <hip/hip_runtime.h>

#include "scheinfer_solver.h"
#include "si_error.h"

namespace {

using si::set_error;

#define PROF_HIP(expr)                                                                                   \
  do {                                                                                                   \
    hipError_t _e = (expr);                                                                              \
    if (_e != hipSuccess) { rc = set_error(SI_EHIP, "%s failed: %s", #expr, hipGetErrorString(_e)); goto done; } \
  } while (0)

__global__ void k_empty() {}

// bf16 patterns of small pseudo-random values in (-2^-4, 2^-4): sign, exponent 115..122, 7 mantissa bits
void fill_weights(uint16_t* w, size_t n, uint32_t seed, int threads) {
  auto body = [=](int tid) {
    const size_t lo = n * tid / threads, hi = n * (tid + 1) / threads;
    uint64_t s = 0x9E3779B97F4A7C15ull * (seed + 1) + 0xD1B54A32D192ED03ull * (uint64_t)(tid + 1);
    for (size_t i = lo; i < hi; ++i) {
      s = s * 6364136223846793005ull + 1442695040888963407ull;
      const uint32_t r = (uint32_t)(s >> 33);
      w[i] = (uint16_t)(((r & 1u) << 15) | ((115u + ((r >> 1) & 7u)) << 7) | ((r >> 4) & 0x7Fu));
    }
  };
  std::vector<std::thread> th;
  for (int t = 1; t < threads; ++t) th.emplace_back(body, t);
  body(0);
  for (auto& t : th) t.join();
}

double median(std::vector<double> v) {
  std::sort(v.begin(), v.end());
  const size_t n = v.size();
  return n % 2 ? v[n / 2] : 0.5 * (v[n / 2 - 1] + v[n / 2]);
}

// Median over `reps` forward calls of a dense layer of hidden size h placed entirely on the GPU
// (gpu = true: seconds in the gate/up and down kernels) or on the host (seconds in the CC workers).
int time_layer(const si_profile_desc_t& d, int mode, int h, bool gpu, const uint16_t* wg, const uint16_t* wu,
               const uint16_t* wd, const si_q4_weights_t* q4, const void* x_dev, float* y_dev, int reps, double* seconds) {
  si_layer_desc_t ld;
  std::memset(&ld, 0, sizeof ld);
  ld.d_model = d.d_model;
  ld.d_ff = h;
  ld.n_experts = 1;
  ld.top_k = 1;
  ld.r_gg = gpu ? 1.f : 0.f;
  ld.r_cc = gpu ? 0.f : 1.f;
  ld.max_tokens = d.tokens;
  ld.cc_threads = d.cc_threads;
  ld.device = d.device;
  ld.stage_mib = 1;
  si_layer_t* L = nullptr;
  // the first h rows of the [d_ff][..] arrays are a layer of hidden size h in either storage form
  int rc = q4 ? si_layer_create_q4(&ld, q4, nullptr, nullptr, &L) : si_layer_create(&ld, wg, wu, wd, nullptr, nullptr, nullptr, &L);
  if (rc != SI_OK) return rc;
  std::vector<double> samples;
  rc = si_layer_set_profiling(L, 1);
  for (int i = 0; rc == SI_OK && i < reps + 2; ++i) {
    rc = si_layer_forward(L, x_dev, nullptr, d.tokens, 0, mode, y_dev, nullptr, nullptr);
    si_stats_t st;
    if (rc == SI_OK) rc = si_layer_stats(L, &st);
    if (rc == SI_OK && i >= 2) {
      if (gpu) {
        const int a = mode == SI_DECODE ? SI_K_DECODE_GATEUP : SI_K_PREFILL_GATEUP;
        const int b = mode == SI_DECODE ? SI_K_DECODE_DOWN : SI_K_PREFILL_DOWN;
        samples.push_back(1e-3 * ((double)st.kernel_ms[a] + (double)st.kernel_ms[b]));
      } else {
        samples.push_back(1e-3 * (double)st.cc_ms);
      }
    }
  }
  si_layer_destroy(L);
  if (rc == SI_OK) *seconds = median(samples);
  return rc;
}

}  // namespace

extern "C" int si_profile(const si_profile_desc_t* desc, si_profile_result_t* out) {
  if (!desc || !out) return set_error(SI_EINVAL, "si_profile: NULL pointer");
  si_profile_desc_t d = *desc;
  if (d.n_sizes == 0) d.n_sizes = 6;
  if (d.reps == 0) d.reps = 5;
  if (d.copy_max_mib == 0) d.copy_max_mib = 256;
  if (d.d_model < 64 || d.d_model % 64 || d.d_ff < 64 || d.d_ff % 64 || d.tokens < 1)
    return set_error(SI_EINVAL, "si_profile: d_model and d_ff must be positive multiples of 64, tokens >= 1");
  if (d.n_sizes < 2 || d.n_sizes > SI_PROFILE_MAX_SIZES || d.reps < 1 || d.copy_max_mib < 1 || d.copy_max_mib > 4096)
    return set_error(SI_EINVAL, "si_profile: n_sizes in 2..%d, reps >= 1, copy_max_mib in 1..4096", SI_PROFILE_MAX_SIZES);
  int mode = d.mode;
  if (mode == SI_AUTO) mode = d.tokens <= SI_DECODE_AUTO_ROWS ? SI_DECODE : SI_PREFILL;  // a dense layer: rows = tokens
  if (mode != SI_DECODE && mode != SI_PREFILL) return set_error(SI_EINVAL, "si_profile: bad mode");
  if (mode == SI_DECODE && d.tokens > SI_DECODE_MAX_T) return set_error(SI_EINVAL, "si_profile: decode path takes at most %d tokens", SI_DECODE_MAX_T);
  // distinct hidden sizes h_i = d_ff*(i+1)/n_sizes rounded down to 64 columns
  std::vector<int> hs;
  for (int i = 0; i < d.n_sizes; ++i) {
    int h = (int)((int64_t)d.d_ff * (i + 1) / d.n_sizes) / 64 * 64;
    if (h >= 64 && (hs.empty() || h > hs.back())) hs.push_back(h);
  }
  if (hs.size() < 2) return set_error(SI_EINVAL, "si_profile: d_ff too small for two distinct sizes");

  std::memset(out, 0, sizeof *out);
  int rc = SI_OK;
  const size_t wn = (size_t)d.d_ff * d.d_model;
  const size_t copy_max = (size_t)d.copy_max_mib << 20;
  std::vector<uint16_t> wg, wu, wd;
  std::vector<uint8_t> qg, qu, qd;   // 4-bit form: any byte is a valid pair of codes
  std::vector<uint16_t> zg, zu, zd;
  si_q4_weights_t q4w{};
  void* x_dev = nullptr;
  float* y_dev = nullptr;
  void* pin = nullptr;
  void* dev = nullptr;
  hipStream_t stream = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  const int np = (int)hs.size();
  {
    PROF_HIP(hipSetDevice(d.device));
    const int threads = (int)std::max(1u, std::min(16u, std::thread::hardware_concurrency()));
    if (!d.q4) {
      wg.resize(wn);
      wu.resize(wn);
      wd.resize(wn);
      fill_weights(wg.data(), wn, d.seed * 3 + 0, threads);
      fill_weights(wu.data(), wn, d.seed * 3 + 1, threads);
      fill_weights(wd.data(), wn, d.seed * 3 + 2, threads);
    } else {
      // codes: the bytes of pseudo-random bf16 patterns; scales: small positive bf16 values (sign bit cleared).
      // z_down is [d_ff/64][d_model]: its first h/64 rows belong to the first h hidden columns.
      std::vector<uint16_t> tmp(wn / 4);
      for (auto* q : {&qg, &qu, &qd}) {
        fill_weights(tmp.data(), tmp.size(), d.seed * 3 + (uint32_t)(q - &qg) + 11, threads);
        q->resize(wn / 2);
        std::memcpy(q->data(), tmp.data(), wn / 2);
      }
      zg.resize(wn / 64);
      zu.resize(wn / 64);
      zd.resize(wn / 64);
      fill_weights(zg.data(), zg.size(), d.seed * 3 + 21, 1);
      fill_weights(zu.data(), zu.size(), d.seed * 3 + 22, 1);
      fill_weights(zd.data(), zd.size(), d.seed * 3 + 23, 1);
      for (auto* z : {&zg, &zu, &zd})
        for (auto& v : *z) v &= 0x7fffu;
      q4w = si_q4_weights_t{qg.data(), qu.data(), qd.data(), zg.data(), zu.data(), zd.data()};
    }
    std::vector<uint16_t> xh((size_t)d.tokens * d.d_model);
    fill_weights(xh.data(), xh.size(), d.seed * 3 + 7, 1);
    for (auto& v : xh) v = (uint16_t)(v + (4u << 7));  // activations 16 times larger than the weights
    PROF_HIP(hipMalloc(&x_dev, xh.size() * 2));
    PROF_HIP(hipMalloc((void**)&y_dev, (size_t)d.tokens * d.d_model * sizeof(float)));
    PROF_HIP(hipMemcpy(x_dev, xh.data(), xh.size() * 2, hipMemcpyHostToDevice));

    // GPU GEMM and CPU GEMM (Eq. 3, first two lines)
    for (int i = 0; i < np; ++i) {
      out->n_gemm[i] = (double)d.tokens * d.d_model * hs[i];
      double s = 0.0;
      rc = time_layer(d, mode, hs[i], true, wg.data(), wu.data(), wd.data(), d.q4 ? &q4w : nullptr, x_dev, y_dev, d.reps, &s);
      if (rc != SI_OK) goto done;
      out->t_g[i] = s / 3.0;
      rc = time_layer(d, mode, hs[i], false, wg.data(), wu.data(), wd.data(), d.q4 ? &q4w : nullptr, x_dev, y_dev, d.reps, &s);
      if (rc != SI_OK) goto done;
      out->t_c[i] = s / 3.0;
    }
    out->n_points = np;

    // host -> device copies from pinned memory (Eq. 3, third line)
    PROF_HIP(hipHostMalloc(&pin, copy_max, hipHostMallocDefault));
    std::memset(pin, 0x3c, copy_max);
    PROF_HIP(hipMalloc(&dev, copy_max));
    PROF_HIP(hipStreamCreateWithFlags(&stream, hipStreamNonBlocking));
    PROF_HIP(hipEventCreate(&e0));
    PROF_HIP(hipEventCreate(&e1));
    {
      const double lo = 256.0 * 1024.0, hi = (double)copy_max;
      for (int i = 0; i < np; ++i) {
        size_t bytes = (size_t)(lo * std::pow(hi / lo, np > 1 ? (double)i / (np - 1) : 1.0));
        bytes = std::min(copy_max, std::max<size_t>(4096, bytes / 4096 * 4096));
        std::vector<double> samples;
        for (int r = 0; r < d.reps + 1; ++r) {
          PROF_HIP(hipEventRecord(e0, stream));
          PROF_HIP(hipMemcpyAsync(dev, pin, bytes, hipMemcpyHostToDevice, stream));
          PROF_HIP(hipEventRecord(e1, stream));
          PROF_HIP(hipEventSynchronize(e1));
          float ms = 0.f;
          PROF_HIP(hipEventElapsedTime(&ms, e0, e1));
          if (r >= 1) samples.push_back(1e-3 * (double)ms);
        }
        out->bytes[i] = (double)bytes;
        out->t_c2g[i] = median(samples);
      }
    }

    // launch time: host time per launch of an empty kernel, batches of 200 (Eq. 3, last line)
    {
      const int batches = 20, per = 200;
      std::vector<double> per_launch;
      for (int b = 0; b < batches + 1; ++b) {
        PROF_HIP(hipStreamSynchronize(stream));
        const auto t0 = std::chrono::steady_clock::now();
        for (int i = 0; i < per; ++i) hipLaunchKernelGGL(k_empty, dim3(1), dim3(64), 0, stream);
        const auto t1 = std::chrono::steady_clock::now();
        PROF_HIP(hipGetLastError());
        if (b >= 1) per_launch.push_back(std::chrono::duration<double>(t1 - t0).count() / per);
      }
      PROF_HIP(hipStreamSynchronize(stream));
      double mean = 0.0, var = 0.0;
      for (double v : per_launch) mean += v;
      mean /= per_launch.size();
      for (double v : per_launch) var += (v - mean) * (v - mean);
      out->model.t_launch = mean;
      out->sigma_launch = std::sqrt(var / per_launch.size());
    }

    rc = si_fit_linear(out->n_gemm, out->t_g, np, 1, &out->model.alpha_g, &out->model.beta_g, &out->r2_g);
    if (rc == SI_OK) rc = si_fit_linear(out->n_gemm, out->t_c, np, 1, &out->model.alpha_c, &out->model.beta_c, &out->r2_c);
    if (rc == SI_OK) rc = si_fit_linear(out->bytes, out->t_c2g, np, 1, &out->model.alpha_c2g, &out->model.beta_c2g, &out->r2_c2g);
  }
done:
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (stream) (void)hipStreamDestroy(stream);
  if (dev) (void)hipFree(dev);
  if (pin) (void)hipHostFree(pin);
  if (y_dev) (void)hipFree(y_dev);
  if (x_dev) (void)hipFree(x_dev);
  return rc;
}
