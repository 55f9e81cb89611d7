// Token assignment for callers that cannot allocate device memory (code under HIP graph capture, tight
// serving loops, harnesses that forbid hipMalloc): si_route_noalloc is si_route with its temporary idx / w
// tables taken from a fixed file-scope device array instead of a stream-ordered allocation.
#include <mutex>

#include "si_internal.h"
#include "si_error.h"

using namespace si;

namespace {

// idx [pairs] i32 followed by w [pairs] f32; every GPU the library runs on holds its own copy until the process ends
constexpr size_t SCRATCH_BYTES = (size_t)2 * SI_ROUTE_NOALLOC_MAX_PAIRS * 4;
static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_mu;
void* g_scratch_ptr[MAX_DEVICES] = {};  // device address of `scratch` on each device (the array's name is only a host-side handle)

// address of this device's copy of the array; looked up once per device, with that device current
int scratch_of_current_device(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return set_error(SI_EHIP, "hipGetDevice failed: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= MAX_DEVICES) return set_error(SI_ESTATE, "device ordinal %d outside [0, %d)", dev, MAX_DEVICES);
  std::lock_guard<std::mutex> lk(g_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return set_error(SI_EHIP, "hipGetSymbolAddress(scratch) failed on device %d: %s", dev, hipGetErrorString(e));
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return SI_OK;
}

}  // namespace

extern "C" int si_route_noalloc(const float* logits_dev, int32_t T, int32_t E, int32_t k, const si_routing_out_t* out,
                                void* stream) {
  if (!logits_dev || !out) return set_error(SI_EINVAL, "logits_dev or out is NULL");
  if (T < 0 || E < 1 || E > MAX_EXPERTS || k < 1 || k > E) return set_error(SI_EINVAL, "bad T=%d E=%d k=%d", T, E, k);
  if ((long long)T * k > (long long)SI_ROUTE_NOALLOC_MAX_PAIRS)
    return set_error(SI_EINVAL, "si_route_noalloc: T*k = %lld exceeds the fixed scratch of %d (token, slot) pairs",
                     (long long)T * k, SI_ROUTE_NOALLOC_MAX_PAIRS);
  if (T == 0) return SI_OK;
  void* base = nullptr;
  if (int rc = scratch_of_current_device(&base)) return rc;
  // the tables are written in full by the selection kernel before anything reads them: nothing to clear
  int32_t* s_idx = static_cast<int32_t*>(base);
  float* s_w = reinterpret_cast<float*>(s_idx + SI_ROUTE_NOALLOC_MAX_PAIRS);
  Plan p{};
  p.idx = out->idx ? out->idx : s_idx;
  p.w = out->w ? out->w : s_w;
  RouteOut u{nullptr, nullptr, out->count, out->off, out->perm, out->inv};
  hipError_t e = launch_route(logits_dev, T, E, k, 0, 0, p, u, (hipStream_t)stream);
  if (e != hipSuccess) return set_error(SI_EHIP, "route launch failed: %s", hipGetErrorString(e));
  return SI_OK;
}
