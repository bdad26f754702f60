// lsam_step_grads_static: the raw-vector iteration of lsam_step_grads for callers that cannot
// allocate (code under HIP graph capture, tight serving loops, harnesses that forbid
// hipMalloc).  All state is the caller's; the only device memory beyond inputs and outputs --
// the partial sums of squares of the gradient-norm reduction, the norms and the perturbation
// scales -- lives in a file-scope device array of fixed size, one copy per GPU, resolved to a
// device address once per device.  No hipMalloc, hipFree or allocating library call is made.
#include <mutex>

#include "engine.h"

namespace lsam {
namespace {

constexpr int kMaxBlocks = 1024;                    // partial sums per replica at most
constexpr int kMaxDevices = 64;
constexpr size_t kPartialBytes = (size_t)kMaxK * kMaxBlocks * sizeof(double);   // 512 KiB
constexpr size_t kScratchBytes = kPartialBytes + 2 * kMaxK * sizeof(float);     // + norms, scales

// Host code never passes this name to a kernel: it is a stand-in on the host side.  The device
// address of each GPU's copy comes from hipGetSymbolAddress below.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

std::mutex g_lock;
void* g_scratch_ptr[kMaxDevices] = {nullptr};

thread_local char g_msg[256];

int report(int code) {
  set_last_error(g_msg);
  return code;
}

// Device address of the current device's copy of `scratch` (looked up on first use per device).
int scratch_for_current_device(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) {
    snprintf(g_msg, sizeof g_msg, "hipGetDevice: %s", hipGetErrorString(e));
    return report(LSAM_EHIP);
  }
  if (dev < 0 || dev >= kMaxDevices) {
    snprintf(g_msg, sizeof g_msg, "device index %d beyond the %d this entry point keeps track of", dev,
             kMaxDevices);
    return report(LSAM_EINVAL);
  }
  std::lock_guard<std::mutex> hold(g_lock);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || p == nullptr) {
      snprintf(g_msg, sizeof g_msg, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
      return report(LSAM_EHIP);
    }
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return LSAM_OK;
}

}  // namespace

}  // namespace lsam

using namespace lsam;

extern "C" int lsam_step_grads_static(const lsam_update_desc* u, float* x, float* v, float* S,
                                      const float* y, const float* g1, const float* g2, float* xt,
                                      float* norms_out, void* stream) {
  auto bad = [](const char* why) {
    set_last_error(why);
    return LSAM_EINVAL;
  };
  if (!u || !x || !v || !S || !y || !g1 || !g2) return bad("NULL argument");
  if (u->K < 1 || u->K > LSAM_MAX_REPLICAS) return bad("K outside 1..LSAM_MAX_REPLICAS");
  if (u->d < 1 || u->d > LSAM_STATIC_MAX_D) return bad("d outside 1..LSAM_STATIC_MAX_D");
  if (u->stride < u->d || u->g_stride < u->d) return bad("row strides must be >= d");
  if (!u->lambda) return bad("lambda is NULL");
  if (!(u->rho >= 0.f) || !(u->gamma >= 0.f) || !(u->lr >= 0.f) || !(u->momentum >= 0.f && u->momentum < 1.f))
    return bad("rho, gamma, lr must be >= 0 and momentum in [0, 1)");
  if (u->rho != 0.f && !xt) return bad("xt is NULL although rho > 0");
  const uintptr_t align = reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(v) |
                          reinterpret_cast<uintptr_t>(S) | reinterpret_cast<uintptr_t>(y) |
                          reinterpret_cast<uintptr_t>(xt);
  if ((align & 15) || (u->stride % 4)) return bad("x, v, S, y, xt must be 16-byte aligned with a row stride that is a multiple of 4");
  if ((reinterpret_cast<uintptr_t>(g1) & 3) || (reinterpret_cast<uintptr_t>(g2) & 3))
    return bad("gradients must be 4-byte aligned");

  void* base = nullptr;
  int rc = scratch_for_current_device(&base);
  if (rc != LSAM_OK) return rc;
  double* partials = static_cast<double*>(base);
  float* norms = reinterpret_cast<float*>(static_cast<char*>(base) + kPartialBytes);
  float* scale = norms + kMaxK;
  if (norms_out) norms = norms_out;       // the caller's array takes the norms directly

  hipStream_t s = static_cast<hipStream_t>(stream);
  const int K = u->K;
  const int64_t d = u->d;
  // as many partial sums per replica as the context-based call uses for the same d
  int64_t nb = ((d + 63) / 64 * 64 + 65535) / 65536;
  const int nblk = (int)(nb < 1 ? 1 : (nb > kMaxBlocks ? kMaxBlocks : nb));
  // every slot that is read below is written first, so nothing of an earlier call is seen
  launch_sumsq_partials(g1, u->g_stride, d, K, partials, nblk, s);
  launch_norm_finish(partials, nblk, nblk, K, u->rho, u->gamma, norms, scale, nullptr, 0, nullptr, s);
  if (u->rho != 0.f)
    launch_perturb(x, g1, u->g_stride, scale, xt, nullptr, nullptr, 0, u->stride, d, K, s);
  ReplicaScalars lam;
  for (int i = 0; i < K; ++i) lam.v[i] = u->lambda[i];
  launch_descent(x, g2, u->g_stride, v, S, y, nullptr, nullptr, 0, u->stride, d, K, lam, u->lr,
                 u->momentum, u->nesterov, nullptr, s);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    set_last_error(hipGetErrorString(e));
    return LSAM_EHIP;
  }
  return LSAM_OK;
}
