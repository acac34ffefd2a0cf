// egp_kmm_noalloc: the fused kernel-matrix multiply for callers that cannot allocate device memory (code under HIP
// graph capture, tight serving loops, harnesses that forbid hipMalloc). Its workspace -- packed points, packed
// right-hand sides, per-split partial sums, the int64 column-side slab of the symmetric kernels -- is a file-scope
// device array of fixed size instead of a buffer the caller provides. The kernels are egp_kmm's own; they receive the
// array's device address as their workspace pointer exactly as they receive a caller's buffer.
#include <mutex>

#include "egp_internal.h"

namespace {

// One copy per GPU the library runs on, held until the process ends. Zero-initialised storage: it takes no room
// in the library file.
static __device__ __align__(256) unsigned char scratch[EGP_NOALLOC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
void* g_scratch_ptr[kMaxDevices] = {};      // device address of `scratch` on each device, looked up once per device

// In host code the name `scratch` is only a handle for the symbol, not a device address: the address of the
// current device's copy comes from hipGetSymbolAddress, and that address is what kernels and copies are given.
int scratch_of_current_device(void** out) {
  int dev = -1;
  EGP_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return egp::fail(EGP_ERR_DEVICE, "device index %d outside 0..%d", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lk(g_mu);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    EGP_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (p == nullptr) return egp::fail(EGP_ERR_DEVICE, "hipGetSymbolAddress returned a null address for the scratch array");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return EGP_OK;
}

}  // namespace

extern "C" int egp_kmm_noalloc(const float* X, int64_t n, const float* V, int32_t t, const egp_hyper_t* h, float* out,
                               void* stream) {
  // sizes first: the workspace query is host arithmetic and returns 0 for sizes outside the library's limits
  if (h == nullptr) return egp::fail(EGP_ERR_ARG, "hyper-parameter struct is NULL");
  const size_t need = egp_kmm_ws_bytes(n, h->d, t);
  if (need == 0) return egp::fail(EGP_ERR_ARG, "n = %lld, d = %d or t = %d outside the library's limits", (long long)n, h->d, t);
  if (need > (size_t)EGP_NOALLOC_SCRATCH_BYTES)
    return egp::fail(EGP_ERR_ARG,
                     "egp_kmm_noalloc: n = %lld, d = %d, t = %d needs %zu bytes of workspace, the built-in scratch array "
                     "holds %zu; use egp_kmm with a caller-provided workspace",
                     (long long)n, h->d, t, need, (size_t)EGP_NOALLOC_SCRATCH_BYTES);
  void* ws = nullptr;
  if (int rc = scratch_of_current_device(&ws)) return rc;
  // every buffer the kernels expect at zero (the column-side slab) is cleared by egp_kmm's own fill kernels, so the
  // previous call's contents do not matter
  return egp_kmm(X, n, V, t, h, out, ws, (size_t)EGP_NOALLOC_SCRATCH_BYTES, stream);
}
