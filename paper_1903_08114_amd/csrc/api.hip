// C ABI of libegp: argument validation, workspace carving and launch sequencing.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <cmath>

#include "egp_internal.h"

namespace egp {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

int validate_ptr(const void* p, const char* name) {
  if (p == nullptr) return fail(EGP_ERR_ARG, "%s is NULL", name);
  if ((reinterpret_cast<uintptr_t>(p) & 15u) != 0) return fail(EGP_ERR_ARG, "%s is not 16-byte aligned", name);
  return EGP_OK;
}

int validate_hyper(const egp_hyper_t* h) {
  if (h == nullptr) return fail(EGP_ERR_ARG, "hyper-parameter struct is NULL");
  if (h->kernel_type < EGP_RBF || h->kernel_type > EGP_MATERN52)
    return fail(EGP_ERR_ARG, "unknown kernel_type %d", h->kernel_type);
  if (h->d < 1 || h->d > EGP_D_MAX) return fail(EGP_ERR_ARG, "d = %d outside 1..%d", h->d, EGP_D_MAX);
  if (h->lengthscales == nullptr) return fail(EGP_ERR_ARG, "lengthscales is NULL");
  for (int k = 0; k < h->d; ++k)
    if (!(h->lengthscales[k] > 0.f) || !std::isfinite(h->lengthscales[k]))
      return fail(EGP_ERR_ARG, "lengthscale %d is not a positive finite number", k);
  if (!(h->outputscale > 0.f) || !std::isfinite(h->outputscale))
    return fail(EGP_ERR_ARG, "outputscale must be positive and finite");
  if (!(h->noise >= 0.f) || !std::isfinite(h->noise)) return fail(EGP_ERR_ARG, "noise must be >= 0 and finite");
  if (ksteps_for(h->d) > 8)
    return fail(EGP_ERR_ARG, "d = %d: this build's fused kernel supports d <= 31", h->d);
  return EGP_OK;
}

}  // namespace egp

using namespace egp;

extern "C" {

const char* egp_last_error(void) { return g_err; }
const char* egp_version(void) { return "0.1"; }

size_t egp_kmm_ws_bytes(int64_t n, int32_t d, int32_t t) {
  if (n < 1 || d < 1 || d > EGP_D_MAX || t < 1 || t > EGP_T_MAX) return 0;
  return prepared_bytes(n, d) + kmm_core_ws_bytes(n, t);
}

int egp_kmm(const float* X, int64_t n, const float* V, int32_t t, const egp_hyper_t* h, float* out, void* ws,
            size_t ws_bytes, void* stream) {
  int rc;
  if ((rc = validate_hyper(h)) != EGP_OK) return rc;
  if (n < 1 || n > ((int64_t)1 << 31)) return fail(EGP_ERR_ARG, "n = %lld outside 1..2^31", (long long)n);
  if (t < 1 || t > EGP_T_MAX) return fail(EGP_ERR_ARG, "t = %d outside 1..%d", t, EGP_T_MAX);
  if ((rc = validate_ptr(X, "X")) != EGP_OK) return rc;
  if ((rc = validate_ptr(V, "V")) != EGP_OK) return rc;
  if ((rc = validate_ptr(out, "out")) != EGP_OK) return rc;
  if ((rc = validate_ptr(ws, "ws")) != EGP_OK) return rc;
  if (out == V) return fail(EGP_ERR_ARG, "out must not alias V");
  const size_t need = egp_kmm_ws_bytes(n, h->d, t);
  if (ws_bytes < need) return fail(EGP_ERR_WS, "workspace of %zu bytes is smaller than the %zu needed", ws_bytes, need);
  hipStream_t s = static_cast<hipStream_t>(stream);
  Prepared P;
  if ((rc = prepare_points(X, n, h, ws, &P, s)) != EGP_OK) return rc;
  return kmm_core(P, V, t, out, static_cast<char*>(ws) + prepared_bytes(n, h->d), s);
}

}  // extern "C"
