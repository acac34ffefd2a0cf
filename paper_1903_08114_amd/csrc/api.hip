// C ABI of libegp: argument validation, workspace carving and launch sequencing.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <atomic>
#include <cmath>
#include <mutex>
#include <vector>

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

int validate_hyper(const egp_hyper_t* h, int d_max) {
  if (h == nullptr) return fail(EGP_ERR_ARG, "hyper-parameter struct is NULL");
  if (h->kernel_type < EGP_RBF || h->kernel_type > EGP_MATERN12)
    return fail(EGP_ERR_ARG, "unknown kernel_type %d", h->kernel_type);
  if (h->d < 1 || h->d > d_max) return fail(EGP_ERR_ARG, "d = %d outside 1..%d for this entry point", h->d, d_max);
  if (h->lengthscales == nullptr) return fail(EGP_ERR_ARG, "lengthscales is NULL");
  for (int k = 0; k < h->d; ++k)
    if (!(h->lengthscales[k] > 0.f) || !std::isfinite(h->lengthscales[k]))
      return fail(EGP_ERR_ARG, "lengthscale %d is not a positive finite number", k);
  if (!(h->outputscale > 0.f) || !std::isfinite(h->outputscale))
    return fail(EGP_ERR_ARG, "outputscale must be positive and finite");
  if (!(h->noise >= 0.f) || !std::isfinite(h->noise)) return fail(EGP_ERR_ARG, "noise must be >= 0 and finite");
  return EGP_OK;
}

// Process-wide defaults of the per-call options. They are read exactly once per library call, by resolve_opts() at
// the extern "C" entry point; everything below works on the CallOpts copy it returns.
static std::atomic<int> g_kmm_mode{EGP_KMM_FP32};
static std::atomic<int> g_mbcg_shrink{0};

static int resolve_opts(const egp_call_opts_t* o, CallOpts* co) {
  co->mode = g_kmm_mode.load();
  co->shrink = g_mbcg_shrink.load() != 0;
  if (o == nullptr) return EGP_OK;
  if (o->kmm_mode != -1) {
    if (o->kmm_mode < EGP_KMM_FP32 || o->kmm_mode > EGP_KMM_FP32_ONE_SIDED)
      return fail(EGP_ERR_ARG, "unknown kmm mode %d in the call options", o->kmm_mode);
    co->mode = o->kmm_mode;
  }
  if (o->mbcg_shrink != -1) {
    if (o->mbcg_shrink != 0 && o->mbcg_shrink != 1)
      return fail(EGP_ERR_ARG, "mbcg_shrink = %d in the call options (0, 1 or -1)", o->mbcg_shrink);
    co->shrink = o->mbcg_shrink == 1;
  }
  return EGP_OK;
}

// ---- profiling: event pairs kept until egp_profile_read drains them ----
struct ProfSlot { hipEvent_t a, b; };
static std::mutex g_prof_mu;
static bool g_prof_on = false;
static std::vector<ProfSlot> g_prof[kProfTags];
static double g_prof_ms[kProfTags];
static long g_prof_n[kProfTags];

ProfScope::ProfScope(int tag, hipStream_t stream) : tag_(tag), stream_(stream), slot_(nullptr) {
  if (!g_prof_on) return;
  ProfSlot* s = new ProfSlot;
  if (hipEventCreate(&s->a) != hipSuccess || hipEventCreate(&s->b) != hipSuccess) {
    delete s;
    return;
  }
  (void)hipEventRecord(s->a, stream);
  slot_ = s;
}

ProfScope::~ProfScope() {
  if (slot_ == nullptr) return;
  ProfSlot* s = static_cast<ProfSlot*>(slot_);
  (void)hipEventRecord(s->b, stream_);
  std::lock_guard<std::mutex> lk(g_prof_mu);
  g_prof[tag_].push_back(*s);
  delete s;
}

static void prof_drain() {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  for (int t = 0; t < kProfTags; ++t) {
    for (ProfSlot& s : g_prof[t]) {
      float ms = 0.f;
      if (hipEventSynchronize(s.b) == hipSuccess && hipEventElapsedTime(&ms, s.a, s.b) == hipSuccess) {
        g_prof_ms[t] += ms;
        g_prof_n[t] += 1;
      }
      (void)hipEventDestroy(s.a);
      (void)hipEventDestroy(s.b);
    }
    g_prof[t].clear();
  }
}

__global__ __launch_bounds__(256) void calib_copy_kernel(const float4* __restrict__ src, float4* __restrict__ dst,
                                                        int64_t count4) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count4; i += (int64_t)gridDim.x * 256)
    dst[i] = src[i];
}

}  // namespace egp

using namespace egp;

extern "C" {

const char* egp_last_error(void) { return g_err; }
const char* egp_version(void) { return "0.1"; }

int egp_set_kmm_mode(int32_t mode) {
  if (mode < EGP_KMM_FP32 || mode > EGP_KMM_FP32_ONE_SIDED) return fail(EGP_ERR_ARG, "unknown kmm mode %d", mode);
  g_kmm_mode.store(mode);
  return EGP_OK;
}
int egp_get_kmm_mode(void) { return g_kmm_mode.load(); }

int egp_set_mbcg_shrink(int32_t on) {
  g_mbcg_shrink.store(on ? 1 : 0);
  return EGP_OK;
}
int egp_get_mbcg_shrink(void) { return g_mbcg_shrink.load(); }

int egp_kmm_plan_splits_ex(int64_t n_rows, int64_t n_cols, int32_t d, int32_t t, const egp_call_opts_t* opts,
                           int32_t* used, int32_t* sized) {
  CallOpts co;
  int rc;
  if ((rc = resolve_opts(opts, &co)) != EGP_OK) return rc;
  if (n_rows < 1 || n_cols < 1 || d < 1 || d > EGP_D_WIDE_MAX || t < 1 || t > EGP_T_MAX || !used || !sized)
    return fail(EGP_ERR_ARG, "egp_kmm_plan_splits: size out of range or null output");
  int u = 0, s = 0;
  kmm_plan_splits(n_rows, n_cols, d, t, co.mode, &u, &s);
  *used = u;
  *sized = s;
  return EGP_OK;
}
int egp_kmm_plan_splits(int64_t n_rows, int64_t n_cols, int32_t d, int32_t t, int32_t* used, int32_t* sized) {
  return egp_kmm_plan_splits_ex(n_rows, n_cols, d, t, nullptr, used, sized);
}

int egp_calib_copy(const float* src, float* dst, int64_t count, void* stream) {
  int rc;
  if ((rc = validate_ptr(src, "src")) != EGP_OK) return rc;
  if ((rc = validate_ptr(dst, "dst")) != EGP_OK) return rc;
  if (count < 4 || (count & 3) != 0) return fail(EGP_ERR_ARG, "count must be a positive multiple of 4");
  hipLaunchKernelGGL(calib_copy_kernel, dim3(4096), dim3(256), 0, static_cast<hipStream_t>(stream),
                     reinterpret_cast<const float4*>(src), reinterpret_cast<float4*>(dst), count / 4);
  EGP_HIP(hipGetLastError());
  return EGP_OK;
}

int egp_profile_enable(int on) {
  prof_drain();
  std::lock_guard<std::mutex> lk(g_prof_mu);
  g_prof_on = on != 0;
  for (int t = 0; t < kProfTags; ++t) {
    g_prof_ms[t] = 0.0;
    g_prof_n[t] = 0;
  }
  return EGP_OK;
}

int egp_profile_read(int32_t group, double* total_ms, int64_t* launches) {
  if (group < 0 || group >= kProfTags) return fail(EGP_ERR_ARG, "profile group %d outside 0..%d", group, kProfTags - 1);
  prof_drain();
  std::lock_guard<std::mutex> lk(g_prof_mu);
  if (total_ms) *total_ms = g_prof_ms[group];
  if (launches) *launches = g_prof_n[group];
  return EGP_OK;
}

size_t egp_kmm_ws_bytes(int64_t n, int32_t d, int32_t t) {
  if (n < 1 || d < 1 || d > EGP_D_WIDE_MAX || t < 1 || t > EGP_T_MAX) return 0;
  return prepared_bytes(n, d) + kmm_core_ws_bytes(n, t);
}

static int check_n(int64_t n);

int egp_kmm_ex(const float* X, int64_t n, const float* V, int32_t t, const egp_hyper_t* h, float* out, void* ws,
               size_t ws_bytes, void* stream, const egp_call_opts_t* opts) {
  int rc;
  CallOpts co;
  if ((rc = resolve_opts(opts, &co)) != EGP_OK) return rc;
  if ((rc = validate_hyper(h)) != EGP_OK) return rc;
  if ((rc = check_n(n)) != EGP_OK) return rc;
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
  if ((rc = prepare_points(X, n, h, ws, &P, s, co.mode)) != EGP_OK) return rc;
  return kmm_core(P, V, t, out, static_cast<char*>(ws) + prepared_bytes(n, h->d), s);
}
int egp_kmm(const float* X, int64_t n, const float* V, int32_t t, const egp_hyper_t* h, float* out, void* ws,
            size_t ws_bytes, void* stream) {
  return egp_kmm_ex(X, n, V, t, h, out, ws, ws_bytes, stream, nullptr);
}

size_t egp_kmm_grad_ws_bytes(int64_t n, int32_t d, int32_t t) {
  if (n < 1 || d < 1 || d > EGP_D_MAX || t < 1 || t > EGP_T_MAX) return 0;
  return prepared_bytes(n, d) + kmm_grad_core_ws_bytes(n, d, t);
}

int egp_kmm_grad(const float* X, int64_t n, const float* V, int32_t t, const egp_hyper_t* h, float* dout, void* ws,
                 size_t ws_bytes, void* stream) {
  int rc;
  if ((rc = validate_hyper(h, EGP_D_MAX)) != EGP_OK) return rc;
  if (n < 1 || n > ((int64_t)1 << 31) - 1) return fail(EGP_ERR_ARG, "n = %lld outside 1..2^31-1", (long long)n);
  if (t < 1 || t > EGP_T_MAX) return fail(EGP_ERR_ARG, "t = %d outside 1..%d", t, EGP_T_MAX);
  if ((rc = validate_ptr(X, "X")) != EGP_OK) return rc;
  if ((rc = validate_ptr(V, "V")) != EGP_OK) return rc;
  if ((rc = validate_ptr(dout, "dout")) != EGP_OK) return rc;
  if ((rc = validate_ptr(ws, "ws")) != EGP_OK) return rc;
  const size_t need = egp_kmm_grad_ws_bytes(n, h->d, t);
  if (ws_bytes < need) return fail(EGP_ERR_WS, "workspace of %zu bytes is smaller than the %zu needed", ws_bytes, need);
  hipStream_t s = static_cast<hipStream_t>(stream);
  Prepared P;
  if ((rc = prepare_points(X, n, h, ws, &P, s, EGP_KMM_FP32)) != EGP_OK) return rc;      // fp32 in every mode
  return kmm_grad_core(P, h, V, t, dout, static_cast<char*>(ws) + prepared_bytes(n, h->d), s);
}

size_t egp_kmm_grad_bilinear_ws_bytes(int64_t n, int32_t d, int32_t t) {
  if (n < 1 || d < 1 || d > EGP_D_WIDE_MAX || t < 1 || t > 36) return 0;
  return prepared_bytes(n, d) + bilinear_core_ws_bytes(n, d, t);
}

int egp_kmm_grad_bilinear(const float* X, int64_t n, const float* A, const float* B, int32_t t, const float* w,
                          const egp_hyper_t* h, double* out, void* ws, size_t ws_bytes, void* stream) {
  int rc;
  if ((rc = validate_hyper(h)) != EGP_OK) return rc;
  if ((rc = check_n(n)) != EGP_OK) return rc;
  if (t < 1 || t > 36) return fail(EGP_ERR_ARG, "t = %d outside 1..36", t);
  if (out == nullptr) return fail(EGP_ERR_ARG, "out is NULL");
  if ((rc = validate_ptr(X, "X")) != EGP_OK) return rc;
  if ((rc = validate_ptr(A, "A")) != EGP_OK) return rc;
  if ((rc = validate_ptr(B, "B")) != EGP_OK) return rc;
  if ((rc = validate_ptr(ws, "ws")) != EGP_OK) return rc;
  const size_t need = egp_kmm_grad_bilinear_ws_bytes(n, h->d, t);
  if (ws_bytes < need) return fail(EGP_ERR_WS, "workspace of %zu bytes is smaller than the %zu needed", ws_bytes, need);
  hipStream_t s = static_cast<hipStream_t>(stream);
  Prepared P;
  if ((rc = prepare_points(X, n, h, ws, &P, s, EGP_KMM_FP32)) != EGP_OK) return rc;      // fp32 in every mode
  return bilinear_core(P, h, A, B, t, w, out, static_cast<char*>(ws) + prepared_bytes(n, h->d), s);
}

size_t egp_mll_ws_bytes(int64_t n, int32_t d, int32_t tp, int32_t rank, int32_t max_iter) {
  if (n < 1 || d < 1 || d > EGP_D_WIDE_MAX || tp < 1 || tp > 32 || rank < 0 || rank > EGP_RANK_MAX || max_iter < 1)
    return 0;
  return mll_ws_bytes_core(n, d, tp, rank, max_iter);
}

int egp_mll_ex(const float* X, int64_t n, const float* y, const float* W1, const float* W2, int32_t tp,
               const egp_hyper_t* h, int32_t rank, int32_t max_iter, float tol, egp_mll_result_t* out, void* ws,
               size_t ws_bytes, void* stream, const egp_call_opts_t* opts) {
  int rc;
  CallOpts co;
  if ((rc = resolve_opts(opts, &co)) != EGP_OK) return rc;
  if ((rc = validate_hyper(h)) != EGP_OK) return rc;
  if ((rc = check_n(n)) != EGP_OK) return rc;
  if (tp < 1 || tp > 32) return fail(EGP_ERR_ARG, "tp = %d outside 1..32", tp);
  if (rank < 0 || rank > EGP_RANK_MAX || rank > n) return fail(EGP_ERR_ARG, "rank = %d outside 0..min(n, %d)", rank, EGP_RANK_MAX);
  if (rank > 0 && !(h->noise > 0.f)) return fail(EGP_ERR_ARG, "a preconditioned evaluation needs noise > 0");
  if (max_iter < 1 || max_iter > 100000) return fail(EGP_ERR_ARG, "max_iter = %d outside 1..100000", max_iter);
  if (!(tol >= 0.f)) return fail(EGP_ERR_ARG, "tol must be >= 0");
  if (out == nullptr) return fail(EGP_ERR_ARG, "out is NULL");
  if ((rc = validate_ptr(X, "X")) != EGP_OK) return rc;
  if ((rc = validate_ptr(y, "y")) != EGP_OK) return rc;
  if ((rc = validate_ptr(W2, "W2")) != EGP_OK) return rc;
  if (rank > 0 && (rc = validate_ptr(W1, "W1")) != EGP_OK) return rc;
  if ((rc = validate_ptr(ws, "ws")) != EGP_OK) return rc;
  const size_t need = mll_ws_bytes_core(n, h->d, tp, rank, max_iter);
  if (ws_bytes < need) return fail(EGP_ERR_WS, "workspace of %zu bytes is smaller than the %zu needed", ws_bytes, need);
  return mll_core(X, n, y, W1, W2, tp, h, rank, max_iter, tol, out, ws, static_cast<hipStream_t>(stream), co);
}
int egp_mll(const float* X, int64_t n, const float* y, const float* W1, const float* W2, int32_t tp,
            const egp_hyper_t* h, int32_t rank, int32_t max_iter, float tol, egp_mll_result_t* out, void* ws,
            size_t ws_bytes, void* stream) {
  return egp_mll_ex(X, n, y, W1, W2, tp, h, rank, max_iter, tol, out, ws, ws_bytes, stream, nullptr);
}

int egp_train_adam_ex(const float* X, int64_t n, const float* y, const float* W1, const float* W2, int32_t tp,
                      int32_t kernel_type, int32_t d, float* lengthscales, float* outputscale, float* noise,
                      int32_t rank, int32_t max_iter, float tol, const egp_adam_t* opt, egp_mll_result_t* last,
                      double* mll_history, void* ws, size_t ws_bytes, void* stream, const egp_call_opts_t* opts) {
  CallOpts co;
  if (int rco = resolve_opts(opts, &co)) return rco;
  if (lengthscales == nullptr || outputscale == nullptr || noise == nullptr || opt == nullptr)
    return fail(EGP_ERR_ARG, "lengthscales / outputscale / noise / opt is NULL");
  if (opt->steps < 0 || opt->steps > 100000 || !(opt->lr > 0.f) || !(opt->beta1 >= 0.f && opt->beta1 < 1.f) ||
      !(opt->beta2 >= 0.f && opt->beta2 < 1.f) || !(opt->eps > 0.f) || !(opt->noise_floor >= 0.f))
    return fail(EGP_ERR_ARG, "bad Adam settings");
  egp_hyper_t h = {kernel_type, d, lengthscales, *outputscale, *noise};
  int rc;
  if ((rc = validate_hyper(&h)) != EGP_OK) return rc;
  if ((rc = check_n(n)) != EGP_OK) return rc;
  if (tp < 1 || tp > 32) return fail(EGP_ERR_ARG, "tp = %d outside 1..32", tp);
  if (rank < 0 || rank > EGP_RANK_MAX || rank > n) return fail(EGP_ERR_ARG, "rank = %d outside 0..min(n, %d)", rank, EGP_RANK_MAX);
  if (max_iter < 1 || max_iter > 100000) return fail(EGP_ERR_ARG, "max_iter = %d outside 1..100000", max_iter);
  if (!(tol >= 0.f)) return fail(EGP_ERR_ARG, "tol must be >= 0");
  if ((rc = validate_ptr(X, "X")) != EGP_OK) return rc;
  if ((rc = validate_ptr(y, "y")) != EGP_OK) return rc;
  if ((rc = validate_ptr(W2, "W2")) != EGP_OK) return rc;
  if (rank > 0 && (rc = validate_ptr(W1, "W1")) != EGP_OK) return rc;
  if ((rc = validate_ptr(ws, "ws")) != EGP_OK) return rc;
  const size_t need = mll_ws_bytes_core(n, d, tp, rank, max_iter);
  if (ws_bytes < need) return fail(EGP_ERR_WS, "workspace of %zu bytes is smaller than the %zu needed", ws_bytes, need);
  rc = train_adam_core(X, n, y, W1, W2, tp, &h, lengthscales, rank, max_iter, tol, opt, last, mll_history, ws,
                       static_cast<hipStream_t>(stream), co);
  *outputscale = h.outputscale;
  *noise = h.noise;
  return rc;
}
int egp_train_adam(const float* X, int64_t n, const float* y, const float* W1, const float* W2, int32_t tp,
                   int32_t kernel_type, int32_t d, float* lengthscales, float* outputscale, float* noise,
                   int32_t rank, int32_t max_iter, float tol, const egp_adam_t* opt, egp_mll_result_t* last,
                   double* mll_history, void* ws, size_t ws_bytes, void* stream) {
  return egp_train_adam_ex(X, n, y, W1, W2, tp, kernel_type, d, lengthscales, outputscale, noise, rank, max_iter, tol,
                           opt, last, mll_history, ws, ws_bytes, stream, nullptr);
}

int egp_tridiag_logquad(const double* diag, const double* off, int32_t m, double* out) {
  if (diag == nullptr || out == nullptr || m < 1 || (m > 1 && off == nullptr))
    return fail(EGP_ERR_ARG, "bad tridiagonal arguments");
  std::vector<double> a(diag, diag + m), b;
  if (m > 1) b.assign(off, off + m - 1);
  if (!tridiag_log_quadrature(a, b, out)) return fail(EGP_ERR_BREAKDOWN, "tridiagonal matrix is not positive definite");
  return EGP_OK;
}

size_t egp_kmm_cross_ws_bytes(int64_t nq, int64_t n, int32_t d, int32_t t) {
  if (nq < 1 || n < 1 || d < 1 || d > EGP_D_WIDE_MAX || t < 1 || t > EGP_T_MAX) return 0;
  return cross_ws_bytes_core(nq, n, d, t);
}

int egp_kmm_cross(const float* Xq, int64_t nq, const float* X, int64_t n, const float* V, int32_t t,
                  const egp_hyper_t* h, float* out, void* ws, size_t ws_bytes, void* stream) {
  int rc;
  if ((rc = validate_hyper(h)) != EGP_OK) return rc;
  if ((rc = check_n(n)) != EGP_OK) return rc;
  if ((rc = check_n(nq)) != EGP_OK) return rc;
  if (t < 1 || t > EGP_T_MAX) return fail(EGP_ERR_ARG, "t = %d outside 1..%d", t, EGP_T_MAX);
  if ((rc = validate_ptr(Xq, "Xq")) != EGP_OK) return rc;
  if ((rc = validate_ptr(X, "X")) != EGP_OK) return rc;
  if ((rc = validate_ptr(V, "V")) != EGP_OK) return rc;
  if ((rc = validate_ptr(out, "out")) != EGP_OK) return rc;
  if ((rc = validate_ptr(ws, "ws")) != EGP_OK) return rc;
  const size_t need = cross_ws_bytes_core(nq, n, h->d, t);
  if (ws_bytes < need) return fail(EGP_ERR_WS, "workspace of %zu bytes is smaller than the %zu needed", ws_bytes, need);
  CallOpts co;
  if ((rc = resolve_opts(nullptr, &co)) != EGP_OK) return rc;
  return cross_core(Xq, nq, X, n, V, t, h, out, ws, static_cast<hipStream_t>(stream), 0, co.mode);
}

size_t egp_lanczos_ws_bytes(int64_t n, int32_t d, int32_t r) {
  if (n < 1 || d < 1 || d > EGP_D_WIDE_MAX || r < 1 || r > EGP_RANK_MAX) return 0;
  return lanczos_ws_bytes_core(n, d, r);
}

int egp_lanczos(const float* X, int64_t n, const egp_hyper_t* h, const float* b, int32_t r, float* Q, double* alpha,
                double* beta, int32_t* steps, void* ws, size_t ws_bytes, void* stream) {
  int rc;
  if ((rc = validate_hyper(h)) != EGP_OK) return rc;
  if ((rc = check_n(n)) != EGP_OK) return rc;
  if (r < 1 || r > EGP_RANK_MAX || r > n) return fail(EGP_ERR_ARG, "r = %d outside 1..min(n, %d)", r, EGP_RANK_MAX);
  if (alpha == nullptr || steps == nullptr || (r > 1 && beta == nullptr))
    return fail(EGP_ERR_ARG, "alpha / beta / steps is NULL");
  if ((rc = validate_ptr(X, "X")) != EGP_OK) return rc;
  if ((rc = validate_ptr(b, "b")) != EGP_OK) return rc;
  if ((rc = validate_ptr(Q, "Q")) != EGP_OK) return rc;
  if ((rc = validate_ptr(ws, "ws")) != EGP_OK) return rc;
  const size_t need = lanczos_ws_bytes_core(n, h->d, r);
  if (ws_bytes < need) return fail(EGP_ERR_WS, "workspace of %zu bytes is smaller than the %zu needed", ws_bytes, need);
  CallOpts co;
  if ((rc = resolve_opts(nullptr, &co)) != EGP_OK) return rc;
  return lanczos_core(X, n, h, b, r, Q, alpha, beta, steps, ws, static_cast<hipStream_t>(stream), co.mode);
}

size_t egp_block_lanczos_ws_bytes(int64_t n, int32_t d, int32_t b, int32_t blocks) {
  if (n < 1 || d < 1 || d > EGP_D_WIDE_MAX || b < 1 || b > 32 || blocks < 1 || (int64_t)b * blocks > EGP_RANK_MAX) return 0;
  return block_lanczos_ws_bytes_core(n, d, b, blocks);
}

int egp_block_lanczos(const float* X, int64_t n, const egp_hyper_t* h, const float* B0, int32_t b, int32_t blocks,
                      float* Q, double* T, int32_t* rows, void* ws, size_t ws_bytes, void* stream) {
  int rc;
  if ((rc = validate_hyper(h)) != EGP_OK) return rc;
  if ((rc = check_n(n)) != EGP_OK) return rc;
  if (b < 1 || b > 32) return fail(EGP_ERR_ARG, "b = %d outside 1..32", b);
  if (blocks < 1 || (int64_t)b * blocks > EGP_RANK_MAX || (int64_t)b * blocks > n)
    return fail(EGP_ERR_ARG, "b * blocks = %lld outside 1..min(n, %d)", (long long)b * blocks, EGP_RANK_MAX);
  if (T == nullptr || rows == nullptr) return fail(EGP_ERR_ARG, "T / rows is NULL");
  if ((rc = validate_ptr(X, "X")) != EGP_OK) return rc;
  if ((rc = validate_ptr(B0, "B0")) != EGP_OK) return rc;
  if ((rc = validate_ptr(Q, "Q")) != EGP_OK) return rc;
  if ((rc = validate_ptr(ws, "ws")) != EGP_OK) return rc;
  const size_t need = block_lanczos_ws_bytes_core(n, h->d, b, blocks);
  if (ws_bytes < need) return fail(EGP_ERR_WS, "workspace of %zu bytes is smaller than the %zu needed", ws_bytes, need);
  CallOpts co;
  if ((rc = resolve_opts(nullptr, &co)) != EGP_OK) return rc;
  return block_lanczos_core(X, n, h, B0, b, blocks, Q, T, rows, ws, static_cast<hipStream_t>(stream), co.mode);
}

int egp_predict_dense(const float* Xq, int64_t nq, const float* X, int64_t n, const egp_hyper_t* h, const float* a,
                      const float* Q, int32_t r, const double* T, int32_t ldt, float* mean, float* var, void* ws,
                      size_t ws_bytes, void* stream) {
  int rc;
  if ((rc = validate_hyper(h)) != EGP_OK) return rc;
  if ((rc = check_n(n)) != EGP_OK) return rc;
  if ((rc = check_n(nq)) != EGP_OK) return rc;
  if (r < 1 || r > EGP_RANK_MAX || ldt < r) return fail(EGP_ERR_ARG, "r = %d outside 1..%d or ldt < r", r, EGP_RANK_MAX);
  if (T == nullptr) return fail(EGP_ERR_ARG, "T is NULL");
  if ((rc = validate_ptr(Xq, "Xq")) != EGP_OK) return rc;
  if ((rc = validate_ptr(X, "X")) != EGP_OK) return rc;
  if ((rc = validate_ptr(a, "a")) != EGP_OK) return rc;
  if ((rc = validate_ptr(mean, "mean")) != EGP_OK) return rc;
  if ((rc = validate_ptr(var, "var")) != EGP_OK) return rc;
  if ((rc = validate_ptr(Q, "Q")) != EGP_OK) return rc;
  if ((rc = validate_ptr(ws, "ws")) != EGP_OK) return rc;
  const size_t need = predict_ws_bytes_core(nq, n, h->d, r);
  if (ws_bytes < need) return fail(EGP_ERR_WS, "workspace of %zu bytes is smaller than the %zu needed", ws_bytes, need);
  CallOpts co;
  if ((rc = resolve_opts(nullptr, &co)) != EGP_OK) return rc;
  return predict_core(Xq, nq, X, n, h, a, Q, r, nullptr, nullptr, mean, var, ws, static_cast<hipStream_t>(stream),
                      co.mode, T, ldt);
}

size_t egp_predict_ws_bytes(int64_t nq, int64_t n, int32_t d, int32_t r) {
  if (nq < 1 || n < 1 || d < 1 || d > EGP_D_WIDE_MAX || r < 0 || r > EGP_RANK_MAX) return 0;
  return predict_ws_bytes_core(nq, n, d, r);
}

int egp_predict(const float* Xq, int64_t nq, const float* X, int64_t n, const egp_hyper_t* h, const float* a,
                const float* Q, int32_t r, const double* alpha, const double* beta, float* mean, float* var, void* ws,
                size_t ws_bytes, void* stream) {
  int rc;
  if ((rc = validate_hyper(h)) != EGP_OK) return rc;
  if ((rc = check_n(n)) != EGP_OK) return rc;
  if ((rc = check_n(nq)) != EGP_OK) return rc;
  if (r < 0 || r > EGP_RANK_MAX) return fail(EGP_ERR_ARG, "r = %d outside 0..%d", r, EGP_RANK_MAX);
  if ((rc = validate_ptr(Xq, "Xq")) != EGP_OK) return rc;
  if ((rc = validate_ptr(X, "X")) != EGP_OK) return rc;
  if ((rc = validate_ptr(a, "a")) != EGP_OK) return rc;
  if ((rc = validate_ptr(mean, "mean")) != EGP_OK) return rc;
  if (var != nullptr) {
    if ((rc = validate_ptr(var, "var")) != EGP_OK) return rc;
    if (r < 1 || alpha == nullptr || (r > 1 && beta == nullptr)) return fail(EGP_ERR_ARG, "a variance needs r >= 1, alpha and beta");
    if ((rc = validate_ptr(Q, "Q")) != EGP_OK) return rc;
  }
  if ((rc = validate_ptr(ws, "ws")) != EGP_OK) return rc;
  const size_t need = predict_ws_bytes_core(nq, n, h->d, var ? r : 0);
  if (ws_bytes < need) return fail(EGP_ERR_WS, "workspace of %zu bytes is smaller than the %zu needed", ws_bytes, need);
  CallOpts co;
  if ((rc = resolve_opts(nullptr, &co)) != EGP_OK) return rc;
  return predict_core(Xq, nq, X, n, h, a, Q, r, alpha, beta, mean, var, ws, static_cast<hipStream_t>(stream), co.mode);
}

static int check_n(int64_t n) {
  if (n < 1 || n > ((int64_t)1 << 31) - 1) return fail(EGP_ERR_ARG, "n = %lld outside 1..2^31-1", (long long)n);
  return EGP_OK;
}

static int check_precond(const egp_precond_t* P, int64_t n, bool filled) {
  if (P == nullptr) return fail(EGP_ERR_ARG, "preconditioner struct is NULL");
  if (P->rank < (filled ? 0 : 1) || P->rank > EGP_RANK_MAX || P->rank > n)
    return fail(EGP_ERR_ARG, "preconditioner rank %d outside 1..min(n, %d)", P->rank, EGP_RANK_MAX);
  int rc;
  if ((rc = validate_ptr(P->L, "P->L")) != EGP_OK) return rc;
  if ((rc = validate_ptr(P->small_dev, "P->small_dev")) != EGP_OK) return rc;
  if (!filled && (P->pivots == nullptr || P->small == nullptr))
    return fail(EGP_ERR_ARG, "P->pivots / P->small is NULL");
  return EGP_OK;
}

size_t egp_piv_chol_precond_ws_bytes(int64_t n, int32_t d, int32_t rank) {
  if (n < 1 || d < 1 || d > EGP_D_WIDE_MAX || rank < 1 || rank > EGP_RANK_MAX) return 0;
  return pivchol_ws_bytes(n, d, rank);
}

int egp_piv_chol_precond(const float* X, int64_t n, const egp_hyper_t* h, float tol_abs, egp_precond_t* P,
                         void* ws, size_t ws_bytes, void* stream) {
  int rc;
  if ((rc = validate_hyper(h)) != EGP_OK) return rc;
  if ((rc = check_n(n)) != EGP_OK) return rc;
  if (!(h->noise > 0.f)) return fail(EGP_ERR_ARG, "the preconditioner P = L L^T + noise I needs noise > 0");
  if (!(tol_abs >= 0.f)) return fail(EGP_ERR_ARG, "tol_abs must be >= 0");
  if ((rc = validate_ptr(X, "X")) != EGP_OK) return rc;
  if ((rc = check_precond(P, n, false)) != EGP_OK) return rc;
  if ((rc = validate_ptr(ws, "ws")) != EGP_OK) return rc;
  const size_t need = egp_piv_chol_precond_ws_bytes(n, h->d, P->rank);
  if (ws_bytes < need) return fail(EGP_ERR_WS, "workspace of %zu bytes is smaller than the %zu needed", ws_bytes, need);
  return pivchol_core(X, n, h, tol_abs, P, ws, static_cast<hipStream_t>(stream));
}

size_t egp_precond_apply_ws_bytes(int64_t n, int32_t t, int32_t rank) {
  if (n < 1 || t < 1 || t > 33 || rank < 1 || rank > EGP_RANK_MAX) return 0;
  return precond_apply_ws(n, t, rank);
}

int egp_precond_apply(const egp_precond_t* P, int64_t n, float noise, const float* R, int32_t t, float* Z,
                      void* ws, size_t ws_bytes, void* stream) {
  int rc;
  if ((rc = check_n(n)) != EGP_OK) return rc;
  if ((rc = check_precond(P, n, true)) != EGP_OK) return rc;
  if (P->rank < 1) return fail(EGP_ERR_ARG, "preconditioner has rank 0");
  if (!(noise > 0.f)) return fail(EGP_ERR_ARG, "noise must be > 0");
  if (t < 1 || t > 33) return fail(EGP_ERR_ARG, "t = %d outside 1..33", t);
  if ((rc = validate_ptr(R, "R")) != EGP_OK) return rc;
  if ((rc = validate_ptr(Z, "Z")) != EGP_OK) return rc;
  if ((rc = validate_ptr(ws, "ws")) != EGP_OK) return rc;
  const size_t need = precond_apply_ws(n, t, P->rank);
  if (ws_bytes < need) return fail(EGP_ERR_WS, "workspace of %zu bytes is smaller than the %zu needed", ws_bytes, need);
  return precond_apply_core(P->L, P->rank, P->small_dev, n, noise, R, t, Z, nullptr, ws,
                            static_cast<hipStream_t>(stream));
}

size_t egp_mbcg_ws_bytes(int64_t n, int32_t d, int32_t t, int32_t rank, int32_t max_iter) {
  if (n < 1 || d < 1 || d > EGP_D_WIDE_MAX || t < 1 || t > 33 || rank < 0 || rank > EGP_RANK_MAX || max_iter < 0)
    return 0;
  return mbcg_ws_bytes_core(n, d, t, rank, max_iter);
}

int egp_mbcg_ex(const float* X, int64_t n, const float* B, int32_t t, const egp_hyper_t* h, const egp_precond_t* P,
                int32_t max_iter, float tol, float* U, double* cg_coef, double* gamma0, int32_t* iters_done,
                float* rel_resid, float* resid_hist, void* ws, size_t ws_bytes, void* stream,
                const egp_call_opts_t* opts) {
  int rc;
  CallOpts co;
  if ((rc = resolve_opts(opts, &co)) != EGP_OK) return rc;
  if ((rc = validate_hyper(h)) != EGP_OK) return rc;
  if ((rc = check_n(n)) != EGP_OK) return rc;
  if (t < 1 || t > 33) return fail(EGP_ERR_ARG, "t = %d outside 1..33", t);
  if (max_iter < 0 || max_iter > 100000) return fail(EGP_ERR_ARG, "max_iter = %d outside 0..100000", max_iter);
  if (!(tol >= 0.f)) return fail(EGP_ERR_ARG, "tol must be >= 0");
  if ((rc = validate_ptr(X, "X")) != EGP_OK) return rc;
  if ((rc = validate_ptr(B, "B")) != EGP_OK) return rc;
  if ((rc = validate_ptr(U, "U")) != EGP_OK) return rc;
  if ((rc = validate_ptr(ws, "ws")) != EGP_OK) return rc;
  if (U == B) return fail(EGP_ERR_ARG, "U must not alias B");
  if (P != nullptr) {
    if ((rc = check_precond(P, n, true)) != EGP_OK) return rc;
    if (!(h->noise > 0.f)) return fail(EGP_ERR_ARG, "a preconditioned solve needs noise > 0");
    if (P->rank == 0) P = nullptr;
  }
  const size_t need = mbcg_ws_bytes_core(n, h->d, t, P ? P->rank : 0, max_iter);
  if (ws_bytes < need) return fail(EGP_ERR_WS, "workspace of %zu bytes is smaller than the %zu needed", ws_bytes, need);
  return mbcg_core(X, n, B, t, h, P, max_iter, tol, U, cg_coef, gamma0, iters_done, rel_resid, resid_hist, ws,
                   static_cast<hipStream_t>(stream), co);
}
int egp_mbcg(const float* X, int64_t n, const float* B, int32_t t, const egp_hyper_t* h, const egp_precond_t* P,
             int32_t max_iter, float tol, float* U, double* cg_coef, double* gamma0, int32_t* iters_done,
             float* rel_resid, float* resid_hist, void* ws, size_t ws_bytes, void* stream) {
  return egp_mbcg_ex(X, n, B, t, h, P, max_iter, tol, U, cg_coef, gamma0, iters_done, rel_resid, resid_hist, ws,
                     ws_bytes, stream, nullptr);
}

}  // extern "C"
