// One marginal-likelihood evaluation with its gradient, assembled from the pieces of this library.
//
// Paper, Eq. 1 and Eq. 2, and Background (last paragraph of "Conjugate gradients"): one batched solve
// with right-hand sides [y | probes] yields Khat^{-1} y, the log-determinant (stochastic Lanczos
// quadrature on the tridiagonals of the probe columns) and the trace terms of the gradient.
//   L      = -1/2 y^T u - 1/2 log|Khat| - n/2 log(2 pi),              u = Khat^{-1} y
//   dL/dth = 1/2 u^T (dKhat/dth) u - 1/2 tr(Khat^{-1} dKhat/dth)
//   log|Khat|              ~ log|P| + mean_c gamma0_c e1^T log(T_c) e1,   gamma0_c = z_c^T P^{-1} z_c
//   tr(Khat^{-1} dKhat/dth) ~ mean_c (Khat^{-1} z_c)^T (dKhat/dth) (P^{-1} z_c)
// with probe vectors z_c = L w1_c + sqrt(noise) w2_c of covariance P = L L^T + noise I built from the
// caller's Rademacher draws (the library draws no random numbers). (Eq. 2 as printed is not a valid
// identity; the form above is the standard one.)

#include <math.h>

#include <vector>

#include "egp_internal.h"

namespace egp {

namespace {

// Z[i][c] = sum_m L[m][i] W1[m][c] + sigma W2[i][c]   (tp <= 32 columns); also B = [y | Z]
template <int TT>
__global__ __launch_bounds__(256) void make_probes(const float* __restrict__ L, int rank, int64_t n,
                                                   const float* __restrict__ W1, const float* __restrict__ W2,
                                                   int tp, float sigma, const float* __restrict__ y,
                                                   float* __restrict__ B /*n x (tp+1)*/) {
  const int t = tp + 1;      // W1 is indexed uniformly across the wave: its entries arrive as scalar operands
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    float acc[TT];
#pragma unroll
    for (int c = 0; c < TT; ++c) acc[c] = 0.f;
    for (int m = 0; m < rank; ++m) {
      const float l = L[(int64_t)m * n + i];
      const float* w = W1 + m * tp;
#pragma unroll
      for (int c = 0; c < TT; ++c)
        if (c < tp) acc[c] = __builtin_fmaf(l, w[c], acc[c]);
    }
    B[i * t] = y[i];
#pragma unroll
    for (int c = 0; c < TT; ++c)
      if (c < tp) B[i * t + 1 + c] = __builtin_fmaf(sigma, W2[i * tp + c], acc[c]);
  }
}

// dst[i][dc] = src[i][sc] for all i (column copy between row-major matrices)
__global__ __launch_bounds__(256) void copy_columns(const float* __restrict__ src, int ts, int sc, int64_t n,
                                                    float* __restrict__ dst, int td, int dc, int count) {
  for (int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x; g < n * count; g += (int64_t)gridDim.x * 256) {
    const int64_t i = g / count;
    const int c = (int)(g % count);
    dst[i * td + dc + c] = src[i * ts + sc + c];
  }
}

// part[block][c] = partial sums over rows of A[i][c] * B[i][c]
__global__ __launch_bounds__(256) void coldot_partial(const float* __restrict__ A, const float* __restrict__ B,
                                                      int64_t n, int t, int tp2, float* __restrict__ part) {
  __shared__ float sh[256];
  const int rows = 256 / tp2, c = threadIdx.x % tp2, rl = threadIdx.x / tp2;
  float acc = 0.f;
  if (c < t)
    for (int64_t i = (int64_t)blockIdx.x * rows + rl; i < n; i += (int64_t)gridDim.x * rows)
      acc = __builtin_fmaf(A[i * t + c], B[i * t + c], acc);
  sh[threadIdx.x] = acc;
  __syncthreads();
  if (rl == 0 && c < t) {
    float s = 0.f;
    for (int r = 0; r < rows; ++r) s += sh[r * tp2 + c];
    part[(int64_t)blockIdx.x * t + c] = s;
  }
}

constexpr int kDotBlocks = 512;

// host: column dots of two n x t matrices, fp64 final reduction
int column_dots(const float* A, const float* B, int64_t n, int t, float* part_dev, std::vector<double>* out,
                hipStream_t stream) {
  int tp2 = 16;
  while (tp2 < t) tp2 *= 2;
  hipLaunchKernelGGL(coldot_partial, dim3(kDotBlocks), dim3(256), 0, stream, A, B, n, t, tp2, part_dev);
  EGP_HIP(hipGetLastError());
  std::vector<float> h((size_t)kDotBlocks * t);
  EGP_HIP(hipMemcpyAsync(h.data(), part_dev, h.size() * sizeof(float), hipMemcpyDeviceToHost, stream));
  EGP_HIP(hipStreamSynchronize(stream));
  out->assign(t, 0.0);
  for (int b = 0; b < kDotBlocks; ++b)
    for (int c = 0; c < t; ++c) (*out)[c] += (double)h[(size_t)b * t + c];
  return EGP_OK;
}

}  // namespace

// e1^T log(T) e1 for the symmetric positive definite tridiagonal T (diagonal a, off-diagonal b):
// implicit symmetric QR steps with Wilkinson shifts (Givens rotations chase the bulge down the active
// block, small off-diagonals deflate it), carrying only the first row z of the eigenvector matrix.
// Then e1^T log(T) e1 = sum_i z_i^2 log(lambda_i): the Gauss quadrature rule of the Lanczos process.
bool tridiag_log_quadrature(std::vector<double> a, std::vector<double> b, double* result) {
  const int m = (int)a.size();
  if (m == 0) { *result = 0.0; return true; }
  b.resize(m > 1 ? m - 1 : 0);
  std::vector<double> z(m, 0.0);
  z[0] = 1.0;
  const double eps = 1.1e-16;
  int hi = m - 1;
  long budget = 60L * m + 200;
  while (hi > 0) {
    if (fabs(b[hi - 1]) <= eps * (fabs(a[hi - 1]) + fabs(a[hi]))) {
      b[hi - 1] = 0.0;
      --hi;
      continue;
    }
    if (--budget < 0) return false;
    int lo = hi - 1;
    while (lo > 0 && fabs(b[lo - 1]) > eps * (fabs(a[lo - 1]) + fabs(a[lo]))) --lo;
    const double dlt = 0.5 * (a[hi - 1] - a[hi]);
    const double bb = b[hi - 1] * b[hi - 1];
    const double den = dlt + (dlt >= 0.0 ? 1.0 : -1.0) * sqrt(dlt * dlt + bb);
    const double mu = a[hi] - (den != 0.0 ? bb / den : 0.0);
    double x = a[lo] - mu, bulge = b[lo];
    for (int k = lo; k < hi; ++k) {
      const double r = hypot(x, bulge);
      const double c = r > 0.0 ? x / r : 1.0, sn = r > 0.0 ? bulge / r : 0.0;
      if (k > lo) b[k - 1] = r;
      const double ak = a[k], ak1 = a[k + 1], bk = b[k];
      a[k] = c * c * ak + 2.0 * c * sn * bk + sn * sn * ak1;
      a[k + 1] = sn * sn * ak - 2.0 * c * sn * bk + c * c * ak1;
      b[k] = (c * c - sn * sn) * bk + c * sn * (ak1 - ak);
      if (k < hi - 1) {
        bulge = sn * b[k + 1];
        b[k + 1] = c * b[k + 1];
        x = b[k];
      }
      const double zk = z[k], zk1 = z[k + 1];
      z[k] = c * zk + sn * zk1;
      z[k + 1] = -sn * zk + c * zk1;
    }
  }
  double acc = 0.0;
  for (int i = 0; i < m; ++i) {
    if (!(a[i] > 0.0)) return false;
    acc += z[i] * z[i] * log(a[i]);
  }
  *result = acc;
  return true;
}

namespace {

struct MllWs {
  size_t prep, Lbuf, small_dev, B, U, Vp, Zp, part, sub, total;
};

MllWs mll_layout(int64_t n, int d, int tp, int rank, int max_iter) {
  MllWs w;
  const int t = tp + 1;
  const size_t vec = round_up((size_t)n * t * sizeof(float), 256);
  w.prep = prepared_bytes(n, d);
  w.Lbuf = round_up((size_t)(rank > 0 ? rank : 1) * n * sizeof(float), 256);
  w.small_dev = round_up((size_t)(rank > 0 ? rank * rank : 1) * sizeof(double), 256);
  w.B = vec;
  w.U = vec;
  w.Vp = vec;
  w.Zp = vec;
  w.part = round_up((size_t)kDotBlocks * 64 * sizeof(float), 256);
  size_t sub = mbcg_ws_bytes_core(n, d, t, rank, max_iter);
  const size_t pc = rank > 0 ? pivchol_ws_bytes(n, d, rank) : 0;
  const size_t kg = bilinear_core_ws_bytes(n, d, t);
  const size_t km = 0;
  const size_t pa = rank > 0 ? precond_apply_ws(n, t, rank) : 0;
  if (pc > sub) sub = pc;
  if (kg > sub) sub = kg;
  if (km > sub) sub = km;
  if (pa > sub) sub = pa;
  w.sub = round_up(sub, 256);
  w.total = w.prep + w.Lbuf + w.small_dev + w.B + w.U + w.Vp + w.Zp + w.part + w.sub;
  return w;
}

}  // namespace

size_t mll_ws_bytes_core(int64_t n, int d, int tp, int rank, int max_iter) {
  return mll_layout(n, d, tp, rank, max_iter).total;
}

int mll_core(const float* X, int64_t n, const float* y, const float* W1, const float* W2, int tp,
             const egp_hyper_t* h, int rank_req, int max_iter, float tol, egp_mll_result_t* res, void* ws,
             hipStream_t stream, const CallOpts& co) {
  const int d = h->d, t = tp + 1;
  const MllWs lay = mll_layout(n, d, tp, rank_req, max_iter);
  char* w = static_cast<char*>(ws);
  char* prep_ws = w;            w += lay.prep;
  float* Lbuf = (float*)w;      w += lay.Lbuf;
  double* small_dev = (double*)w; w += lay.small_dev;
  float* B = (float*)w;         w += lay.B;
  float* U = (float*)w;         w += lay.U;
  float* Vp = (float*)w;        w += lay.Vp;
  float* Zp = (float*)w;        w += lay.Zp;
  float* part = (float*)w;      w += lay.part;
  void* sub = w;

  // ---- preconditioner ----
  std::vector<int32_t> pivots(rank_req > 0 ? rank_req : 1);
  std::vector<double> small((size_t)(rank_req > 0 ? rank_req * rank_req : 0) + 1, 0.0);
  egp_precond_t P;
  P.rank = rank_req;
  P.L = Lbuf;
  P.pivots = pivots.data();
  P.small = small.data();
  P.small_dev = small_dev;
  double logdetP = 0.0;
  int rc;
  if (rank_req > 0) {
    rc = pivchol_core(X, n, h, 0.f, &P, sub, stream);      // (uses no fused multiply: no mode to pass)
    if (rc != EGP_OK) return rc;
    logdetP = small[(size_t)rank_req * rank_req];
  }
  const int rank = rank_req > 0 ? P.rank : 0;
  const egp_precond_t* Pp = rank > 0 ? &P : nullptr;

  // ---- right-hand sides [y | probes with covariance P] ----
  {
    const float sigma = rank > 0 ? sqrtf(h->noise) : 1.0f;
    int64_t nb = (n + 255) / 256;
    const int blocks = (int)(nb > 2048 ? 2048 : nb);
    const size_t shb = 0;
    if (tp <= 16)
      hipLaunchKernelGGL(make_probes<16>, dim3(blocks), dim3(256), shb, stream, Lbuf, rank, n, W1, W2, tp, sigma, y, B);
    else
      hipLaunchKernelGGL(make_probes<32>, dim3(blocks), dim3(256), shb, stream, Lbuf, rank, n, W1, W2, tp, sigma, y, B);
    EGP_HIP(hipGetLastError());
  }

  // ---- batched solve ----
  std::vector<double> coef((size_t)(max_iter > 0 ? max_iter : 1) * 2 * t, 0.0), gamma0(t, 0.0);
  std::vector<float> rel(t, 0.f);
  int32_t iters = 0;
  // (with column shrinking on, a probe's tridiagonal below ends where the probe left the iteration)
  rc = mbcg_core(X, n, B, t, h, Pp, max_iter, tol, U, coef.data(), gamma0.data(), &iters, rel.data(), nullptr, sub,
                 stream, co);
  if (rc != EGP_OK) return rc;
  res->iters = iters;
  res->precond_rank = rank;
  res->rel_resid_max = 0.f;
  for (int c = 0; c < t; ++c)
    if (rel[c] > res->rel_resid_max) res->rel_resid_max = rel[c];

  // ---- log-determinant by Lanczos quadrature on the probe columns ----
  double ld_sum = 0.0;
  for (int c = 1; c < t; ++c) {
    std::vector<double> a(iters), b(iters > 0 ? iters - 1 : 0);
    for (int j = 0; j < iters; ++j) {
      const double alpha = coef[((size_t)j * 2 + 0) * t + c];
      if (!(alpha > 0.0)) {   // a column that stopped moving: truncate its tridiagonal here
        a.resize(j);
        b.resize(j > 0 ? j - 1 : 0);
        break;
      }
      double diag = 1.0 / alpha;
      if (j > 0) {
        const double ap = coef[((size_t)(j - 1) * 2 + 0) * t + c], bp = coef[((size_t)(j - 1) * 2 + 1) * t + c];
        diag += bp / ap;
      }
      a[j] = diag;
      if (j + 1 < iters) b[j] = sqrt(fmax(coef[((size_t)j * 2 + 1) * t + c], 0.0)) / alpha;
    }
    if (b.size() + 1 > a.size()) b.resize(a.size() > 0 ? a.size() - 1 : 0);
    double quad = 0.0;
    if (!tridiag_log_quadrature(a, b, &quad))
      return fail(EGP_ERR_BREAKDOWN, "Lanczos tridiagonal of probe %d is not positive definite", c - 1);
    ld_sum += gamma0[c] * quad;
  }
  res->logdet = logdetP + (tp > 0 ? ld_sum / tp : 0.0);

  // ---- V' = [u_y | P^{-1} z_c] ----
  if (rank > 0) {
    rc = precond_apply_core(Lbuf, rank, small_dev, n, h->noise, B, t, Zp, nullptr, sub, stream);
    if (rc != EGP_OK) return rc;
  } else {
    hipLaunchKernelGGL(copy_columns, dim3(1024), dim3(256), 0, stream, B, t, 0, n, Zp, t, 0, t);
  }
  hipLaunchKernelGGL(copy_columns, dim3(1024), dim3(256), 0, stream, Zp, t, 0, n, Vp, t, 0, t);
  hipLaunchKernelGGL(copy_columns, dim3(1024), dim3(256), 0, stream, U, t, 0, n, Vp, t, 0, 1);
  EGP_HIP(hipGetLastError());

  std::vector<double> dots;
  // quadratic term y^T u: column 0 of B . U
  rc = column_dots(B, U, n, t, part, &dots, stream);
  if (rc != EGP_OK) return rc;
  res->quad = dots[0];
  res->mll = -0.5 * res->quad - 0.5 * res->logdet - 0.5 * (double)n * log(2.0 * M_PI);

  // ---- gradient: every term is a bilinear form with weights +1/2 (data term) and -1/(2 tp) (probes) ----
  std::vector<float> wcol(t);
  wcol[0] = 0.5f;
  for (int c = 1; c < t; ++c) wcol[c] = -0.5f / (float)tp;
  Prepared prep;
  rc = prepare_points(X, n, h, prep_ws, &prep, stream, EGP_KMM_FP32);      // the gradient forms are fp32 in every mode
  if (rc != EGP_OK) return rc;
  std::vector<double> forms(d + 1, 0.0);
  rc = bilinear_core(prep, h, U, Vp, t, wcol.data(), forms.data(), sub, stream);
  if (rc != EGP_OK) return rc;
  for (int k = 0; k <= d; ++k) res->grad[k] = forms[k];      // lengthscales, then outputscale (dKhat/ds = K / s)
  // ---- noise: dKhat/dnoise = I ----
  rc = column_dots(U, Vp, n, t, part, &dots, stream);
  if (rc != EGP_OK) return rc;
  double gn = 0.0;
  for (int c = 0; c < t; ++c) gn += (double)wcol[c] * dots[c];
  res->grad[d + 1] = gn;
  for (int k = d + 2; k < EGP_D_WIDE_MAX + 2; ++k) res->grad[k] = 0.0;
  return EGP_OK;
}

// Adam ascent on the log marginal likelihood in log-parameters (paper, Experiment details: hyper-parameters are
// fitted with Adam, step size 0.1, a few steps on the full data after pre-training on a subset; the learned
// noise is kept above a floor). Parameters: phi = (log l_1..log l_d, log s, log(noise - floor)); the gradient
// with respect to phi is theta dL/dtheta by the chain rule. The objective is scaled by 1/n as is usual, which
// Adam's normalisation makes immaterial. The same probe draws are used at every step.
int train_adam_core(const float* X, int64_t n, const float* y, const float* W1, const float* W2, int tp,
                    egp_hyper_t* h, float* lengthscales_io, int rank, int max_iter, float tol,
                    const egp_adam_t* opt, egp_mll_result_t* last, double* mll_history, void* ws,
                    hipStream_t stream, const CallOpts& co) {
  const int d = h->d, np = d + 2;
  const double floor_ = opt->noise_floor > 0.f ? (double)opt->noise_floor : 0.0;
  std::vector<double> phi(np), m(np, 0.0), v(np, 0.0);
  for (int k = 0; k < d; ++k) phi[k] = log((double)lengthscales_io[k]);
  phi[d] = log((double)h->outputscale);
  double excess = (double)h->noise - floor_;
  if (!(excess > 0.0)) excess = 1e-4 * (floor_ > 0.0 ? floor_ : 1.0);
  phi[d + 1] = log(excess);
  const double b1 = opt->beta1, b2 = opt->beta2, eps = opt->eps, lr = opt->lr;
  egp_mll_result_t res;
  for (int step = 0; step <= opt->steps; ++step) {
    for (int k = 0; k < d; ++k) lengthscales_io[k] = (float)exp(phi[k]);
    h->lengthscales = lengthscales_io;
    h->outputscale = (float)exp(phi[d]);
    h->noise = (float)(floor_ + exp(phi[d + 1]));
    if (step == opt->steps && last == nullptr && mll_history == nullptr) break;
    const int rc = mll_core(X, n, y, W1, W2, tp, h, rank, max_iter, tol, &res, ws, stream, co);
    if (rc != EGP_OK) return rc;
    if (mll_history) mll_history[step] = res.mll;
    if (step == opt->steps) break;        // the last evaluation only reports the objective at the final parameters
    for (int k = 0; k < np; ++k) {
      const double theta = k < d ? exp(phi[k]) : (k == d ? exp(phi[d]) : exp(phi[d + 1]));
      const double g = theta * res.grad[k] / (double)n;        // ascent direction on L / n in log-parameters
      m[k] = b1 * m[k] + (1.0 - b1) * g;
      v[k] = b2 * v[k] + (1.0 - b2) * g * g;
      const double mh = m[k] / (1.0 - pow(b1, step + 1)), vh = v[k] / (1.0 - pow(b2, step + 1));
      phi[k] += lr * mh / (sqrt(vh) + eps);
    }
  }
  if (last) *last = res;
  return EGP_OK;
}

}  // namespace egp
