// Prediction path: rectangular products K(Xq, X) V, a Lanczos cache of Khat, predictive mean and variance.
//
// Paper, Method "Predictions" and Eq. (predictive mean, predictive variance): the mean needs only
// K(xq, X) a with the cached solve a = Khat^{-1} y; the variance k(xq,xq) - k_q^T Khat^{-1} k_q is served from a
// training-data-dependent cache so that no solve happens at test time and each test point costs O(n). The
// paper cites the cache construction; here it is the rank-r Galerkin approximation of Khat^{-1} on a Krylov
// space: r Lanczos steps with full re-orthogonalisation give Q (orthonormal rows) and tridiagonal T = Q Khat Q^T,
// and var(xq) ~= s - g^T T^{-1} g with g = Q K(X, xq). Because Q T^{-1} Q^T <= Khat^{-1}, the cached variance is
// never below the exact one and decreases monotonically to it as r grows.

#include <math.h>

#include <vector>

#include "egp_internal.h"

namespace egp {

namespace {

__global__ __launch_bounds__(256) void sumsq_partial(const float* __restrict__ v, int64_t n, float* __restrict__ part) {
  __shared__ float red[4];
  float acc = 0.f;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256)
    acc = __builtin_fmaf(v[i], v[i], acc);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) part[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

// dst1[i] = dst2[i] = scale * src[i] for i < n; dst2 is zero-padded up to npad
__global__ __launch_bounds__(256) void scale_store(const float* __restrict__ src, float scale, int64_t n, int64_t npad,
                                                   float* __restrict__ dst1, float* __restrict__ dst2) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < npad; i += (int64_t)gridDim.x * 256) {
    const float v = i < n ? scale * src[i] : 0.f;
    if (i < n) dst1[i] = v;
    dst2[i] = v;
  }
}

constexpr int kNormBlocks = 256;

int vec_norm(const float* v, int64_t n, float* part_dev, double* out, hipStream_t stream) {
  hipLaunchKernelGGL(sumsq_partial, dim3(kNormBlocks), dim3(256), 0, stream, v, n, part_dev);
  EGP_HIP(hipGetLastError());
  float h[kNormBlocks];
  EGP_HIP(hipMemcpyAsync(h, part_dev, sizeof(h), hipMemcpyDeviceToHost, stream));
  EGP_HIP(hipStreamSynchronize(stream));
  double s = 0.0;
  for (int b = 0; b < kNormBlocks; ++b) s += (double)h[b];
  *out = sqrt(s);
  return EGP_OK;
}

struct LanczosWs { size_t prep, kmm, vec, part, pre, total; };
LanczosWs lanczos_layout(int64_t n, int d, int r) {
  LanczosWs w;
  const int64_t ld = padded_points(n);
  w.prep = prepared_bytes(n, d);
  w.kmm = kmm_core_ws_bytes(n, 1);
  w.vec = 3 * round_up((size_t)ld * sizeof(float), 256);     // v (padded), w, w2
  w.part = round_up((size_t)1024 * sizeof(float), 256);
  w.pre = precond_apply_ws(n, 1, r);
  w.total = w.prep + w.kmm + w.vec + w.part + w.pre;
  return w;
}

}  // namespace

size_t lanczos_ws_bytes_core(int64_t n, int d, int r) { return lanczos_layout(n, d, r).total; }

// r Lanczos steps on Khat from the start vector b, full re-orthogonalisation (two projection passes per step).
// Q: device [r][n]; alpha[r], beta[r-1] on the host; *steps <= r (fewer when the Krylov space is exhausted).
int lanczos_core(const float* X, int64_t n, const egp_hyper_t* h, const float* b, int r, float* Q, double* alpha,
                 double* beta, int32_t* steps, void* ws, hipStream_t stream, int mode) {
  const LanczosWs lay = lanczos_layout(n, h->d, r);
  const int64_t ld = padded_points(n);
  char* w = static_cast<char*>(ws);
  Prepared prep;
  int rc = prepare_points(X, n, h, w, &prep, stream, mode);
  if (rc != EGP_OK) return rc;
  w += lay.prep;
  void* kmm_ws = w;
  w += lay.kmm;
  const size_t vb = round_up((size_t)ld * sizeof(float), 256);
  float* v = reinterpret_cast<float*>(w);
  float* wv = reinterpret_cast<float*>(w + vb);
  float* w2 = reinterpret_cast<float*>(w + 2 * vb);
  w += lay.vec;
  float* part = reinterpret_cast<float*>(w);
  w += lay.part;
  void* pre_ws = w;

  double nb = 0.0;
  rc = vec_norm(b, n, part, &nb, stream);
  if (rc != EGP_OK) return rc;
  if (!(nb > 0.0)) return fail(EGP_ERR_ARG, "the Lanczos start vector is zero");
  hipLaunchKernelGGL(scale_store, dim3(1024), dim3(256), 0, stream, b, (float)(1.0 / nb), n, ld, Q, v);
  int done = 0;
  double first_beta = 0.0;
  for (int j = 0; j < r; ++j) {
    // w = Khat q_j; the multiply's epilogue leaves the partial sums of q_j . w
    rc = kmm_core_cm(prep, v, 1, wv, kmm_ws, part, 1024, stream);
    if (rc != EGP_OK) return rc;
    float hp[64];
    const int nblk = kmm_cm_dot_blocks(ld);
    EGP_HIP(hipMemcpyAsync(hp, part, sizeof(float) * nblk, hipMemcpyDeviceToHost, stream));
    EGP_HIP(hipStreamSynchronize(stream));
    double a = 0.0;
    for (int k = 0; k < nblk; ++k) a += (double)hp[k];
    alpha[j] = a;
    done = j + 1;
    if (j + 1 == r) break;
    // w <- w - Q_j (Q_j^T w), twice: removes alpha_j q_j, beta_{j-1} q_{j-1} and the drift against older vectors
    rc = precond_apply_cm(Q, j + 1, nullptr, n, 1.0f, wv, ld, 1, w2, nullptr, 0, pre_ws, stream);
    if (rc != EGP_OK) return rc;
    rc = precond_apply_cm(Q, j + 1, nullptr, n, 1.0f, w2, ld, 1, wv, nullptr, 0, pre_ws, stream);
    if (rc != EGP_OK) return rc;
    double bj = 0.0;
    rc = vec_norm(wv, n, part, &bj, stream);
    if (rc != EGP_OK) return rc;
    if (j == 0) first_beta = bj;
    if (!(bj > 1e-6 * (fabs(alpha[0]) + first_beta))) break;      // invariant subspace reached
    beta[j] = bj;
    hipLaunchKernelGGL(scale_store, dim3(1024), dim3(256), 0, stream, wv, (float)(1.0 / bj), n, ld,
                       Q + (int64_t)(j + 1) * n, v);
    EGP_HIP(hipGetLastError());
  }
  *steps = done;
  EGP_HIP(hipStreamSynchronize(stream));
  return EGP_OK;
}

// ------------------------------------------------------------------------------------------------
// Block variant: orthonormal basis of span{B0, Khat B0, .., Khat^(blocks-1) B0} and T = Q Khat Q^T (dense).
// The variance cache only needs an orthonormal Q and the projected matrix (Galerkin: Q^T T^{-1} Q <= Khat^{-1}), and
// a fused multiply costs the same for 1 and for 16 columns, so b start vectors make the cache b times cheaper per
// basis vector. Per block: one multiply, two projection passes against every earlier vector (their coefficients
// are the entries of T), Cholesky-QR applied twice to the remainder.
// ------------------------------------------------------------------------------------------------
namespace {

struct BlockWs { size_t prep, kmm, vec, small, gram, pre, total; };
BlockWs block_layout(int64_t n, int d, int b, int rcap) {
  BlockWs w;
  const int64_t ld = padded_points(n);
  w.prep = prepared_bytes(n, d);
  w.kmm = kmm_core_ws_bytes(n, b);
  w.vec = 3 * round_up((size_t)ld * b * sizeof(float), 256);
  w.small = 2 * round_up((size_t)32 * 32 * sizeof(double), 256);
  w.gram = gram_cm_ws_bytes(n, b, b);
  w.pre = precond_apply_ws(n, b, rcap);
  w.total = w.prep + w.kmm + w.vec + w.small + w.gram + w.pre;
  return w;
}

}  // namespace

size_t block_lanczos_ws_bytes_core(int64_t n, int d, int b, int blocks) { return block_layout(n, d, b, b * blocks).total; }

int block_lanczos_core(const float* X, int64_t n, const egp_hyper_t* h, const float* B0, int b, int blocks, float* Q,
                       double* T, int32_t* rows_out, void* ws, hipStream_t stream, int mode) {
  const int rcap = b * blocks;
  const BlockWs lay = block_layout(n, h->d, b, rcap);
  const int64_t ld = padded_points(n);
  char* w = static_cast<char*>(ws);
  Prepared prep;
  int rc = prepare_points(X, n, h, w, &prep, stream, mode);
  if (rc != EGP_OK) return rc;
  w += lay.prep;
  void* kmm_ws = w;
  w += lay.kmm;
  const size_t vb = round_up((size_t)ld * b * sizeof(float), 256);
  float* V = reinterpret_cast<float*>(w);
  float* W = reinterpret_cast<float*>(w + vb);
  float* W2 = reinterpret_cast<float*>(w + 2 * vb);
  w += lay.vec;
  double* Gdev = reinterpret_cast<double*>(w);
  double* Cfdev = reinterpret_cast<double*>(w + round_up((size_t)32 * 32 * sizeof(double), 256));
  w += lay.small;
  void* gram_ws = w;
  w += lay.gram;
  void* pre_ws = w;

  EGP_HIP(hipMemsetAsync(V, 0, 3 * vb, stream));      // the padding beyond n stays zero throughout
  launch_to_colmajor(B0, n, b, ld, W, stream);

  std::vector<double> G((size_t)b * b), R((size_t)b * b), Rinv((size_t)b * b);
  // dst = src R^{-1} with src^T src = R^T R (upper R). Returns 1 when the block has lost rank.
  auto cholqr = [&](const float* src, float* dst, int* deficient) -> int {
    *deficient = 0;
    int rc2 = gram_cm(src, b, ld, src, b, ld, n, Gdev, gram_ws, stream);
    if (rc2 != EGP_OK) return rc2;
    EGP_HIP(hipMemcpyAsync(G.data(), Gdev, sizeof(double) * b * b, hipMemcpyDeviceToHost, stream));
    EGP_HIP(hipStreamSynchronize(stream));
    double gmax = 0.0;
    for (int i = 0; i < b; ++i) gmax = fmax(gmax, G[(size_t)i * b + i]);
    std::fill(R.begin(), R.end(), 0.0);
    for (int j = 0; j < b; ++j) {            // R^T R = G, R upper: row j of R
      double s = G[(size_t)j * b + j];
      for (int c = 0; c < j; ++c) s -= R[(size_t)c * b + j] * R[(size_t)c * b + j];
      if (!(s > 1e-10 * gmax)) {
        *deficient = 1;
        return EGP_OK;
      }
      const double dj = sqrt(s);
      R[(size_t)j * b + j] = dj;
      for (int i = j + 1; i < b; ++i) {
        double v = 0.5 * (G[(size_t)j * b + i] + G[(size_t)i * b + j]);
        for (int c = 0; c < j; ++c) v -= R[(size_t)c * b + j] * R[(size_t)c * b + i];
        R[(size_t)j * b + i] = v / dj;
      }
    }
    std::fill(Rinv.begin(), Rinv.end(), 0.0);      // upper-triangular inverse by back substitution per column
    for (int c = 0; c < b; ++c) {
      Rinv[(size_t)c * b + c] = 1.0 / R[(size_t)c * b + c];
      for (int i = c - 1; i >= 0; --i) {
        double v = 0.0;
        for (int k = i + 1; k <= c; ++k) v -= R[(size_t)i * b + k] * Rinv[(size_t)k * b + c];
        Rinv[(size_t)i * b + c] = v / R[(size_t)i * b + i];
      }
    }
    EGP_HIP(hipMemcpyAsync(Cfdev, Rinv.data(), sizeof(double) * b * b, hipMemcpyHostToDevice, stream));
    rc2 = combine_cm(src, b, ld, Cfdev, b, n, dst, ld, stream);
    if (rc2 != EGP_OK) return rc2;
    EGP_HIP(hipStreamSynchronize(stream));         // Rinv (host) is reused by the next call
    return EGP_OK;
  };

  int deficient = 0;
  rc = cholqr(W, W2, &deficient);
  if (rc != EGP_OK) return rc;
  if (!deficient) rc = cholqr(W2, V, &deficient);
  if (rc != EGP_OK) return rc;
  if (deficient) return fail(EGP_ERR_ARG, "the start block of the block Lanczos process is rank deficient");
  EGP_HIP(hipMemcpy2DAsync(Q, sizeof(float) * n, V, sizeof(float) * ld, sizeof(float) * n, b,
                           hipMemcpyDeviceToDevice, stream));
  int rtot = b;
  std::vector<double> U((size_t)rcap * rcap, 0.0), C1, C2;
  for (int j = 0; j < blocks; ++j) {
    rc = kmm_core_cm(prep, V, b, W, kmm_ws, nullptr, 0, stream);      // W = Khat V_j
    if (rc != EGP_OK) return rc;
    const double* coef = nullptr;
    int ldy = 0;
    rc = precond_apply_cm(Q, rtot, nullptr, n, 1.0f, W, ld, b, W2, nullptr, 0, pre_ws, stream, &coef, &ldy);
    if (rc != EGP_OK) return rc;
    C1.resize((size_t)rtot * ldy);
    EGP_HIP(hipMemcpyAsync(C1.data(), coef, sizeof(double) * rtot * ldy, hipMemcpyDeviceToHost, stream));
    EGP_HIP(hipStreamSynchronize(stream));
    rc = precond_apply_cm(Q, rtot, nullptr, n, 1.0f, W2, ld, b, W, nullptr, 0, pre_ws, stream, &coef, &ldy);
    if (rc != EGP_OK) return rc;
    C2.resize((size_t)rtot * ldy);
    EGP_HIP(hipMemcpyAsync(C2.data(), coef, sizeof(double) * rtot * ldy, hipMemcpyDeviceToHost, stream));
    EGP_HIP(hipStreamSynchronize(stream));
    for (int i = 0; i < rtot; ++i)
      for (int c = 0; c < b; ++c) U[(size_t)i * rcap + j * b + c] = C1[(size_t)i * ldy + c] + C2[(size_t)i * ldy + c];
    if (j + 1 == blocks) break;
    rc = cholqr(W, W2, &deficient);
    if (rc != EGP_OK) return rc;
    if (!deficient) rc = cholqr(W2, V, &deficient);
    if (rc != EGP_OK) return rc;
    if (deficient) break;                            // invariant subspace reached
    EGP_HIP(hipMemcpy2DAsync(Q + (int64_t)rtot * n, sizeof(float) * n, V, sizeof(float) * ld, sizeof(float) * n, b,
                             hipMemcpyDeviceToDevice, stream));
    rtot += b;
  }
  // T: entries were measured as Q_all^T (Khat V_j); take the upper block triangle, symmetrise the diagonal blocks
  for (size_t e = 0; e < (size_t)rcap * rcap; ++e) T[e] = 0.0;
  for (int i = 0; i < rtot; ++i)
    for (int k = i; k < rtot; ++k) {
      double v = U[(size_t)i * rcap + k];
      if (i / b == k / b) v = 0.5 * (v + U[(size_t)k * rcap + i]);
      T[(size_t)i * rcap + k] = v;
      T[(size_t)k * rcap + i] = v;
    }
  *rows_out = rtot;
  EGP_HIP(hipStreamSynchronize(stream));
  return EGP_OK;
}

size_t cross_ws_bytes_core(int64_t nq, int64_t n, int d, int t) {
  return prepared_bytes(n, d) + prepared_bytes(nq, d) + kmm_cross_ws_bytes(nq, n, t);
}

int cross_core(const float* Xq, int64_t nq, const float* X, int64_t n, const float* V, int t, const egp_hyper_t* h,
               float* out, void* ws, hipStream_t stream, int64_t v_ld, int mode) {
  char* w = static_cast<char*>(ws);
  Prepared P, Qs;
  int rc = prepare_points(X, n, h, w, &P, stream, mode);
  if (rc != EGP_OK) return rc;
  w += prepared_bytes(n, h->d);
  rc = prepare_points(Xq, nq, h, w, &Qs, stream, mode, P.mean);
  if (rc != EGP_OK) return rc;
  w += prepared_bytes(nq, h->d);
  return kmm_cross(P, Qs, V, t, out, w, stream, v_ld);
}

static int predict_cross_t(int r) { return r > 1 ? 33 : 1; }   // widest column group the variance pass can need

size_t predict_ws_bytes_core(int64_t nq, int64_t n, int d, int r) {
  return cross_ws_bytes_core(nq, n, d, predict_cross_t(r)) + round_up((size_t)nq * (r > 0 ? r : 1) * sizeof(float), 256);
}

// mean = K(Xq, X) a; var = s - g^T T^{-1} g with g = Q K(X, xq) (var may be NULL). Synchronises.
int predict_core(const float* Xq, int64_t nq, const float* X, int64_t n, const egp_hyper_t* h, const float* a,
                 const float* Q, int r, const double* alpha, const double* beta, float* mean, float* var, void* ws,
                 hipStream_t stream, int mode, const double* Tdense, int ldt) {
  int rc = cross_core(Xq, nq, X, n, a, 1, h, mean, ws, stream, 0, mode);
  if (rc != EGP_OK) return rc;
  if (var == nullptr) {
    EGP_HIP(hipStreamSynchronize(stream));
    return EGP_OK;
  }
  if (Q == nullptr || r < 1) return fail(EGP_ERR_ARG, "a variance needs the Lanczos cache (Q, alpha, beta)");
  // Cholesky of T (host, fp64): T = Lt Lt^T with Lt lower bidiagonal (diagonal dd, sub-diagonal ee) for the
  // tridiagonal cache, dense lower Ld for the block cache
  std::vector<double> dd(Tdense ? 0 : r), ee(!Tdense && r > 1 ? r - 1 : 0), Ld(Tdense ? (size_t)r * r : 0, 0.0);
  if (Tdense) {
    for (int j = 0; j < r; ++j) {
      double s = Tdense[(size_t)j * ldt + j];
      for (int c = 0; c < j; ++c) s -= Ld[(size_t)j * r + c] * Ld[(size_t)j * r + c];
      if (!(s > 0.0)) return fail(EGP_ERR_BREAKDOWN, "the projected matrix T is not positive definite at row %d", j);
      const double dj = sqrt(s);
      Ld[(size_t)j * r + j] = dj;
      for (int i = j + 1; i < r; ++i) {
        double v = Tdense[(size_t)i * ldt + j];
        const double* li = &Ld[(size_t)i * r];
        const double* lj = &Ld[(size_t)j * r];
        for (int c = 0; c < j; ++c) v -= li[c] * lj[c];
        Ld[(size_t)i * r + j] = v / dj;
      }
    }
  } else {
    for (int j = 0; j < r; ++j) {
      double s = alpha[j] - (j > 0 ? ee[j - 1] * ee[j - 1] : 0.0);
      if (!(s > 0.0)) return fail(EGP_ERR_BREAKDOWN, "the Lanczos tridiagonal is not positive definite at step %d", j);
      dd[j] = sqrt(s);
      if (j + 1 < r) ee[j] = beta[j] / dd[j];
    }
  }
  char* w = static_cast<char*>(ws);
  const size_t sub = cross_ws_bytes_core(nq, n, h->d, predict_cross_t(r));
  float* G = reinterpret_cast<float*>(w + sub);
  rc = cross_core(Xq, nq, X, n, Q, r, h, G, ws, stream, n, mode);      // G (nq x r) = K(Xq, X) Q^T
  if (rc != EGP_OK) return rc;
  std::vector<float> Gh((size_t)nq * r), vh(nq);
  EGP_HIP(hipMemcpyAsync(Gh.data(), G, Gh.size() * sizeof(float), hipMemcpyDeviceToHost, stream));
  EGP_HIP(hipStreamSynchronize(stream));
  std::vector<double> y(r);
  for (int64_t qi = 0; qi < nq; ++qi) {
    // forward substitution Lt y = g, then g^T T^{-1} g = |y|^2
    double acc = 0.0;
    if (Tdense) {
      for (int j = 0; j < r; ++j) {
        double v = (double)Gh[(size_t)qi * r + j];
        const double* lj = &Ld[(size_t)j * r];
        for (int c = 0; c < j; ++c) v -= lj[c] * y[c];
        y[j] = v / lj[j];
        acc += y[j] * y[j];
      }
    } else {
      for (int j = 0; j < r; ++j) {
        double v = (double)Gh[(size_t)qi * r + j];
        if (j > 0) v -= ee[j - 1] * y[j - 1];
        y[j] = v / dd[j];
        acc += y[j] * y[j];
      }
    }
    const double v = (double)h->outputscale - acc;
    vh[qi] = (float)(v > 0.0 ? v : 0.0);      // rounding can leave a tiny negative value where the cache is exact
  }
  EGP_HIP(hipMemcpyAsync(var, vh.data(), sizeof(float) * nq, hipMemcpyHostToDevice, stream));
  EGP_HIP(hipStreamSynchronize(stream));
  return EGP_OK;
}

}  // namespace egp
