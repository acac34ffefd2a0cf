// Batched preconditioned conjugate gradients on Khat U = B, all t columns advanced together.
//
// Paper, Background "Conjugate gradients" and Method "O(n) memory MVM-based inference": per column
// the solver keeps four vectors (solution u, residual r, search direction, preconditioned residual z)
// and touches the kernel matrix only through the product Khat D, which is the fused kernel of kmm.hip.
// The modified PCG the paper cites additionally records the CG coefficients alpha_j, beta_j of every
// column, from which the caller builds Lanczos tridiagonals for the log-determinant estimate.
//
// The vector kernels below are HBM-bound. Per-column scalars never travel to the host inside an
// iteration: every block re-reduces the per-block partial sums in the same fixed order, so all blocks
// agree on alpha and beta bit for bit. The host reads back only the t relative residuals per iteration.

#include <math.h>

#include <vector>

#include "egp_internal.h"

namespace egp {

int precond_apply_blocks(int64_t n);
size_t precond_apply_ws(int64_t n, int t, int rank);
int precond_apply_core(const float* L, int rank, const float* Minv_dev, int64_t n, float noise, const float* R,
                       int t, float* Z, float* rz_partial, void* ws, hipStream_t stream);

namespace {

constexpr int kVecBlocks = 1024;
constexpr int kTMax = 33;

// Thread layout of the vector kernels: TP = power of two >= t columns, 256/TP rows per pass.
struct Lay { int tp, rows; };
Lay layout_for(int t) {
  int tp = 1;
  while (tp < t) tp *= 2;
  if (tp < 16) tp = 16;
  return {tp, 256 / tp};
}

// Sum `parts` per-block partials of column c in a fixed order (identical in every block).
__device__ float reduce_partials(const float* __restrict__ part, int parts, int t, int c, int rl, int rows,
                                 float* sh /*[256]*/) {
  double s = 0.0;
  if (c < t)
    for (int b = rl; b < parts; b += rows) s += (double)part[(int64_t)b * t + c];
  __syncthreads();
  sh[threadIdx.x] = (float)s;
  __syncthreads();
  double tot = 0.0;
  const int tp = 256 / rows;
  if (c < t)
    for (int r = 0; r < rows; ++r) tot += (double)sh[r * tp + c];
  return (float)tot;
}

// Per-block column sums of `val` (thread (rl, c)) -> out[blockIdx][c].
__device__ void write_partial(float val, int t, int c, int rl, int rows, float* sh, float* __restrict__ out) {
  __syncthreads();
  sh[threadIdx.x] = val;
  __syncthreads();
  if (rl == 0 && c < t) {
    const int tp = 256 / rows;
    float s = 0.f;
    for (int r = 0; r < rows; ++r) s += sh[r * tp + c];
    out[(int64_t)blockIdx.x * t + c] = s;
  }
}

// R = B, U = 0, (Z = R when there is no preconditioner), partial sums of B.B
__global__ __launch_bounds__(256) void cg_init(const float* __restrict__ B, int64_t n, int t, int tp,
                                               float* __restrict__ U, float* __restrict__ R,
                                               float* __restrict__ Zopt, float* __restrict__ bb_part) {
  __shared__ float sh[256];
  const int rows = 256 / tp, c = threadIdx.x % tp, rl = threadIdx.x / tp;
  float acc = 0.f;
  if (c < t)
    for (int64_t i = (int64_t)blockIdx.x * rows + rl; i < n; i += (int64_t)gridDim.x * rows) {
      const float b = B[i * t + c];
      U[i * t + c] = 0.f;
      R[i * t + c] = b;
      if (Zopt) Zopt[i * t + c] = b;
      acc = __builtin_fmaf(b, b, acc);
    }
  write_partial(acc, t, c, rl, rows, sh, bb_part);
}

__global__ __launch_bounds__(256) void cg_copy(const float* __restrict__ src, int64_t count,
                                               float* __restrict__ dst) {
  for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < count; e += (int64_t)gridDim.x * 256)
    dst[e] = src[e];
}

// partial sums of D.W per column
__global__ __launch_bounds__(256) void cg_dot(const float* __restrict__ D, const float* __restrict__ W, int64_t n,
                                              int t, int tp, float* __restrict__ part) {
  __shared__ float sh[256];
  const int rows = 256 / tp, c = threadIdx.x % tp, rl = threadIdx.x / tp;
  float acc = 0.f;
  if (c < t)
    for (int64_t i = (int64_t)blockIdx.x * rows + rl; i < n; i += (int64_t)gridDim.x * rows)
      acc = __builtin_fmaf(D[i * t + c], W[i * t + c], acc);
  write_partial(acc, t, c, rl, rows, sh, part);
}

struct CgLog {
  double* alpha;     // device [max_iter][t]
  double* beta;      // device [max_iter][t]
  float* rel;        // device [t]
  int* breakdown;    // device flag
};

// alpha = gamma / delta; U += alpha D; R -= alpha W; partial sums of R.R
__global__ __launch_bounds__(256) void cg_update(const float* __restrict__ D, const float* __restrict__ W,
                                                 int64_t n, int t, int tp, const float* __restrict__ gamma_part,
                                                 int gparts, const float* __restrict__ delta_part, int dparts,
                                                 float* __restrict__ U, float* __restrict__ R,
                                                 float* __restrict__ rr_part, int iter, CgLog log) {
  __shared__ float sh[256];
  const int rows = 256 / tp, c = threadIdx.x % tp, rl = threadIdx.x / tp;
  const float gamma = reduce_partials(gamma_part, gparts, t, c, rl, rows, sh);
  const float delta = reduce_partials(delta_part, dparts, t, c, rl, rows, sh);
  float alpha = 0.f;
  if (c < t) {
    if (delta > 0.f && gamma > 0.f) alpha = gamma / delta;
    if (blockIdx.x == 0 && rl == 0) {
      log.alpha[(int64_t)iter * t + c] = (delta > 0.f && gamma > 0.f) ? (double)gamma / (double)delta : 0.0;
      if (gamma > 0.f && !(delta > 0.f)) *log.breakdown = 1;
    }
  }
  float acc = 0.f;
  if (c < t)
    for (int64_t i = (int64_t)blockIdx.x * rows + rl; i < n; i += (int64_t)gridDim.x * rows) {
      const int64_t o = i * t + c;
      U[o] = __builtin_fmaf(alpha, D[o], U[o]);
      const float r = __builtin_fmaf(-alpha, W[o], R[o]);
      R[o] = r;
      acc = __builtin_fmaf(r, r, acc);
    }
  write_partial(acc, t, c, rl, rows, sh, rr_part);
}

// beta = gamma_new / gamma_old; D = Z + beta D; block 0 also logs beta and the relative residuals.
__global__ __launch_bounds__(256) void cg_direction(const float* __restrict__ Z, int64_t n, int t, int tp,
                                                    const float* __restrict__ gnew_part, int gnparts,
                                                    const float* __restrict__ gold_part, int goparts,
                                                    const float* __restrict__ rr_part, int rrparts,
                                                    const float* __restrict__ bb_part, int bbparts,
                                                    float* __restrict__ D, int iter, CgLog log) {
  __shared__ float sh[256];
  const int rows = 256 / tp, c = threadIdx.x % tp, rl = threadIdx.x / tp;
  const float gnew = reduce_partials(gnew_part, gnparts, t, c, rl, rows, sh);
  const float gold = reduce_partials(gold_part, goparts, t, c, rl, rows, sh);
  float beta = 0.f;
  if (c < t && gold > 0.f && gnew > 0.f) beta = gnew / gold;
  if (blockIdx.x == 0) {
    const float rr = reduce_partials(rr_part, rrparts, t, c, rl, rows, sh);
    const float bb = reduce_partials(bb_part, bbparts, t, c, rl, rows, sh);
    if (c < t && rl == 0) {
      log.beta[(int64_t)iter * t + c] = (gold > 0.f && gnew > 0.f) ? (double)gnew / (double)gold : 0.0;
      log.rel[c] = bb > 0.f ? sqrtf(rr / bb) : 0.f;
    }
  }
  if (c < t)
    for (int64_t i = (int64_t)blockIdx.x * rows + rl; i < n; i += (int64_t)gridDim.x * rows) {
      const int64_t o = i * t + c;
      D[o] = __builtin_fmaf(beta, D[o], Z[o]);
    }
}

// gamma0[c] = total of gamma partials (one block)
__global__ __launch_bounds__(256) void cg_gamma0(const float* __restrict__ part, int parts, int t, int tp,
                                                 double* __restrict__ out) {
  __shared__ float sh[256];
  const int rows = 256 / tp, c = threadIdx.x % tp, rl = threadIdx.x / tp;
  const float g = reduce_partials(part, parts, t, c, rl, rows, sh);
  if (c < t && rl == 0) out[c] = (double)g;
}

}  // namespace

struct MbcgWs {
  size_t prep, kmm, state, part, log, pre, total;
};

static MbcgWs mbcg_layout(int64_t n, int d, int t, int rank, int max_iter) {
  MbcgWs w;
  w.prep = prepared_bytes(n, d);
  w.kmm = kmm_core_ws_bytes(n, t);
  w.state = 4 * round_up((size_t)n * t * sizeof(float), 256);               // R, D, Z, W
  w.part = 5 * round_up((size_t)kVecBlocks * kTMax * sizeof(float), 256);   // bb, rr, delta, gamma x2
  w.log = round_up((size_t)2 * (max_iter > 0 ? max_iter : 1) * t * sizeof(double), 256) + 512;
  w.pre = rank > 0 ? precond_apply_ws(n, t, rank) : 0;
  w.total = w.prep + w.kmm + w.state + w.part + w.log + w.pre;
  return w;
}

size_t mbcg_ws_bytes_core(int64_t n, int d, int t, int rank, int max_iter) {
  return mbcg_layout(n, d, t, rank, max_iter).total;
}

int mbcg_core(const float* X, int64_t n, const float* B, int t, const egp_hyper_t* h, const egp_precond_t* P,
              int max_iter, float tol, float* U, double* cg_coef, double* gamma0, int32_t* iters_done,
              float* rel_resid, float* resid_hist, void* ws, hipStream_t stream) {
  const int rank = P ? P->rank : 0;
  const MbcgWs lay = mbcg_layout(n, h->d, t, rank, max_iter);
  char* w = static_cast<char*>(ws);
  Prepared prep;
  int rc = prepare_points(X, n, h, w, &prep, stream);
  if (rc != EGP_OK) return rc;
  w += lay.prep;
  void* kmm_ws = w;
  w += lay.kmm;
  const size_t vec = round_up((size_t)n * t * sizeof(float), 256);
  float* R = reinterpret_cast<float*>(w);
  float* D = reinterpret_cast<float*>(w + vec);
  float* Z = reinterpret_cast<float*>(w + 2 * vec);
  float* W = reinterpret_cast<float*>(w + 3 * vec);
  w += lay.state;
  const size_t pb = round_up((size_t)kVecBlocks * kTMax * sizeof(float), 256);
  float* bb_part = reinterpret_cast<float*>(w);
  float* rr_part = reinterpret_cast<float*>(w + pb);
  float* delta_part = reinterpret_cast<float*>(w + 2 * pb);
  float* gam_part[2] = {reinterpret_cast<float*>(w + 3 * pb), reinterpret_cast<float*>(w + 4 * pb)};
  w += lay.part;
  CgLog log;
  const int mi = max_iter > 0 ? max_iter : 1;
  log.alpha = reinterpret_cast<double*>(w);
  log.beta = log.alpha + (size_t)mi * t;
  char* tail = w + round_up((size_t)2 * mi * t * sizeof(double), 256);
  log.rel = reinterpret_cast<float*>(tail);
  log.breakdown = reinterpret_cast<int*>(tail + 256);
  w += lay.log;
  void* pre_ws = w;

  const Lay ly = layout_for(t);
  int64_t want = (n + ly.rows - 1) / ly.rows;
  const int blocks = (int)(want > kVecBlocks ? kVecBlocks : want);
  const int pblocks = precond_apply_blocks(n);
  // with a preconditioner gamma partials come from the Woodbury kernel (pblocks of them), else they
  // are the r.r partials of the update kernel (blocks of them)
  int gparts[2];

  EGP_HIP(hipMemsetAsync(log.breakdown, 0, sizeof(int), stream));
  hipLaunchKernelGGL(cg_init, dim3(blocks), dim3(256), 0, stream, B, n, t, ly.tp, U, R, P ? nullptr : Z, bb_part);
  if (P) {
    rc = precond_apply_core(P->L, rank, P->small_dev, n, h->noise, R, t, Z, gam_part[0], pre_ws, stream);
    if (rc != EGP_OK) return rc;
    gparts[0] = pblocks;
  } else {
    hipLaunchKernelGGL(cg_copy, dim3(blocks), dim3(256), 0, stream, bb_part, (int64_t)blocks * t, gam_part[0]);
    gparts[0] = blocks;
  }
  hipLaunchKernelGGL(cg_copy, dim3(1024), dim3(256), 0, stream, Z, n * t, D);
  EGP_HIP(hipGetLastError());
  if (gamma0 != nullptr) {
    // reuse the start of delta_part as a staging area for t doubles
    double* g0 = reinterpret_cast<double*>(delta_part);
    hipLaunchKernelGGL(cg_gamma0, dim3(1), dim3(256), 0, stream, gam_part[0], gparts[0], t, ly.tp, g0);
    EGP_HIP(hipMemcpyAsync(gamma0, g0, sizeof(double) * t, hipMemcpyDeviceToHost, stream));
    EGP_HIP(hipStreamSynchronize(stream));
  }

  std::vector<float> rel(t, 0.f);
  int it = 0;
  int cur = 0;
  for (; it < max_iter;) {
    rc = kmm_core(prep, D, t, W, kmm_ws, stream);
    if (rc != EGP_OK) return rc;
    ProfScope* vprof = new ProfScope(kProfCgVec, stream);
    hipLaunchKernelGGL(cg_dot, dim3(blocks), dim3(256), 0, stream, D, W, n, t, ly.tp, delta_part);
    hipLaunchKernelGGL(cg_update, dim3(blocks), dim3(256), 0, stream, D, W, n, t, ly.tp, gam_part[cur],
                       gparts[cur], delta_part, blocks, U, R, rr_part, it, log);
    delete vprof;
    const int nxt = cur ^ 1;
    const float* Zsrc;
    if (P) {
      rc = precond_apply_core(P->L, rank, P->small_dev, n, h->noise, R, t, Z, gam_part[nxt], pre_ws, stream);
      if (rc != EGP_OK) return rc;
      gparts[nxt] = pblocks;
      Zsrc = Z;
    } else {
      hipLaunchKernelGGL(cg_copy, dim3(blocks), dim3(256), 0, stream, rr_part, (int64_t)blocks * t, gam_part[nxt]);
      gparts[nxt] = blocks;
      Zsrc = R;
    }
    {
      ProfScope dprof(kProfCgVec, stream);
      hipLaunchKernelGGL(cg_direction, dim3(blocks), dim3(256), 0, stream, Zsrc, n, t, ly.tp, gam_part[nxt],
                         gparts[nxt], gam_part[cur], gparts[cur], rr_part, blocks, bb_part, blocks, D, it, log);
    }
    EGP_HIP(hipGetLastError());
    EGP_HIP(hipMemcpyAsync(rel.data(), log.rel, sizeof(float) * t, hipMemcpyDeviceToHost, stream));
    EGP_HIP(hipStreamSynchronize(stream));
    cur = nxt;
    ++it;
    float worst = 0.f;
    bool finite = true;
    if (resid_hist)
      for (int c = 0; c < t; ++c) resid_hist[(size_t)(it - 1) * t + c] = rel[c];
    for (int c = 0; c < t; ++c) {
      if (!std::isfinite(rel[c])) finite = false;
      if (rel[c] > worst) worst = rel[c];
    }
    if (!finite) {
      if (iters_done) *iters_done = it;
      return fail(EGP_ERR_BREAKDOWN, "non-finite residual at iteration %d", it);
    }
    if (worst <= tol) break;
  }
  if (iters_done) *iters_done = it;
  if (rel_resid)
    for (int c = 0; c < t; ++c) rel_resid[c] = rel[c];
  int broke = 0;
  EGP_HIP(hipMemcpyAsync(&broke, log.breakdown, sizeof(int), hipMemcpyDeviceToHost, stream));
  if (cg_coef != nullptr && it > 0) {
    std::vector<double> a((size_t)it * t), b((size_t)it * t);
    EGP_HIP(hipMemcpyAsync(a.data(), log.alpha, sizeof(double) * it * t, hipMemcpyDeviceToHost, stream));
    EGP_HIP(hipMemcpyAsync(b.data(), log.beta, sizeof(double) * it * t, hipMemcpyDeviceToHost, stream));
    EGP_HIP(hipStreamSynchronize(stream));
    for (int j = 0; j < it; ++j)
      for (int c = 0; c < t; ++c) {
        cg_coef[((size_t)j * 2 + 0) * t + c] = a[(size_t)j * t + c];
        cg_coef[((size_t)j * 2 + 1) * t + c] = (j + 1 < it) ? b[(size_t)j * t + c] : 0.0;
      }
  }
  EGP_HIP(hipStreamSynchronize(stream));
  if (broke) return fail(EGP_ERR_BREAKDOWN, "non-positive curvature d^T Khat d met during CG");
  return EGP_OK;
}

}  // namespace egp
