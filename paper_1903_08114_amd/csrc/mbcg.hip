// Batched preconditioned conjugate gradients on Khat U = B, all t columns advanced together.
//
// Paper, Background "Conjugate gradients" and Method "O(n) memory MVM-based inference": per column
// the solver keeps four vectors (solution u, residual r, search direction, preconditioned residual z)
// and touches the kernel matrix only through the product Khat D, which is the fused kernel of kmm.hip.
// The modified PCG the paper cites additionally records the CG coefficients alpha_j, beta_j of every
// column, from which the caller builds Lanczos tridiagonals for the log-determinant estimate.
//
// State is held column-major ([t][ld], one right-hand side contiguous, ld = n rounded up to 512 with
// zero padding), so every vector kernel is a 16-byte-per-lane stream over one column (grid.y = column)
// and every per-column scalar is block-uniform. The vector kernels are HBM-bound. Scalars never travel
// to the host inside an iteration: every block re-reduces the per-block partial sums of its column in the
// same fixed order, so all blocks agree on alpha and beta bit for bit. The host reads back only the t
// relative residuals per iteration. d^T Khat d comes for free from the multiply's epilogue.

#include <math.h>

#include <vector>

#include "egp_internal.h"

namespace egp {

namespace {

constexpr int kColBlocks = 64;     // blocks per column in the vector kernels
constexpr int kPartLd = 1024;      // leading dimension of every per-column partial-sum array

__device__ __forceinline__ float block_sum(float v, float* red /*[4]*/) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}

// Sum of `count` partials (fixed order: thread-strided, then the block tree) in double.
__device__ double reduce_partials(const float* __restrict__ part, int count, double* red /*[4]*/) {
  double s = 0.0;
  for (int b = threadIdx.x; b < count; b += 256) s += (double)part[b];
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}

// B (row-major n x t) -> R (column-major), U = 0, optional Z = R; partial sums of b.b per column.
// grid = (kColBlocks, t)
__global__ __launch_bounds__(256) void cg_init(const float* __restrict__ B, int64_t n, int t, int64_t ld,
                                               float* __restrict__ U, float* __restrict__ R,
                                               float* __restrict__ Zopt, float* __restrict__ bb_part) {
  __shared__ float red[4];
  const int c = blockIdx.y;
  float acc = 0.f;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < ld; i += (int64_t)gridDim.x * 256) {
    const float b = i < n ? B[i * t + c] : 0.f;
    const int64_t o = (int64_t)c * ld + i;
    U[o] = 0.f;
    R[o] = b;
    if (Zopt) Zopt[o] = b;
    acc = __builtin_fmaf(b, b, acc);
  }
  const float s = block_sum(acc, red);
  if (threadIdx.x == 0) bb_part[c * kPartLd + blockIdx.x] = s;
}

__global__ __launch_bounds__(256) void cg_copy(const float4* __restrict__ src, int64_t count4,
                                               float4* __restrict__ dst) {
  for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < count4; e += (int64_t)gridDim.x * 256)
    dst[e] = src[e];
}

struct CgLog {
  double* alpha;     // device [max_iter][t]
  double* beta;      // device [max_iter][t]
  float* rel;        // device [t]
  int* breakdown;    // device flag
};

// alpha = gamma / delta; U += alpha D; R -= alpha W; partial sums of r.r.   grid = (kColBlocks, t)
__global__ __launch_bounds__(256) void cg_update(const float* __restrict__ D, const float* __restrict__ W,
                                                 int64_t ld, int t, const float* __restrict__ gamma_part, int gparts,
                                                 const float* __restrict__ delta_part, int dparts,
                                                 float* __restrict__ U, float* __restrict__ R,
                                                 float* __restrict__ rr_part, int iter, CgLog log) {
  __shared__ double redd[4];
  __shared__ float red[4];
  const int c = blockIdx.y;
  const double gamma = reduce_partials(gamma_part + c * kPartLd, gparts, redd);
  const double delta = reduce_partials(delta_part + c * kPartLd, dparts, redd);
  const bool ok = delta > 0.0 && gamma > 0.0;
  const float alpha = ok ? (float)(gamma / delta) : 0.f;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    log.alpha[(int64_t)iter * t + c] = ok ? gamma / delta : 0.0;
    if (gamma > 0.0 && !(delta > 0.0)) *log.breakdown = 1;
  }
  const float4* d4 = reinterpret_cast<const float4*>(D + (int64_t)c * ld);
  const float4* w4 = reinterpret_cast<const float4*>(W + (int64_t)c * ld);
  float4* u4 = reinterpret_cast<float4*>(U + (int64_t)c * ld);
  float4* r4 = reinterpret_cast<float4*>(R + (int64_t)c * ld);
  float acc = 0.f;
  for (int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x; g < (ld >> 2); g += (int64_t)gridDim.x * 256) {
    const float4 d = d4[g], w = w4[g];
    float4 u = u4[g], r = r4[g];
    u.x = __builtin_fmaf(alpha, d.x, u.x); u.y = __builtin_fmaf(alpha, d.y, u.y);
    u.z = __builtin_fmaf(alpha, d.z, u.z); u.w = __builtin_fmaf(alpha, d.w, u.w);
    r.x = __builtin_fmaf(-alpha, w.x, r.x); r.y = __builtin_fmaf(-alpha, w.y, r.y);
    r.z = __builtin_fmaf(-alpha, w.z, r.z); r.w = __builtin_fmaf(-alpha, w.w, r.w);
    u4[g] = u;
    r4[g] = r;
    acc = __builtin_fmaf(r.x, r.x, acc); acc = __builtin_fmaf(r.y, r.y, acc);
    acc = __builtin_fmaf(r.z, r.z, acc); acc = __builtin_fmaf(r.w, r.w, acc);
  }
  const float s = block_sum(acc, red);
  if (threadIdx.x == 0) rr_part[c * kPartLd + blockIdx.x] = s;
}

// beta = gamma_new / gamma_old; D = Z + beta D; block 0 of each column logs beta and the relative residual.
__global__ __launch_bounds__(256) void cg_direction(const float* __restrict__ Z, int64_t ld, int t,
                                                    const float* __restrict__ gnew_part, int gnparts,
                                                    const float* __restrict__ gold_part, int goparts,
                                                    const float* __restrict__ rr_part, int rrparts,
                                                    const float* __restrict__ bb_part, int bbparts,
                                                    float* __restrict__ D, int iter, CgLog log) {
  __shared__ double redd[4];
  const int c = blockIdx.y;
  const double gnew = reduce_partials(gnew_part + c * kPartLd, gnparts, redd);
  const double gold = reduce_partials(gold_part + c * kPartLd, goparts, redd);
  const bool ok = gold > 0.0 && gnew > 0.0;
  const float beta = ok ? (float)(gnew / gold) : 0.f;
  if (blockIdx.x == 0) {
    const double rr = reduce_partials(rr_part + c * kPartLd, rrparts, redd);
    const double bb = reduce_partials(bb_part + c * kPartLd, bbparts, redd);
    if (threadIdx.x == 0) {
      log.beta[(int64_t)iter * t + c] = ok ? gnew / gold : 0.0;
      log.rel[c] = bb > 0.0 ? (float)sqrt(rr / bb) : 0.f;
    }
  }
  const float4* z4 = reinterpret_cast<const float4*>(Z + (int64_t)c * ld);
  float4* d4 = reinterpret_cast<float4*>(D + (int64_t)c * ld);
  for (int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x; g < (ld >> 2); g += (int64_t)gridDim.x * 256) {
    const float4 z = z4[g];
    float4 d = d4[g];
    d.x = __builtin_fmaf(beta, d.x, z.x); d.y = __builtin_fmaf(beta, d.y, z.y);
    d.z = __builtin_fmaf(beta, d.z, z.z); d.w = __builtin_fmaf(beta, d.w, z.w);
    d4[g] = d;
  }
}

// gamma0[c] = total of the gamma partials of column c.  grid = (1, t)
__global__ __launch_bounds__(256) void cg_gamma0(const float* __restrict__ part, int parts, double* __restrict__ out) {
  __shared__ double redd[4];
  const double g = reduce_partials(part + blockIdx.y * kPartLd, parts, redd);
  if (threadIdx.x == 0) out[blockIdx.y] = g;
}

}  // namespace

void launch_to_rowmajor(const float* src, int64_t n, int t, int64_t ld, float* dst, hipStream_t stream);

struct MbcgWs {
  size_t prep, kmm, state, part, log, pre, total;
};

static MbcgWs mbcg_layout(int64_t n, int d, int t, int rank, int max_iter) {
  MbcgWs w;
  const int64_t ld = padded_points(n);
  w.prep = prepared_bytes(n, d);
  w.kmm = kmm_core_ws_bytes(n, t);
  w.state = 5 * round_up((size_t)ld * t * sizeof(float), 256);              // U, R, D, Z, W (column-major)
  w.part = 5 * round_up((size_t)33 * kPartLd * sizeof(float), 256);         // bb, rr, delta, gamma x2
  w.log = round_up((size_t)2 * (max_iter > 0 ? max_iter : 1) * t * sizeof(double), 256) + 1024;
  w.pre = rank > 0 ? precond_apply_ws(n, t, rank) : 0;
  w.total = w.prep + w.kmm + w.state + w.part + w.log + w.pre;
  return w;
}

size_t mbcg_ws_bytes_core(int64_t n, int d, int t, int rank, int max_iter) {
  return mbcg_layout(n, d, t, rank, max_iter).total;
}

int mbcg_core(const float* X, int64_t n, const float* B, int t, const egp_hyper_t* h, const egp_precond_t* P,
              int max_iter, float tol, float* U, double* cg_coef, double* gamma0, int32_t* iters_done,
              float* rel_resid, float* resid_hist, void* ws, hipStream_t stream, const CallOpts& co) {
  const bool shrink = co.shrink;
  const int rank = P ? P->rank : 0;
  const MbcgWs lay = mbcg_layout(n, h->d, t, rank, max_iter);
  const int64_t ld = padded_points(n);
  char* w = static_cast<char*>(ws);
  Prepared prep;
  int rc = prepare_points(X, n, h, w, &prep, stream, co.mode);
  if (rc != EGP_OK) return rc;
  w += lay.prep;
  void* kmm_ws = w;
  w += lay.kmm;
  const size_t vec = round_up((size_t)ld * t * sizeof(float), 256);
  float* Uc = reinterpret_cast<float*>(w);
  float* R = reinterpret_cast<float*>(w + vec);
  float* D = reinterpret_cast<float*>(w + 2 * vec);
  float* Z = reinterpret_cast<float*>(w + 3 * vec);
  float* W = reinterpret_cast<float*>(w + 4 * vec);
  w += lay.state;
  const size_t pb = round_up((size_t)33 * kPartLd * sizeof(float), 256);
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
  double* g0_dev = reinterpret_cast<double*>(tail + 512);     // 33 doubles fit in the remaining 512 bytes
  w += lay.log;
  void* pre_ws = w;

  const int pblocks = precond_apply_blocks(n);
  const int dot_blocks = kmm_cm_dot_blocks(ld);
  int gparts[2];

  EGP_HIP(hipMemsetAsync(log.breakdown, 0, sizeof(int), stream));
  // the coefficient log starts at zero: a column that leaves the iteration early (shrink) keeps zeros from there on
  EGP_HIP(hipMemsetAsync(log.alpha, 0, (size_t)2 * mi * t * sizeof(double), stream));
  hipLaunchKernelGGL(cg_init, dim3(kColBlocks, t), dim3(256), 0, stream, B, n, t, ld, Uc, R, Z, bb_part);   // Z = R also zeroes Z's padding
  if (P) {
    rc = precond_apply_cm(P->L, rank, P->small_dev, n, h->noise, R, ld, t, Z, gam_part[0], kPartLd, pre_ws, stream);
    if (rc != EGP_OK) return rc;
    gparts[0] = pblocks;
  } else {
    hipLaunchKernelGGL(cg_copy, dim3(64), dim3(256), 0, stream, reinterpret_cast<const float4*>(bb_part),
                       (int64_t)t * kPartLd / 4, reinterpret_cast<float4*>(gam_part[0]));
    gparts[0] = kColBlocks;
  }
  hipLaunchKernelGGL(cg_copy, dim3(1024), dim3(256), 0, stream, reinterpret_cast<const float4*>(Z), ld * t / 4,
                     reinterpret_cast<float4*>(D));
  EGP_HIP(hipGetLastError());
  if (gamma0 != nullptr) {
    hipLaunchKernelGGL(cg_gamma0, dim3(1, t), dim3(256), 0, stream, gam_part[0], gparts[0], g0_dev);
    EGP_HIP(hipMemcpyAsync(gamma0, g0_dev, sizeof(double) * t, hipMemcpyDeviceToHost, stream));
    EGP_HIP(hipStreamSynchronize(stream));
  }

  std::vector<float> rel(t, 0.f);
  if (max_iter == 0) {
    // no iteration runs: U = 0, so the residual is b itself and a column's relative residual is 1 (0 for b_c = 0)
    std::vector<float> bb((size_t)t * kPartLd);
    EGP_HIP(hipMemcpyAsync(bb.data(), bb_part, bb.size() * sizeof(float), hipMemcpyDeviceToHost, stream));
    EGP_HIP(hipStreamSynchronize(stream));
    for (int c = 0; c < t; ++c) {
      double s = 0.0;
      for (int b = 0; b < kColBlocks; ++b) s += (double)bb[(size_t)c * kPartLd + b];
      rel[c] = s > 0.0 ? 1.f : 0.f;
    }
  }
  int it = 0;
  int cur = 0;
  // Columns [0, ta) take part in an iteration. Without `shrink` ta stays t (converged columns keep iterating, which
  // is harmless); with it, trailing columns that have met the tolerance leave: every kernel below works on a prefix
  // of the column-major state arrays, and t remains the stride of the coefficient log.
  int ta = t;
  for (; it < max_iter;) {
    const dim3 vgrid(kColBlocks, ta);
    rc = kmm_core_cm(prep, D, ta, W, kmm_ws, delta_part, kPartLd, stream);
    if (rc != EGP_OK) return rc;
    {
      ProfScope vprof(kProfCgVec, stream);
      hipLaunchKernelGGL(cg_update, vgrid, dim3(256), 0, stream, D, W, ld, t, gam_part[cur], gparts[cur], delta_part,
                         dot_blocks, Uc, R, rr_part, it, log);
    }
    const int nxt = cur ^ 1;
    const float* Zsrc;
    if (P) {
      rc = precond_apply_cm(P->L, rank, P->small_dev, n, h->noise, R, ld, ta, Z, gam_part[nxt], kPartLd, pre_ws,
                            stream);
      if (rc != EGP_OK) return rc;
      gparts[nxt] = pblocks;
      Zsrc = Z;
    } else {
      hipLaunchKernelGGL(cg_copy, dim3(64), dim3(256), 0, stream, reinterpret_cast<const float4*>(rr_part),
                         (int64_t)ta * kPartLd / 4, reinterpret_cast<float4*>(gam_part[nxt]));
      gparts[nxt] = kColBlocks;
      Zsrc = R;
    }
    {
      ProfScope dprof(kProfCgVec, stream);
      hipLaunchKernelGGL(cg_direction, vgrid, dim3(256), 0, stream, Zsrc, ld, t, gam_part[nxt], gparts[nxt],
                         gam_part[cur], gparts[cur], rr_part, kColBlocks, bb_part, kColBlocks, D, it, log);
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
    if (shrink)
      while (ta > 1 && rel[ta - 1] <= tol) --ta;
  }
  launch_to_rowmajor(Uc, n, t, ld, U, stream);
  EGP_HIP(hipGetLastError());
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
