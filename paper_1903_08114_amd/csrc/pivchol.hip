// Partial pivoted Cholesky of the noise-free kernel matrix from kernel rows computed on the fly, and
// application of the resulting preconditioner P = L L^T + noise I through the Woodbury identity.
//
// Paper, Method, "Preconditioning": a rank-k pivoted-Cholesky preconditioner needs only k kernel rows
// and is built once before any CG iteration. The paper cites the algorithm; the steps here are the
// textbook diagonal-pivoting Cholesky (greedy largest residual diagonal, ties to the lowest index),
// without row swaps: L stays in original row order.
//
// All k steps are enqueued without a host round trip: step m first reduces the per-block arg-max
// candidates that step m-1 left (every block does the same reduction in the same order, so all agree),
// then forms column m.  HBM-bound: step m reads n (d + m) floats.

#include <math.h>

#include <vector>

#include "egp_internal.h"

namespace egp {

namespace {

constexpr int kPcBlocks = 1024;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ float transform_rt(int kind, float acc) {
  if (kind == EGP_RBF) return __builtin_amdgcn_exp2f(-acc);
  const float a = __builtin_amdgcn_sqrtf(__builtin_fabsf(acc));
  const float e = __builtin_amdgcn_exp2f(-a);
  if (kind == EGP_MATERN32) return __builtin_fmaf(a, kLn2, 1.0f) * e;
  return __builtin_fmaf(__builtin_fmaf(a, kLn2 * kLn2 / 3.0f, kLn2), a, 1.0f) * e;
}

struct Cand { float v; int i; };
__device__ __forceinline__ Cand better(Cand a, Cand b) {
  // larger value wins; on equal values the lower index wins
  if (b.v > a.v || (b.v == a.v && b.i < a.i)) return b;
  return a;
}

__device__ Cand block_argmax(Cand c, Cand* sh /*[4]*/) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    Cand o;
    o.v = __shfl_xor(c.v, off);
    o.i = __shfl_xor(c.i, off);
    c = better(c, o);
  }
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) sh[wave] = c;
  __syncthreads();
  Cand r = sh[0];
  r = better(r, sh[1]);
  r = better(r, sh[2]);
  r = better(r, sh[3]);
  __syncthreads();
  return r;
}

struct PcState {
  int* pivots;     // [rank]
  int* rank_out;   // steps taken
  int* stop;       // sticky flag
  float* cand_v;   // [2][kPcBlocks]
  int* cand_i;     // [2][kPcBlocks]
};

__global__ __launch_bounds__(256) void pc_init(float* __restrict__ diag, int64_t n, float s, PcState st,
                                               int rank) {
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) diag[i] = s;
  if (i == 0) {
    *st.stop = 0;
    *st.rank_out = rank;
  }
}

// One step of the factorisation. Points are read from the packed MFMA-operand layout.
__global__ __launch_bounds__(256) void pc_step(const float* __restrict__ Xp, int ks, int d, int kind, float s,
                                               int64_t n, float* __restrict__ L, float* __restrict__ diag, int m,
                                               float tol_abs, PcState st) {
  __shared__ Cand sh[4];
  __shared__ float xpiv[EGP_D_MAX + 1];
  __shared__ float lrow[EGP_RANK_MAX];
  if (*st.stop) return;

  // ---- pivot of this step ----
  Cand w;
  if (m == 0) {
    w.v = s;      // diag K = s everywhere: an n-way tie, resolved to the lowest index
    w.i = 0;
  } else {
    const float* cv = st.cand_v + (m & 1) * kPcBlocks;
    const int* ci = st.cand_i + (m & 1) * kPcBlocks;
    Cand c = {-INFINITY, 0x7fffffff};
    for (int b = threadIdx.x; b < (int)gridDim.x; b += 256) c = better(c, (Cand){cv[b], ci[b]});
    w = block_argmax(c, sh);
  }
  if (!(w.v > tol_abs)) {
    if (blockIdx.x == 0 && threadIdx.x == 0) {
      *st.stop = 1;
      *st.rank_out = m;
    }
    return;
  }
  const int64_t piv = w.i;
  if (blockIdx.x == 0 && threadIdx.x == 0) st.pivots[m] = w.i;

  const float* pbase = Xp + (piv >> 4) * ks * 64 + (piv & 15);
  for (int f = threadIdx.x; f < d; f += 256) xpiv[f] = pbase[(f >> 2) * 64 + (f & 3) * 16];
  for (int c = threadIdx.x; c < m; c += 256) lrow[c] = L[(int64_t)c * n + piv];
  __syncthreads();
  const float root = sqrtf(w.v);
  const float inv_root = 1.0f / root;

  Cand best = {-INFINITY, 0x7fffffff};
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const float dg = diag[i];
    float col;
    float newd;
    if (i == piv) {
      col = root;
      newd = -INFINITY;
    } else if (dg == -INFINITY) {      // chosen earlier
      col = 0.f;
      newd = -INFINITY;
    } else {
      const float* xb = Xp + (i >> 4) * ks * 64 + (i & 15);
      float r2 = 0.f;
      for (int f = 0; f < d; ++f) {
        const float df = xpiv[f] - xb[(f >> 2) * 64 + (f & 3) * 16];
        r2 = __builtin_fmaf(df, df, r2);
      }
      float acc = s * transform_rt(kind, r2);
      const float* Li = L + i;
      int c = 0;
      float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
      for (; c + 4 <= m; c += 4) {
        a0 = __builtin_fmaf(Li[(int64_t)(c + 0) * n], lrow[c + 0], a0);
        a1 = __builtin_fmaf(Li[(int64_t)(c + 1) * n], lrow[c + 1], a1);
        a2 = __builtin_fmaf(Li[(int64_t)(c + 2) * n], lrow[c + 2], a2);
        a3 = __builtin_fmaf(Li[(int64_t)(c + 3) * n], lrow[c + 3], a3);
      }
      for (; c < m; ++c) a0 = __builtin_fmaf(Li[(int64_t)c * n], lrow[c], a0);
      acc -= (a0 + a1) + (a2 + a3);
      col = acc * inv_root;
      newd = dg - col * col;
    }
    L[(int64_t)m * n + i] = col;
    diag[i] = newd;
    best = better(best, (Cand){newd, (int)i});
  }
  best = block_argmax(best, sh);
  if (threadIdx.x == 0) {
    st.cand_v[((m + 1) & 1) * kPcBlocks + blockIdx.x] = best.v;
    st.cand_i[((m + 1) & 1) * kPcBlocks + blockIdx.x] = best.i;
  }
}

// ---- C[a][b] (+)= sum_i A[a][i] * B(b,i) over a chunk of i: generic 64x64 tile, 4x4 per thread ----
// A is [ra][n] (rows contiguous in i). B is either [rb][n] (BT = false) or [n][rb] row-major (BT = true).
// Partial results go to Cp[chunk][ra][rb]; a second kernel sums chunks in order.
template <bool BT>
__global__ __launch_bounds__(256) void nt_gemm_partial(const float* __restrict__ A, int ra,
                                                       const float* __restrict__ B, int rb, int64_t n,
                                                       int64_t chunk, float* __restrict__ Cp) {
  __shared__ float As[16][64 + 1];
  __shared__ float Bs[16][64 + 1];
  const int ta = blockIdx.y * 64, tb = blockIdx.z * 64;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int64_t i_begin = (int64_t)blockIdx.x * chunk;
  int64_t i_end = i_begin + chunk;
  if (i_end > n) i_end = n;
  float acc[4][4] = {};
  for (int64_t i0 = i_begin; i0 < i_end; i0 += 16) {
    // load 64 rows x 16 points of A (coalesced over i within a row)
    for (int e = threadIdx.x; e < 64 * 16; e += 256) {
      const int r = e >> 4, ii = e & 15;
      const int64_t i = i0 + ii;
      As[ii][r] = (ta + r < ra && i < i_end) ? A[(int64_t)(ta + r) * n + i] : 0.f;
    }
    if (!BT) {
      for (int e = threadIdx.x; e < 64 * 16; e += 256) {
        const int r = e >> 4, ii = e & 15;
        const int64_t i = i0 + ii;
        Bs[ii][r] = (tb + r < rb && i < i_end) ? B[(int64_t)(tb + r) * n + i] : 0.f;
      }
    } else {
      for (int e = threadIdx.x; e < 64 * 16; e += 256) {
        const int ii = e >> 6, r = e & 63;
        const int64_t i = i0 + ii;
        Bs[ii][r] = (tb + r < rb && i < i_end) ? B[i * rb + tb + r] : 0.f;
      }
    }
    __syncthreads();
#pragma unroll
    for (int ii = 0; ii < 16; ++ii) {
      float av[4], bv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        av[u] = As[ii][ty * 4 + u];
        bv[u] = Bs[ii][tx * 4 + u];
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[u][v] = __builtin_fmaf(av[u], bv[v], acc[u][v]);
    }
    __syncthreads();
  }
  float* dst = Cp + (int64_t)blockIdx.x * ra * rb;
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int a = ta + ty * 4 + u, b = tb + tx * 4 + v;
      if (a < ra && b < rb) dst[a * rb + b] = acc[u][v];
    }
}

__global__ __launch_bounds__(256) void sum_chunks(const float* __restrict__ Cp, int chunks, int count,
                                                  float* __restrict__ C) {
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= count) return;
  double s = 0.0;
  for (int c = 0; c < chunks; ++c) s += (double)Cp[(int64_t)c * count + e];
  C[e] = (float)s;
}

// Y[c][tc] = sum_c' Minv[c][c'] * W[c'][tc] with W = sum over chunks of Wp (one block).
__global__ __launch_bounds__(256) void small_solve(const float* __restrict__ Wp, int chunks, int k, int t,
                                                   const float* __restrict__ Minv, float* __restrict__ Y) {
  extern __shared__ float Wsum[];   // k * t
  for (int e = threadIdx.x; e < k * t; e += 256) {
    double s = 0.0;
    for (int c = 0; c < chunks; ++c) s += (double)Wp[(int64_t)c * k * t + e];
    Wsum[e] = (float)s;
  }
  __syncthreads();
  for (int e = threadIdx.x; e < k * t; e += 256) {
    const int c = e / t, tc = e % t;
    float acc = 0.f;
    for (int c2 = 0; c2 < k; ++c2) acc = __builtin_fmaf(Minv[c * k + c2], Wsum[c2 * t + tc], acc);
    Y[e] = acc;
  }
}

// Z[i][:] = (R[i][:] - sum_c L[c][i] Y[c][:]) / noise; optional per-block partial of sum_i R[i][c] Z[i][c].
// One thread per point; TT = compile-time bound on t so the outputs stay in registers.
template <int TT>
__global__ __launch_bounds__(256) void woodbury_finish(const float* __restrict__ L, int k, int64_t n,
                                                       const float* __restrict__ Y, const float* __restrict__ R,
                                                       int t, float inv_noise, float* __restrict__ Z,
                                                       float* __restrict__ rz_partial /*[grid][t] or null*/) {
  extern __shared__ float sh[];      // Y: k * t, then reduction scratch 4 * t
  float* Ys = sh;
  float* red = sh + k * t;
  for (int e = threadIdx.x; e < k * t; e += 256) Ys[e] = Y[e];
  __syncthreads();
  float dot[TT];
#pragma unroll
  for (int c = 0; c < TT; ++c) dot[c] = 0.f;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    float acc[TT];
#pragma unroll
    for (int c = 0; c < TT; ++c) acc[c] = 0.f;
    for (int c2 = 0; c2 < k; ++c2) {
      const float l = L[(int64_t)c2 * n + i];
      const float* y = Ys + c2 * t;
#pragma unroll
      for (int c = 0; c < TT; ++c)
        if (c < t) acc[c] = __builtin_fmaf(l, y[c], acc[c]);
    }
#pragma unroll
    for (int c = 0; c < TT; ++c)
      if (c < t) {
        const float r = R[i * t + c];
        const float z = (r - acc[c]) * inv_noise;
        Z[i * t + c] = z;
        dot[c] = __builtin_fmaf(r, z, dot[c]);
      }
  }
  if (rz_partial != nullptr) {
#pragma unroll
    for (int c = 0; c < TT; ++c) {
      if (c < t) {
        float v = dot[c];
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
        if ((threadIdx.x & 63) == 0) red[(threadIdx.x >> 6) * t + c] = v;
      }
    }
    __syncthreads();
    if ((int)threadIdx.x < t)
      rz_partial[(int64_t)blockIdx.x * t + threadIdx.x] =
          (red[threadIdx.x] + red[t + threadIdx.x]) + (red[2 * t + threadIdx.x] + red[3 * t + threadIdx.x]);
  }
}

int chunks_for(int64_t n, int64_t* chunk_out) {
  int64_t chunk = 4096;
  while ((n + chunk - 1) / chunk > 512) chunk *= 2;
  *chunk_out = chunk;
  return (int)((n + chunk - 1) / chunk);
}

}  // namespace

int precond_apply_blocks(int64_t n) {
  int64_t b = (n + 255) / 256;
  return (int)(b > 1024 ? 1024 : b);
}

size_t precond_apply_ws(int64_t n, int t, int rank) {
  int64_t chunk;
  const int chunks = chunks_for(n, &chunk);
  return round_up((size_t)chunks * rank * t * sizeof(float), 256) + round_up((size_t)rank * t * sizeof(float), 256);
}

// Z = P^{-1} R; rz_partial (optional) receives precond_apply_blocks(n) x t partial sums of R.Z per column.
int precond_apply_core(const float* L, int rank, const float* Minv_dev, int64_t n, float noise, const float* R,
                       int t, float* Z, float* rz_partial, void* ws, hipStream_t stream) {
  if (t > 33) return fail(EGP_ERR_ARG, "preconditioner application supports t <= 33 (got %d)", t);
  ProfScope prof(kProfPrecond, stream);
  int64_t chunk;
  const int chunks = chunks_for(n, &chunk);
  char* w = static_cast<char*>(ws);
  float* Wp = reinterpret_cast<float*>(w);
  w += round_up((size_t)chunks * rank * t * sizeof(float), 256);
  float* Y = reinterpret_cast<float*>(w);
  dim3 grid(chunks, (rank + 63) / 64, (t + 63) / 64);
  hipLaunchKernelGGL(nt_gemm_partial<true>, grid, dim3(256), 0, stream, L, rank, R, t, n, chunk, Wp);
  hipLaunchKernelGGL(small_solve, dim3(1), dim3(256), (size_t)rank * t * sizeof(float), stream, Wp, chunks, rank,
                     t, Minv_dev, Y);
  const int blocks = precond_apply_blocks(n);
  const size_t shb = ((size_t)rank * t + 4 * t) * sizeof(float);
  const float inv_noise = 1.0f / noise;
  if (t <= 16)
    hipLaunchKernelGGL(woodbury_finish<16>, dim3(blocks), dim3(256), shb, stream, L, rank, n, Y, R, t, inv_noise,
                       Z, rz_partial);
  else if (t <= 17)
    hipLaunchKernelGGL(woodbury_finish<17>, dim3(blocks), dim3(256), shb, stream, L, rank, n, Y, R, t, inv_noise,
                       Z, rz_partial);
  else
    hipLaunchKernelGGL(woodbury_finish<33>, dim3(blocks), dim3(256), shb, stream, L, rank, n, Y, R, t, inv_noise,
                       Z, rz_partial);
  EGP_HIP(hipGetLastError());
  return EGP_OK;
}

size_t pivchol_ws_bytes(int64_t n, int d, int rank) {
  int64_t chunk;
  const int chunks = chunks_for(n, &chunk);
  size_t b = prepared_bytes(n, d);
  b += round_up((size_t)n * sizeof(float), 256);                          // diag
  b += round_up((size_t)rank * sizeof(int), 256);                         // pivots
  b += 256;                                                               // rank, stop
  b += round_up((size_t)2 * kPcBlocks * sizeof(float), 256) * 2;          // candidates
  b += round_up((size_t)chunks * rank * rank * sizeof(float), 256);       // Gram partials
  b += round_up((size_t)rank * rank * sizeof(float), 256);                // Gram
  return b;
}

// Factor noise*I + G (fp64, host), write the lower factor + log|P| to `small`, its inverse to `inv`.
static int small_factor(const std::vector<double>& G, int k, int cap, double noise, int64_t n, double* small,
                        std::vector<float>* inv) {
  std::vector<double> A((size_t)k * k), Lc((size_t)k * k, 0.0);
  for (int a = 0; a < k; ++a)
    for (int b = 0; b < k; ++b) A[a * k + b] = 0.5 * (G[a * k + b] + G[b * k + a]) + (a == b ? noise : 0.0);
  double logdet = 0.0;
  for (int j = 0; j < k; ++j) {
    double s = A[j * k + j];
    for (int c = 0; c < j; ++c) s -= Lc[j * k + c] * Lc[j * k + c];
    if (!(s > 0.0)) return fail(EGP_ERR_BREAKDOWN, "noise*I + L^T L is not positive definite at column %d", j);
    const double dj = sqrt(s);
    Lc[j * k + j] = dj;
    logdet += 2.0 * log(dj);
    for (int i = j + 1; i < k; ++i) {
      double v = A[i * k + j];
      for (int c = 0; c < j; ++c) v -= Lc[i * k + c] * Lc[j * k + c];
      Lc[i * k + j] = v / dj;
    }
  }
  logdet += (double)(n - k) * log(noise);
  for (int i = 0; i < cap * cap + 1; ++i) small[i] = 0.0;
  for (int a = 0; a < k; ++a)
    for (int b = 0; b < k; ++b) small[a * k + b] = Lc[a * k + b];
  small[(size_t)cap * cap] = logdet;
  // inverse: solve (Lc Lc^T) Xcol = e_col
  inv->assign((size_t)k * k, 0.f);
  std::vector<double> y(k), x(k);
  for (int col = 0; col < k; ++col) {
    for (int i = 0; i < k; ++i) {
      double v = (i == col) ? 1.0 : 0.0;
      for (int c = 0; c < i; ++c) v -= Lc[i * k + c] * y[c];
      y[i] = v / Lc[i * k + i];
    }
    for (int i = k - 1; i >= 0; --i) {
      double v = y[i];
      for (int c = i + 1; c < k; ++c) v -= Lc[c * k + i] * x[c];
      x[i] = v / Lc[i * k + i];
    }
    for (int i = 0; i < k; ++i) (*inv)[(size_t)i * k + col] = (float)x[i];
  }
  return EGP_OK;
}

int pivchol_core(const float* X, int64_t n, const egp_hyper_t* h, float tol_abs, egp_precond_t* P, void* ws,
                 hipStream_t stream) {
  const int cap = P->rank;
  Prepared prep;
  int rc = prepare_points(X, n, h, ws, &prep, stream);
  if (rc != EGP_OK) return rc;
  int64_t chunk;
  const int chunks = chunks_for(n, &chunk);
  char* w = static_cast<char*>(ws) + prepared_bytes(n, h->d);
  float* diag = reinterpret_cast<float*>(w);
  w += round_up((size_t)n * sizeof(float), 256);
  PcState st;
  st.pivots = reinterpret_cast<int*>(w);
  w += round_up((size_t)cap * sizeof(int), 256);
  st.rank_out = reinterpret_cast<int*>(w);
  st.stop = st.rank_out + 1;
  w += 256;
  st.cand_v = reinterpret_cast<float*>(w);
  w += round_up((size_t)2 * kPcBlocks * sizeof(float), 256);
  st.cand_i = reinterpret_cast<int*>(w);
  w += round_up((size_t)2 * kPcBlocks * sizeof(float), 256);
  float* Gp = reinterpret_cast<float*>(w);
  w += round_up((size_t)chunks * cap * cap * sizeof(float), 256);
  float* Gd = reinterpret_cast<float*>(w);

  int64_t nb = (n + 255) / 256;
  const int blocks = (int)(nb > kPcBlocks ? kPcBlocks : nb);
  {
    ProfScope prof(kProfPivChol, stream);
    hipLaunchKernelGGL(pc_init, dim3((unsigned)nb), dim3(256), 0, stream, diag, n, h->outputscale, st, cap);
    for (int m = 0; m < cap; ++m)
      hipLaunchKernelGGL(pc_step, dim3(blocks), dim3(256), 0, stream, prep.Xp, prep.ks, prep.d, h->kernel_type,
                         h->outputscale, n, P->L, diag, m, tol_abs, st);
  }
  EGP_HIP(hipGetLastError());
  int rank = 0;
  EGP_HIP(hipMemcpyAsync(&rank, st.rank_out, sizeof(int), hipMemcpyDeviceToHost, stream));
  EGP_HIP(hipStreamSynchronize(stream));
  if (rank < 0 || rank > cap) return fail(EGP_ERR_DEVICE, "pivoted Cholesky returned rank %d", rank);
  P->rank = rank;
  if (rank == 0) {
    for (int i = 0; i < cap * cap + 1; ++i) P->small[i] = 0.0;
    P->small[(size_t)cap * cap] = (double)n * log((double)h->noise);
    return EGP_OK;
  }
  EGP_HIP(hipMemcpyAsync(P->pivots, st.pivots, sizeof(int) * rank, hipMemcpyDeviceToHost, stream));
  // Gram matrix of the factor's columns
  dim3 grid(chunks, (rank + 63) / 64, (rank + 63) / 64);
  hipLaunchKernelGGL(nt_gemm_partial<false>, grid, dim3(256), 0, stream, P->L, rank, P->L, rank, n, chunk, Gp);
  hipLaunchKernelGGL(sum_chunks, dim3((rank * rank + 255) / 256), dim3(256), 0, stream, Gp, chunks, rank * rank,
                     Gd);
  EGP_HIP(hipGetLastError());
  std::vector<float> Gh((size_t)rank * rank);
  EGP_HIP(hipMemcpyAsync(Gh.data(), Gd, sizeof(float) * rank * rank, hipMemcpyDeviceToHost, stream));
  EGP_HIP(hipStreamSynchronize(stream));
  std::vector<double> G(Gh.begin(), Gh.end());
  std::vector<float> inv;
  rc = small_factor(G, rank, cap, (double)h->noise, n, P->small, &inv);
  if (rc != EGP_OK) return rc;
  EGP_HIP(hipMemcpyAsync(P->small_dev, inv.data(), sizeof(float) * rank * rank, hipMemcpyHostToDevice, stream));
  EGP_HIP(hipStreamSynchronize(stream));
  return EGP_OK;
}

}  // namespace egp
