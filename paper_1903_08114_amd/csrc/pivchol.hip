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

// ---- C[a][b] = sum_i A[a][i] * B[b][i] over a chunk of i (both operands contiguous in i) ----
// Block tile 128 (a) x 32 (b), 256 threads each 8 x 2 outputs, 32 points per LDS step. Partial results go to
// Cp[chunk][ra][rb]; reduce_chunks sums chunks in a fixed order.
__global__ __launch_bounds__(256) void gram_partial(const float* __restrict__ A, int ra, int64_t lda,
                                                    const float* __restrict__ B, int rb, int64_t ldb, int64_t n,
                                                    int64_t chunk, float* __restrict__ Cp, int vecA, int vecB) {
  __shared__ float As[32][128 + 4];
  __shared__ float Bs[32][32 + 4];
  const int ta = blockIdx.y * 128, tb = blockIdx.z * 32;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int64_t i_begin = (int64_t)blockIdx.x * chunk;
  int64_t i_end = i_begin + chunk;
  if (i_end > n) i_end = n;
  float acc[8][2] = {};
  for (int64_t i0 = i_begin; i0 < i_end; i0 += 32) {
    // 128 rows x 32 points of A: 1024 float4, 4 per thread; row a = e / 8, points 4 (e % 8) .. +3
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int e = threadIdx.x + k * 256;
      const int a = e >> 3, i4 = (e & 7) * 4;
      float4 v = {0.f, 0.f, 0.f, 0.f};
      const int64_t i = i0 + i4;
      if (ta + a < ra) {
        const float* src = A + (int64_t)(ta + a) * lda + i;
        if (vecA && i + 3 < i_end) v = *reinterpret_cast<const float4*>(src);
        else {
          if (i + 0 < i_end) v.x = src[0];
          if (i + 1 < i_end) v.y = src[1];
          if (i + 2 < i_end) v.z = src[2];
          if (i + 3 < i_end) v.w = src[3];
        }
      }
      As[i4 + 0][a] = v.x; As[i4 + 1][a] = v.y; As[i4 + 2][a] = v.z; As[i4 + 3][a] = v.w;
    }
    {
      const int e = threadIdx.x;            // 32 rows x 32 points of B: 256 float4
      const int bb = e >> 3, i4 = (e & 7) * 4;
      float4 v = {0.f, 0.f, 0.f, 0.f};
      const int64_t i = i0 + i4;
      if (tb + bb < rb) {
        const float* src = B + (int64_t)(tb + bb) * ldb + i;
        if (vecB && i + 3 < i_end) v = *reinterpret_cast<const float4*>(src);
        else {
          if (i + 0 < i_end) v.x = src[0];
          if (i + 1 < i_end) v.y = src[1];
          if (i + 2 < i_end) v.z = src[2];
          if (i + 3 < i_end) v.w = src[3];
        }
      }
      Bs[i4 + 0][bb] = v.x; Bs[i4 + 1][bb] = v.y; Bs[i4 + 2][bb] = v.z; Bs[i4 + 3][bb] = v.w;
    }
    __syncthreads();
#pragma unroll 8
    for (int ii = 0; ii < 32; ++ii) {
      const float4 a0 = *reinterpret_cast<const float4*>(&As[ii][ty * 8]);
      const float4 a1 = *reinterpret_cast<const float4*>(&As[ii][ty * 8 + 4]);
      const float2 bv = *reinterpret_cast<const float2*>(&Bs[ii][tx * 2]);
      const float av[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        acc[u][0] = __builtin_fmaf(av[u], bv.x, acc[u][0]);
        acc[u][1] = __builtin_fmaf(av[u], bv.y, acc[u][1]);
      }
    }
    __syncthreads();
  }
  float* dst = Cp + (int64_t)blockIdx.x * ra * rb;
#pragma unroll
  for (int u = 0; u < 8; ++u)
#pragma unroll
    for (int v = 0; v < 2; ++v) {
      const int a = ta + ty * 8 + u, b = tb + tx * 2 + v;
      if (a < ra && b < rb) dst[a * rb + b] = acc[u][v];
    }
}

__global__ __launch_bounds__(256) void reduce_chunks(const float* __restrict__ Cp, int chunks, int count,
                                                     float* __restrict__ C) {
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= count) return;
  double s = 0.0;
  for (int c = 0; c < chunks; ++c) s += (double)Cp[(int64_t)c * count + e];
  C[e] = (float)s;
}

// Y[m][c] = sum_m2 Minv[m][m2] * W[m2][c]   (k x k times k x t, one thread per output)
__global__ __launch_bounds__(256) void small_matmul(const float* __restrict__ Minv, const float* __restrict__ W,
                                                    int k, int t, float* __restrict__ Y) {
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= k * t) return;
  const int m = e / t, c = e % t;
  float acc = 0.f;
  for (int m2 = 0; m2 < k; ++m2) acc = __builtin_fmaf(Minv[m * k + m2], W[m2 * t + c], acc);
  Y[e] = acc;
}

// Column-major Woodbury finish: Z[c][i] = (R[c][i] - sum_m L[m][i] Y[m][c]) / noise for i < n; optional
// per-block partial sums of R[c][i] Z[c][i] into rz_part[c][blockIdx]. One thread per point.
template <int TT>
__global__ __launch_bounds__(256) void woodbury_finish_cm(const float* __restrict__ L, int k, int64_t n, int64_t ldl,
                                                          const float* __restrict__ Y, const float* __restrict__ R,
                                                          int64_t ld, int t, float inv_noise, float* __restrict__ Z,
                                                          float* __restrict__ rz_part, int part_ld) {
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
    for (int m = 0; m < k; ++m) {
      const float l = L[(int64_t)m * ldl + i];
      const float* y = Ys + m * t;
#pragma unroll
      for (int c = 0; c < TT; ++c)
        if (c < t) acc[c] = __builtin_fmaf(l, y[c], acc[c]);
    }
#pragma unroll
    for (int c = 0; c < TT; ++c)
      if (c < t) {
        const float r = R[(int64_t)c * ld + i];
        const float z = (r - acc[c]) * inv_noise;
        Z[(int64_t)c * ld + i] = z;
        dot[c] = __builtin_fmaf(r, z, dot[c]);
      }
  }
  if (rz_part != nullptr) {
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
      rz_part[(int64_t)threadIdx.x * part_ld + blockIdx.x] =
          (red[threadIdx.x] + red[t + threadIdx.x]) + (red[2 * t + threadIdx.x] + red[3 * t + threadIdx.x]);
  }
}

// row-major n x t  <->  column-major [t][ld] (entries beyond n are written as zero on the way in)
__global__ __launch_bounds__(256) void to_colmajor(const float* __restrict__ src, int64_t n, int t, int64_t ld,
                                                   float* __restrict__ dst) {
  for (int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x; g < ld * t; g += (int64_t)gridDim.x * 256) {
    const int c = (int)(g / ld);
    const int64_t i = g % ld;
    dst[g] = i < n ? src[i * t + c] : 0.f;
  }
}

__global__ __launch_bounds__(256) void to_rowmajor(const float* __restrict__ src, int64_t n, int t, int64_t ld,
                                                   float* __restrict__ dst) {
  for (int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x; g < n * t; g += (int64_t)gridDim.x * 256) {
    const int64_t i = g / t;
    const int c = (int)(g % t);
    dst[g] = src[(int64_t)c * ld + i];
  }
}

int chunks_for(int64_t n, int64_t* chunk_out) {
  int64_t chunk = 2048;
  while ((n + chunk - 1) / chunk > 512) chunk *= 2;
  *chunk_out = chunk;
  return (int)((n + chunk - 1) / chunk);
}

}  // namespace

void launch_to_colmajor(const float* src, int64_t n, int t, int64_t ld, float* dst, hipStream_t stream) {
  hipLaunchKernelGGL(to_colmajor, dim3(1024), dim3(256), 0, stream, src, n, t, ld, dst);
}
void launch_to_rowmajor(const float* src, int64_t n, int t, int64_t ld, float* dst, hipStream_t stream) {
  hipLaunchKernelGGL(to_rowmajor, dim3(1024), dim3(256), 0, stream, src, n, t, ld, dst);
}

int precond_apply_blocks(int64_t n) {
  int64_t b = (n + 255) / 256;
  return (int)(b > 1024 ? 1024 : b);
}

size_t precond_apply_ws(int64_t n, int t, int rank) {
  int64_t chunk;
  const int chunks = chunks_for(n, &chunk);
  const int64_t ld = padded_points(n);
  return round_up((size_t)chunks * rank * t * sizeof(float), 256) + 2 * round_up((size_t)rank * t * sizeof(float), 256) +
         2 * round_up((size_t)ld * t * sizeof(float), 256);   // the last two: transposes for the row-major entry point
}

// Column-major core: R, Z are [t][ld]; rz_part (optional) is [t][part_ld] with precond_apply_blocks(n) entries
// per column.
int precond_apply_cm(const float* L, int rank, const float* Minv_dev, int64_t n, float noise, const float* R,
                     int64_t ld, int t, float* Z, float* rz_part, int part_ld, void* ws, hipStream_t stream) {
  if (t > 33) return fail(EGP_ERR_ARG, "preconditioner application supports t <= 33 (got %d)", t);
  ProfScope prof(kProfPrecond, stream);
  int64_t chunk;
  const int chunks = chunks_for(n, &chunk);
  char* w = static_cast<char*>(ws);
  float* Wp = reinterpret_cast<float*>(w);
  w += round_up((size_t)chunks * rank * t * sizeof(float), 256);
  float* Wd = reinterpret_cast<float*>(w);
  w += round_up((size_t)rank * t * sizeof(float), 256);
  float* Y = reinterpret_cast<float*>(w);
  dim3 grid(chunks, (rank + 127) / 128, (t + 31) / 32);
  hipLaunchKernelGGL(gram_partial, grid, dim3(256), 0, stream, L, rank, n, R, t, ld, n, chunk, Wp,
                     (int)((n & 3) == 0 && (reinterpret_cast<uintptr_t>(L) & 15) == 0), (int)((ld & 3) == 0));
  hipLaunchKernelGGL(reduce_chunks, dim3((rank * t + 255) / 256), dim3(256), 0, stream, Wp, chunks, rank * t, Wd);
  hipLaunchKernelGGL(small_matmul, dim3((rank * t + 255) / 256), dim3(256), 0, stream, Minv_dev, Wd, rank, t, Y);
  const int blocks = precond_apply_blocks(n);
  const size_t shb = ((size_t)rank * t + 4 * t) * sizeof(float);
  const float inv_noise = 1.0f / noise;
  if (t <= 16)
    hipLaunchKernelGGL(woodbury_finish_cm<16>, dim3(blocks), dim3(256), shb, stream, L, rank, n, n, Y, R, ld, t,
                       inv_noise, Z, rz_part, part_ld);
  else if (t <= 17)
    hipLaunchKernelGGL(woodbury_finish_cm<17>, dim3(blocks), dim3(256), shb, stream, L, rank, n, n, Y, R, ld, t,
                       inv_noise, Z, rz_part, part_ld);
  else
    hipLaunchKernelGGL(woodbury_finish_cm<33>, dim3(blocks), dim3(256), shb, stream, L, rank, n, n, Y, R, ld, t,
                       inv_noise, Z, rz_part, part_ld);
  EGP_HIP(hipGetLastError());
  return EGP_OK;
}

// Row-major entry (egp_precond_apply, egp_mll): transpose in, apply, transpose out.
int precond_apply_core(const float* L, int rank, const float* Minv_dev, int64_t n, float noise, const float* R,
                       int t, float* Z, float* rz_partial, void* ws, hipStream_t stream) {
  (void)rz_partial;
  int64_t chunk;
  const int chunks = chunks_for(n, &chunk);
  const int64_t ld = padded_points(n);
  char* w = static_cast<char*>(ws);
  w += round_up((size_t)chunks * rank * t * sizeof(float), 256) + 2 * round_up((size_t)rank * t * sizeof(float), 256);
  float* Rc = reinterpret_cast<float*>(w);
  float* Zc = reinterpret_cast<float*>(w + round_up((size_t)ld * t * sizeof(float), 256));
  launch_to_colmajor(R, n, t, ld, Rc, stream);
  const int rc = precond_apply_cm(L, rank, Minv_dev, n, noise, Rc, ld, t, Zc, nullptr, 0, ws, stream);
  if (rc != EGP_OK) return rc;
  launch_to_rowmajor(Zc, n, t, ld, Z, stream);
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
  dim3 grid(chunks, (rank + 127) / 128, (rank + 31) / 32);
  const int vec = (int)((n & 3) == 0);
  hipLaunchKernelGGL(gram_partial, grid, dim3(256), 0, stream, P->L, rank, n, P->L, rank, n, n, chunk, Gp, vec, vec);
  hipLaunchKernelGGL(reduce_chunks, dim3((rank * rank + 255) / 256), dim3(256), 0, stream, Gp, chunks, rank * rank,
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
