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

#include <atomic>
#include <thread>
#include <vector>

#include "egp_internal.h"

namespace egp {

namespace {

typedef float f4 __attribute__((ext_vector_type(4)));

constexpr int kPcBlocks = 1024;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ float transform_rt(int kind, float acc) {
  if (kind == EGP_RBF) return __builtin_amdgcn_exp2f(-acc);
  const float a = __builtin_amdgcn_sqrtf(__builtin_fabsf(acc));
  const float e = __builtin_amdgcn_exp2f(-a);
  if (kind == EGP_MATERN32) return __builtin_fmaf(a, kLn2, 1.0f) * e;
  if (kind == EGP_MATERN12) return e;
  return __builtin_fmaf(__builtin_fmaf(a, kLn2 * kLn2 / 3.0f, kLn2), a, 1.0f) * e;
}

__device__ __forceinline__ f4 fma4(f4 a, f4 b, f4 c) {
  return (f4){__builtin_fmaf(a.x, b.x, c.x), __builtin_fmaf(a.y, b.y, c.y), __builtin_fmaf(a.z, b.z, c.z),
              __builtin_fmaf(a.w, b.w, c.w)};
}
__device__ __forceinline__ f4 fma4(f4 a, float b, f4 c) { return fma4(a, (f4){b, b, b, b}, c); }

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
template <bool VEC>
__global__ __launch_bounds__(256) void pc_step(const float* __restrict__ Xp, int ks, int d, int kind, float s,
                                               int64_t n, float* __restrict__ L, float* __restrict__ diag, int m,
                                               float tol_abs, PcState st) {
  __shared__ Cand sh[4];
  __shared__ float xpiv[EGP_D_WIDE_MAX + 1];
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

  const float* pbase = Xp + (piv >> 4) * ks * 64;
  for (int f = threadIdx.x; f < d; f += 256) xpiv[f] = pbase[xp_offset(ks, f, (int)(piv & 15))];
  for (int c = threadIdx.x; c < m; c += 256) lrow[c] = L[(int64_t)c * n + piv];
  __syncthreads();
  const float root = sqrtf(w.v);
  const float inv_root = 1.0f / root;

  Cand best = {-INFINITY, 0x7fffffff};
  if (VEC) {
    // Four consecutive points per thread (n a multiple of 4, L 16-byte aligned): every column of L is read with
    // 16-byte loads, eight columns in flight per thread. The step is a matrix-vector product with the n x m factor
    // (n (m + d + 3) floats of traffic), so what matters is how many bytes are in flight.
    for (int64_t i0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4; i0 < n; i0 += (int64_t)gridDim.x * 1024) {
      const f4 dg = *reinterpret_cast<const f4*>(diag + i0);
      const float* xb = Xp + (i0 >> 4) * ks * 64;
      const int pp = (int)(i0 & 15);
      f4 r2 = {0.f, 0.f, 0.f, 0.f};
      for (int f = 0; f < d; ++f) {
        const float xp = xpiv[f];
        const int o = xp_offset(ks, f, pp), st4 = xp_offset(ks, f, pp + 1) - o;      // stride between the tile's points
        const f4 df = {xp - xb[o], xp - xb[o + st4], xp - xb[o + 2 * st4], xp - xb[o + 3 * st4]};
        r2 = fma4(df, df, r2);
      }
      f4 acc = {s * transform_rt(kind, r2.x), s * transform_rt(kind, r2.y), s * transform_rt(kind, r2.z),
                s * transform_rt(kind, r2.w)};
      const float* Li = L + i0;
      f4 a0 = {0.f, 0.f, 0.f, 0.f}, a1 = a0, a2 = a0, a3 = a0;
      int c = 0;
      for (; c + 8 <= m; c += 8) {
        f4 l[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) l[u] = *reinterpret_cast<const f4*>(Li + (int64_t)(c + u) * n);
        a0 = fma4(l[0], lrow[c + 0], a0);      // (the same four interleaved sums, in the same order, as the scalar path)
        a1 = fma4(l[1], lrow[c + 1], a1);
        a2 = fma4(l[2], lrow[c + 2], a2);
        a3 = fma4(l[3], lrow[c + 3], a3);
        a0 = fma4(l[4], lrow[c + 4], a0);
        a1 = fma4(l[5], lrow[c + 5], a1);
        a2 = fma4(l[6], lrow[c + 6], a2);
        a3 = fma4(l[7], lrow[c + 7], a3);
      }
      if (c + 4 <= m) {
        a0 = fma4(*reinterpret_cast<const f4*>(Li + (int64_t)(c + 0) * n), lrow[c + 0], a0);
        a1 = fma4(*reinterpret_cast<const f4*>(Li + (int64_t)(c + 1) * n), lrow[c + 1], a1);
        a2 = fma4(*reinterpret_cast<const f4*>(Li + (int64_t)(c + 2) * n), lrow[c + 2], a2);
        a3 = fma4(*reinterpret_cast<const f4*>(Li + (int64_t)(c + 3) * n), lrow[c + 3], a3);
        c += 4;
      }
      for (; c < m; ++c) a0 = fma4(*reinterpret_cast<const f4*>(Li + (int64_t)c * n), lrow[c], a0);
      acc -= (a0 + a1) + (a2 + a3);
      const float dgv[4] = {dg.x, dg.y, dg.z, dg.w}, accv[4] = {acc.x, acc.y, acc.z, acc.w};
      float colv[4], newv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (i0 + u == piv) {
          colv[u] = root;
          newv[u] = -INFINITY;
        } else if (dgv[u] == -INFINITY) {      // chosen earlier
          colv[u] = 0.f;
          newv[u] = -INFINITY;
        } else {
          colv[u] = accv[u] * inv_root;
          newv[u] = dgv[u] - colv[u] * colv[u];
        }
        best = better(best, (Cand){newv[u], (int)(i0 + u)});
      }
      *reinterpret_cast<f4*>(L + (int64_t)m * n + i0) = (f4){colv[0], colv[1], colv[2], colv[3]};
      *reinterpret_cast<f4*>(diag + i0) = (f4){newv[0], newv[1], newv[2], newv[3]};
    }
  } else
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
      const float* xb = Xp + (i >> 4) * ks * 64;
      const int pp = (int)(i & 15);
      float r2 = 0.f;
      for (int f = 0; f < d; ++f) {
        const float df = xpiv[f] - xb[xp_offset(ks, f, pp)];
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

// ---- C[a][b] = sum_i A[a][i] * B[b][i] (both operands contiguous in i) on the fp64 MFMA ----
// Why fp64: P^{-1} r = (r - L M L^T r) / noise subtracts two vectors that agree to a relative noise / lambda in the
// directions L captures (lambda up to ~n s, i.e. 10^-6 at n = 2^20); with L^T r, L^T L or the final combination
// accumulated in fp32 the difference is rounding noise, r^T P^{-1} r can turn negative and CG breaks down. The
// inputs are fp32 values; their products and sums are carried in fp64 (v_mfma_f64_16x16x4_f64, 78.6 TFLOP/s: the
// kernel stays HBM-bound).
// grid = (blocks, ceil(ra/64), ceil(rb/32)), 4 waves per block; a wave owns 4 x 2 output tiles of 16 x 16
// and walks groups of 32 points: lane (q,p) loads points 32 g + 8 q .. + 7 of row p of each operand tile
// (two 16-byte loads) and feeds component s to MFMA step s. Both operands use the same point-to-step map, so
// the pairing is consistent; the order of a sum is free. Every wave writes its own partial result
// Cp[ra][rb][4 * block + wave] (the chunk index contiguous, so that reduce_chunks reads coalesced); reduce_chunks
// sums them in a fixed order.
typedef double d4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f4 load4_guarded(const float* __restrict__ row, int64_t i, int64_t n, int vec) {
  f4 v = {0.f, 0.f, 0.f, 0.f};
  if (vec && i + 3 < n) return *reinterpret_cast<const f4*>(row + i);
  if (i + 0 < n) v.x = row[i + 0];
  if (i + 1 < n) v.y = row[i + 1];
  if (i + 2 < n) v.z = row[i + 2];
  if (i + 3 < n) v.w = row[i + 3];
  return v;
}

constexpr int kGramTa = 4;      // 16-row tiles of A per wave

// FAST: both operands allow 16-byte loads (leading dimensions multiples of 4, 16-byte aligned bases). Then every group
// of 32 points that lies wholly below n is loaded without bounds checks, and rows of the last, partial tile that lie
// beyond the matrix read a clamped (valid) row instead of being zeroed: their products only reach output rows /
// columns that are never written. Only the one group that straddles n takes the guarded loads.
// NTB: 16-row tiles of B per wave. One for up to 17 rows of B (the preconditioner's L^T R: half the accumulators, four
// waves per SIMD), two otherwise (the Gram matrix of the factor, where A is re-read once per block of B rows).
template <bool FAST, int NTB>
__global__ __launch_bounds__(256, NTB == 1 ? 3 : 2) void gram_mfma(const float* __restrict__ A, int ra, int64_t lda,
                                                 const float* __restrict__ B, int rb, int64_t ldb, int64_t n,
                                                 double* __restrict__ Cp, int vecA, int vecB) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int q = lane >> 4, p = lane & 15;
  const int a_base = blockIdx.y * (16 * kGramTa), b_base = blockIdx.z * (16 * NTB);
  int nta = (ra - a_base + 15) / 16;
  if (nta > kGramTa) nta = kGramTa;
  // A lone last row of B (17 or 33 right-hand sides, or a single one) gets no matrix tile of its own, of which
  // fifteen sixteenths would be padding (an fp64 MFMA step takes 64 cycles; with t = 17 half of the matrix work of the
  // preconditioner's L^T R was that padding): the last block of B rows takes it along, its sums as fp64 FMAs on the
  // vector unit (the grid's z extent is computed accordingly, see launch_gram).
  const bool lone = FAST && rb % 16 == 1 && blockIdx.z == gridDim.z - 1;
  const int xrow = lone ? rb - 1 : -1;
  int ntb = ((lone ? rb - 1 : rb) - b_base + 15) / 16;
  if (ntb > NTB) ntb = NTB;
  d4 acc[kGramTa][NTB];
  double accx[kGramTa];
#pragma unroll
  for (int ta = 0; ta < kGramTa; ++ta) {
    accx[ta] = 0.0;
#pragma unroll
    for (int tb = 0; tb < NTB; ++tb) acc[ta][tb] = (d4){0.0, 0.0, 0.0, 0.0};
  }
  // A wave walks a contiguous run of groups of 32 points: lane (q, p) loads points 32 g + 8 q .. + 7 of row p of each
  // operand tile (two 16-byte loads: the four lanes of a row cover one 128-byte line) and feeds its eight values to
  // eight MFMA steps. Both operands use the same point-to-step map, so the pairing is consistent.
  const int64_t groups = (n + 31) / 32;
  const int64_t gper = (groups + (int64_t)gridDim.x * 4 - 1) / ((int64_t)gridDim.x * 4);
  int64_t g = ((int64_t)blockIdx.x * 4 + wave) * gper;
  int64_t g_end = g + gper;
  if (g_end > groups) g_end = groups;

  struct Ops { f4 a[kGramTa][2], b[NTB][2], x[2]; };
  // row pointers of this lane (clamped into the matrix in the fast path)
  const float* arow[kGramTa];
  const float* brow[NTB];
#pragma unroll
  for (int ta = 0; ta < kGramTa; ++ta) {
    int row = a_base + ta * 16 + p;
    if (FAST && row >= ra) row = ra - 1;
    arow[ta] = A + (int64_t)row * lda;
  }
#pragma unroll
  for (int tb = 0; tb < NTB; ++tb) {
    int row = b_base + tb * 16 + p;
    if (FAST && row >= rb) row = rb - 1;
    brow[tb] = B + (int64_t)row * ldb;
  }
  const float* xptr = B + (int64_t)(xrow >= 0 ? xrow : 0) * ldb;
  auto load_fast = [&](int64_t gg, Ops& o) {      // the whole group lies below n
    const int64_t i = gg * 32 + q * 8;
#pragma unroll
    for (int ta = 0; ta < kGramTa; ++ta)
      if (ta < nta) {
        o.a[ta][0] = *reinterpret_cast<const f4*>(arow[ta] + i);
        o.a[ta][1] = *reinterpret_cast<const f4*>(arow[ta] + i + 4);
      }
#pragma unroll
    for (int tb = 0; tb < NTB; ++tb)
      if (tb < ntb) {
        o.b[tb][0] = *reinterpret_cast<const f4*>(brow[tb] + i);
        o.b[tb][1] = *reinterpret_cast<const f4*>(brow[tb] + i + 4);
      }
    if (xrow >= 0) {      // the same eight points as this lane's A values (every lane p of a group reads them)
      o.x[0] = *reinterpret_cast<const f4*>(xptr + i);
      o.x[1] = *reinterpret_cast<const f4*>(xptr + i + 4);
    }
  };
  auto load_guarded = [&](int64_t gg, Ops& o) {
    const int64_t i = gg * 32 + q * 8;
#pragma unroll
    for (int ta = 0; ta < kGramTa; ++ta) {
      const bool on = ta < nta && (FAST || a_base + ta * 16 + p < ra);
      o.a[ta][0] = on ? load4_guarded(arow[ta], i, n, vecA) : (f4){0.f, 0.f, 0.f, 0.f};
      o.a[ta][1] = on ? load4_guarded(arow[ta], i + 4, n, vecA) : (f4){0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int tb = 0; tb < NTB; ++tb) {
      const bool on = tb < ntb && (FAST || b_base + tb * 16 + p < rb);
      o.b[tb][0] = on ? load4_guarded(brow[tb], i, n, vecB) : (f4){0.f, 0.f, 0.f, 0.f};
      o.b[tb][1] = on ? load4_guarded(brow[tb], i + 4, n, vecB) : (f4){0.f, 0.f, 0.f, 0.f};
    }
    if (xrow >= 0) {
      o.x[0] = load4_guarded(xptr, i, n, vecB);
      o.x[1] = load4_guarded(xptr, i + 4, n, vecB);
    }
  };
  auto compute = [&](const Ops& o) {
    if (xrow >= 0) {
#pragma unroll
      for (int ta = 0; ta < kGramTa; ++ta)
        if (ta < nta) {
#pragma unroll
          for (int hlf = 0; hlf < 2; ++hlf) {
            accx[ta] = fma((double)o.a[ta][hlf].x, (double)o.x[hlf].x, accx[ta]);
            accx[ta] = fma((double)o.a[ta][hlf].y, (double)o.x[hlf].y, accx[ta]);
            accx[ta] = fma((double)o.a[ta][hlf].z, (double)o.x[hlf].z, accx[ta]);
            accx[ta] = fma((double)o.a[ta][hlf].w, (double)o.x[hlf].w, accx[ta]);
          }
        }
    }
#pragma unroll
    for (int ta = 0; ta < kGramTa; ++ta) {
      if (ta < nta) {
#pragma unroll
        for (int tb = 0; tb < NTB; ++tb) {
          if (tb < ntb) {
#pragma unroll
            for (int hlf = 0; hlf < 2; ++hlf) {
              const f4 a4 = o.a[ta][hlf], b4 = o.b[tb][hlf];
              acc[ta][tb] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)a4.x, (double)b4.x, acc[ta][tb], 0, 0, 0);
              acc[ta][tb] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)a4.y, (double)b4.y, acc[ta][tb], 0, 0, 0);
              acc[ta][tb] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)a4.z, (double)b4.z, acc[ta][tb], 0, 0, 0);
              acc[ta][tb] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)a4.w, (double)b4.w, acc[ta][tb], 0, 0, 0);
            }
          }
        }
      }
    }
  };

  if constexpr (FAST) {
    // Groups wholly below n, then the one that straddles it (at most one, in the last wave). No software prefetch: the
    // kernel is bound by its fp64 MFMA steps, and three to four waves per SIMD cover each other's load latency; a
    // second operand set in registers would cost that occupancy.
    const int64_t full = n / 32;
    const int64_t f_end = g_end < full ? g_end : full;
    Ops o0;
    for (; g < f_end; ++g) {
      load_fast(g, o0);
      compute(o0);
    }
    if (g < g_end) {
      load_guarded(g, o0);
      compute(o0);
    }
  } else {
    Ops o0;
    for (; g < g_end; ++g) {
      load_guarded(g, o0);
      compute(o0);
    }
  }

  // fp64 accumulator layout (differs from the fp32 one): register r of lane (q,p) is C[16 ta + 4 r + q][16 tb + p]
  const int64_t chunks = (int64_t)gridDim.x * 4, chunk_id = (int64_t)blockIdx.x * 4 + wave;
#pragma unroll
  for (int ta = 0; ta < kGramTa; ++ta)
#pragma unroll
    for (int tb = 0; tb < NTB; ++tb) {
      const double vals[4] = {acc[ta][tb].x, acc[ta][tb].y, acc[ta][tb].z, acc[ta][tb].w};
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int a = a_base + ta * 16 + r * 4 + q, bcol = b_base + tb * 16 + p;
        if (ta < nta && tb < ntb && a < ra && bcol < rb) Cp[(int64_t)(a * rb + bcol) * chunks + chunk_id] = vals[r];
      }
    }
  if (xrow >= 0) {      // the lone row: lane (q, p) holds the part of C[16 ta + p][xrow] over its eight points per group
#pragma unroll
    for (int ta = 0; ta < kGramTa; ++ta) {
      double v = accx[ta];
      v += __shfl_xor(v, 16);
      v += __shfl_xor(v, 32);
      const int a = a_base + ta * 16 + p;
      if (q == 0 && ta < nta && a < ra) Cp[(int64_t)(a * rb + xrow) * chunks + chunk_id] = v;
    }
  }
}

// Launch over `chunks` partial results (a multiple of 4: one per wave): the fast instantiation when both operands allow
// 16-byte loads; one tile of B rows per wave up to 17 rows, two beyond. In the fast path a lone last row of B rides
// with the last block of B rows, so it adds no block of its own.
void launch_gram(int chunks, hipStream_t stream, const float* A, int ra, int64_t lda, const float* B, int rb,
                 int64_t ldb, int64_t n, double* Cp) {
  const int va = (int)((lda & 3) == 0 && (reinterpret_cast<uintptr_t>(A) & 15) == 0);
  const int vb = (int)((ldb & 3) == 0 && (reinterpret_cast<uintptr_t>(B) & 15) == 0);
  const bool fast = va && vb;
  const int ntb = rb <= 17 ? 1 : 2;
  const int brows = (fast && rb % 16 == 1) ? rb - 1 : rb;
  int gz = (brows + 16 * ntb - 1) / (16 * ntb);
  if (gz < 1) gz = 1;
  const dim3 grid(chunks / 4, (ra + 16 * kGramTa - 1) / (16 * kGramTa), gz);
  if (fast && ntb == 1)
    hipLaunchKernelGGL((gram_mfma<true, 1>), grid, dim3(256), 0, stream, A, ra, lda, B, rb, ldb, n, Cp, va, vb);
  else if (fast)
    hipLaunchKernelGGL((gram_mfma<true, 2>), grid, dim3(256), 0, stream, A, ra, lda, B, rb, ldb, n, Cp, va, vb);
  else if (ntb == 1)
    hipLaunchKernelGGL((gram_mfma<false, 1>), grid, dim3(256), 0, stream, A, ra, lda, B, rb, ldb, n, Cp, va, vb);
  else
    hipLaunchKernelGGL((gram_mfma<false, 2>), grid, dim3(256), 0, stream, A, ra, lda, B, rb, ldb, n, Cp, va, vb);
}

// C[e] = sum over chunks of Cp[e][chunk], fp64, fixed order: 64 lanes stride the chunks, then a shuffle tree.
// Block = 4 outputs x 64 lanes.
__global__ __launch_bounds__(256) void reduce_chunks(const double* __restrict__ Cp, int chunks, int count,
                                                     double* __restrict__ C) {
  const int e = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  double s = 0.0;
  if (e < count)
    for (int c = lane; c < chunks; c += 64) s += Cp[(int64_t)e * chunks + c];
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off);
  if (e < count && lane == 0) C[e] = s;
}

// Y[m][c] = sum_m2 Minv[m][m2] * W[m2][c] for c < t, zero for t <= c < ldy (fp64). One wave per output: the
// lanes stride m2, then a shuffle tree (fixed order).
__global__ __launch_bounds__(256) void small_matmul(const double* __restrict__ Minv, const double* __restrict__ W,
                                                    int k, int t, int ldy, double* __restrict__ Y) {
  const int e = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (e >= k * ldy) return;
  const int m = e / ldy, c = e % ldy;
  double acc = 0.0;
  if (c < t) {
    if (Minv == nullptr) {
      acc = lane == 0 ? W[m * t + c] : 0.0;      // identity: plain projection coefficients
    } else {
      for (int m2 = lane; m2 < k; m2 += 64) acc = fma(Minv[m * k + m2], W[m2 * t + c], acc);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off);
  }
  if (lane == 0) Y[e] = acc;
}

// Column-major Woodbury finish: Z[c][i] = (R[c][i] - sum_m L[m][i] Y[m][c]) / noise for i < n, the sum and the
// difference in fp64 (see gram_mfma), the result rounded to fp32; optional per-block partial sums of
// R[c][i] Z[c][i] into rz_part[c][blockIdx]. One thread per point; Y (k x TT, zero-padded columns) is indexed
// uniformly across the wave, so its entries arrive as scalar operands.
template <int TT>
__global__ __launch_bounds__(256) void woodbury_finish_cm(const float* __restrict__ L, int k, int64_t n, int64_t ldl,
                                                          const double* __restrict__ Y, const float* __restrict__ R,
                                                          int64_t ld, int t, double inv_noise, float* __restrict__ Z,
                                                          float* __restrict__ rz_part, int part_ld) {
  __shared__ float red[4 * TT];
  float dot[TT];
#pragma unroll
  for (int c = 0; c < TT; ++c) dot[c] = 0.f;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    double acc[TT];
#pragma unroll
    for (int c = 0; c < TT; ++c) acc[c] = 0.0;
    const float* Li = L + i;
    int m = 0;
    // eight columns of L in flight per thread (the sums stay in the order m = 0, 1, 2, ...)
    for (; m + 8 <= k; m += 8) {
      float l[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) l[u] = Li[(int64_t)(m + u) * ldl];
      const double* y = Y + m * TT;
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const double lu = (double)l[u];
#pragma unroll
        for (int c = 0; c < TT; ++c) acc[c] = fma(lu, y[u * TT + c], acc[c]);
      }
    }
    for (; m < k; ++m) {
      const double l = (double)Li[(int64_t)m * ldl];
      const double* y = Y + m * TT;
#pragma unroll
      for (int c = 0; c < TT; ++c) acc[c] = fma(l, y[c], acc[c]);
    }
#pragma unroll
    for (int c = 0; c < TT; ++c)
      if (c < t) {
        const float r = R[(int64_t)c * ld + i];
        const float z = (float)(((double)r - acc[c]) * inv_noise);
        Z[(int64_t)c * ld + i] = z;
        dot[c] = __builtin_fmaf(r, z, dot[c]);
      }
  }
  if (rz_part != nullptr) {
#pragma unroll
    for (int c = 0; c < TT; ++c) {
      float v = dot[c];
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
      if ((threadIdx.x & 63) == 0) red[(threadIdx.x >> 6) * TT + c] = v;
    }
    __syncthreads();
    if ((int)threadIdx.x < t)
      rz_part[(int64_t)threadIdx.x * part_ld + blockIdx.x] =
          (red[threadIdx.x] + red[TT + threadIdx.x]) + (red[2 * TT + threadIdx.x] + red[3 * TT + threadIdx.x]);
  }
}

// The same with two consecutive points per thread (8-byte loads of L, R and stores of Z; n and ldl even): half the
// load instructions and half the scalar reads of Y per point. The sums of a point are the same, in the same order.
typedef float f2v __attribute__((ext_vector_type(2)));
template <int TT>
__global__ __launch_bounds__(256) void woodbury_finish_cm2(const float* __restrict__ L, int k, int64_t n, int64_t ldl,
                                                           const double* __restrict__ Y, const float* __restrict__ R,
                                                           int64_t ld, int t, double inv_noise, float* __restrict__ Z,
                                                           float* __restrict__ rz_part, int part_ld) {
  __shared__ float red[4 * TT];
  float dot[TT];
#pragma unroll
  for (int c = 0; c < TT; ++c) dot[c] = 0.f;
  for (int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 2; i < n; i += (int64_t)gridDim.x * 512) {
    double a0[TT], a1[TT];
#pragma unroll
    for (int c = 0; c < TT; ++c) a0[c] = a1[c] = 0.0;
    const float* Li = L + i;
    int m = 0;
    for (; m + 8 <= k; m += 8) {
      f2v l[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) l[u] = *reinterpret_cast<const f2v*>(Li + (int64_t)(m + u) * ldl);
      const double* y = Y + m * TT;
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const double l0 = (double)l[u].x, l1 = (double)l[u].y;
#pragma unroll
        for (int c = 0; c < TT; ++c) {
          a0[c] = fma(l0, y[u * TT + c], a0[c]);
          a1[c] = fma(l1, y[u * TT + c], a1[c]);
        }
      }
    }
    for (; m < k; ++m) {
      const f2v l = *reinterpret_cast<const f2v*>(Li + (int64_t)m * ldl);
      const double l0 = (double)l.x, l1 = (double)l.y;
      const double* y = Y + m * TT;
#pragma unroll
      for (int c = 0; c < TT; ++c) {
        a0[c] = fma(l0, y[c], a0[c]);
        a1[c] = fma(l1, y[c], a1[c]);
      }
    }
#pragma unroll
    for (int c = 0; c < TT; ++c)
      if (c < t) {
        const f2v r = *reinterpret_cast<const f2v*>(R + (int64_t)c * ld + i);
        f2v z;
        z.x = (float)(((double)r.x - a0[c]) * inv_noise);
        z.y = (float)(((double)r.y - a1[c]) * inv_noise);
        *reinterpret_cast<f2v*>(Z + (int64_t)c * ld + i) = z;
        dot[c] = __builtin_fmaf(r.x, z.x, dot[c]);
        dot[c] = __builtin_fmaf(r.y, z.y, dot[c]);
      }
  }
  if (rz_part != nullptr) {
#pragma unroll
    for (int c = 0; c < TT; ++c) {
      float v = dot[c];
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
      if ((threadIdx.x & 63) == 0) red[(threadIdx.x >> 6) * TT + c] = v;
    }
    __syncthreads();
    if ((int)threadIdx.x < t)
      rz_part[(int64_t)threadIdx.x * part_ld + blockIdx.x] =
          (red[threadIdx.x] + red[TT + threadIdx.x]) + (red[2 * TT + threadIdx.x] + red[3 * TT + threadIdx.x]);
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

// number of partial results the Gram kernel leaves: 4 waves per block, blocks sized to the point count
int gram_blocks(int64_t n) {
  int64_t b = (n / 32 + 4 * 8 - 1) / (4 * 8);     // at least 8 point groups (of 32) per wave
  if (b < 1) b = 1;
  if (b > 1024) b = 1024;
  return (int)b;
}
// Partial results of a Gram product with ra x rb outputs: the grid's y and z dimensions already spread the output
// tiles, so the point range is cut into only as many chunks as keep ~4096 waves in flight (a multiple of 4: one
// chunk per wave of a block). Keeps the partial buffer small at high rank.
int chunks_for(int64_t n, int ra, int rb) {
  const int tiles = ((ra + 16 * kGramTa - 1) / (16 * kGramTa)) * ((rb + 31) / 32);
  int c = 4096 / (tiles > 0 ? tiles : 1);
  c &= ~3;
  if (c < 4) c = 4;
  const int cap = 4 * gram_blocks(n);
  return c < cap ? c : cap;
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

// Upper bound, in doubles, of chunks_for(n, r, r) * r * r over every r <= cap (the factorisation may stop early)
static size_t gram_partial_doubles(int64_t n, int cap) {
  const size_t a = (size_t)4 * gram_blocks(n) * cap * cap;
  const size_t b = (size_t)4096 * 2048 + (size_t)4 * cap * cap;
  return a < b ? a : b;
}

// Upper bound, in doubles, of chunks_for(n, r, t) * r * t over every r <= rank (the Lanczos process applies
// projections of growing rank through the same workspace)
static size_t apply_partial_doubles(int64_t n, int rank, int t) {
  const size_t a = (size_t)4 * gram_blocks(n) * rank * t;
  const size_t b = (size_t)4096 * 64 * t + (size_t)4 * rank * t;
  return a < b ? a : b;
}

size_t precond_apply_ws(int64_t n, int t, int rank) {
  const int64_t ld = padded_points(n);
  return round_up(apply_partial_doubles(n, rank, t) * sizeof(double), 256) + 2 * round_up((size_t)rank * 33 * sizeof(double), 256) +
         2 * round_up((size_t)ld * t * sizeof(float), 256);   // the last two: transposes for the row-major entry point
}

// Column-major core: R, Z are [t][ld]; rz_part (optional) is [t][part_ld] with precond_apply_blocks(n) entries
// per column.
int precond_apply_cm(const float* L, int rank, const double* Minv_dev, int64_t n, float noise, const float* R,
                     int64_t ld, int t, float* Z, float* rz_part, int part_ld, void* ws, hipStream_t stream,
                     const double** coef_dev, int* coef_ld) {
  if (t > 33) return fail(EGP_ERR_ARG, "preconditioner application supports t <= 33 (got %d)", t);
  ProfScope prof(kProfPrecond, stream);
  const int chunks = chunks_for(n, rank, t);
  char* w = static_cast<char*>(ws);
  double* Wp = reinterpret_cast<double*>(w);
  w += round_up((size_t)chunks * rank * t * sizeof(double), 256);      // within the bound precond_apply_ws reserves
  double* Wd = reinterpret_cast<double*>(w);
  w += round_up((size_t)rank * 33 * sizeof(double), 256);
  double* Y = reinterpret_cast<double*>(w);
  launch_gram(chunks, stream, L, rank, n, R, t, ld, n, Wp);
  hipLaunchKernelGGL(reduce_chunks, dim3((rank * t + 3) / 4), dim3(256), 0, stream, Wp, chunks, rank * t, Wd);
  const int ldy = t <= 16 ? 16 : (t <= 17 ? 17 : 33);
  if (coef_dev) *coef_dev = Y;
  if (coef_ld) *coef_ld = ldy;
  hipLaunchKernelGGL(small_matmul, dim3((rank * ldy + 3) / 4), dim3(256), 0, stream, Minv_dev, Wd, rank, t, ldy,
                     Y);
  const int blocks = precond_apply_blocks(n);
  const size_t shb = 0;
  const double inv_noise = 1.0 / (double)noise;
  // two points per thread where the layout allows 8-byte accesses (the per-block partial sums of r.z keep their count:
  // the grid is the same, a block then covers 512 points per pass)
  const bool two = (n & 1) == 0 && (ld & 1) == 0 && (reinterpret_cast<uintptr_t>(L) & 7) == 0 &&
                   (reinterpret_cast<uintptr_t>(R) & 7) == 0 && (reinterpret_cast<uintptr_t>(Z) & 7) == 0;
  if (t <= 16 && two)
    hipLaunchKernelGGL(woodbury_finish_cm2<16>, dim3(blocks), dim3(256), shb, stream, L, rank, n, n, Y, R, ld, t,
                       inv_noise, Z, rz_part, part_ld);
  else if (t <= 17 && two)
    hipLaunchKernelGGL(woodbury_finish_cm2<17>, dim3(blocks), dim3(256), shb, stream, L, rank, n, n, Y, R, ld, t,
                       inv_noise, Z, rz_part, part_ld);
  else if (t <= 16)
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

size_t gram_cm_ws_bytes(int64_t n, int ra, int rb) {
  return round_up((size_t)chunks_for(n, ra, rb) * ra * rb * sizeof(double), 256);
}

int gram_cm(const float* A, int ra, int64_t lda, const float* B, int rb, int64_t ldb, int64_t n, double* G_dev,
            void* ws, hipStream_t stream) {
  const int chunks = chunks_for(n, ra, rb);
  double* Gp = static_cast<double*>(ws);
  launch_gram(chunks, stream, A, ra, lda, B, rb, ldb, n, Gp);
  hipLaunchKernelGGL(reduce_chunks, dim3((ra * rb + 3) / 4), dim3(256), 0, stream, Gp, chunks, ra * rb, G_dev);
  EGP_HIP(hipGetLastError());
  return EGP_OK;
}

namespace {
// one thread per point; the coefficients are indexed uniformly across the wave (scalar operands)
__global__ __launch_bounds__(256) void combine_kernel(const float* __restrict__ In, int k, int64_t ld_in,
                                                      const double* __restrict__ Cf, int t, int64_t n,
                                                      float* __restrict__ Out, int64_t ld_out) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < ld_out; i += (int64_t)gridDim.x * 256) {
    double acc[32];
#pragma unroll
    for (int c = 0; c < 32; ++c) acc[c] = 0.0;
    if (i < n)
      for (int m = 0; m < k; ++m) {
        const double v = (double)In[(int64_t)m * ld_in + i];
        const double* cf = Cf + m * t;
#pragma unroll
        for (int c = 0; c < 32; ++c)
          if (c < t) acc[c] = fma(v, cf[c], acc[c]);
      }
#pragma unroll
    for (int c = 0; c < 32; ++c)
      if (c < t) Out[(int64_t)c * ld_out + i] = (float)acc[c];
  }
}
}  // namespace

int combine_cm(const float* In, int k, int64_t ld_in, const double* Cf_dev, int t, int64_t n, float* Out,
               int64_t ld_out, hipStream_t stream) {
  if (t > 32) return fail(EGP_ERR_ARG, "combine_cm supports t <= 32 (got %d)", t);
  int64_t nb = (ld_out + 255) / 256;
  hipLaunchKernelGGL(combine_kernel, dim3((unsigned)(nb > 2048 ? 2048 : nb)), dim3(256), 0, stream, In, k, ld_in,
                     Cf_dev, t, n, Out, ld_out);
  EGP_HIP(hipGetLastError());
  return EGP_OK;
}

// Row-major entry (egp_precond_apply, egp_mll): transpose in, apply, transpose out.
int precond_apply_core(const float* L, int rank, const double* Minv_dev, int64_t n, float noise, const float* R,
                       int t, float* Z, float* rz_partial, void* ws, hipStream_t stream) {
  (void)rz_partial;
  const int chunks = chunks_for(n, rank, t);
  const int64_t ld = padded_points(n);
  char* w = static_cast<char*>(ws);
  w += round_up((size_t)chunks * rank * t * sizeof(double), 256) + 2 * round_up((size_t)rank * 33 * sizeof(double), 256);
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
  size_t b = prepared_bytes(n, d);
  b += round_up((size_t)n * sizeof(float), 256);                          // diag
  b += round_up((size_t)rank * sizeof(int), 256);                         // pivots
  b += 256;                                                               // rank, stop
  b += round_up((size_t)2 * kPcBlocks * sizeof(float), 256) * 2;          // candidates
  b += round_up(gram_partial_doubles(n, rank) * sizeof(double), 256);      // Gram partials
  b += round_up((size_t)rank * rank * sizeof(double), 256);               // Gram
  return b;
}

// Factor noise*I + G (fp64, host), write the lower factor + log|P| to `small`, its inverse to `inv`.
// O(k^3) work on a k x k matrix: at the ranks the paper uses (100) it is a fraction of a millisecond; at rank 512 to
// 1024 it would be 0.04 to 0.3 s on one core, so from k = 128 on the rows of each Cholesky column and the columns of the
// inverse are dealt to a few host threads (the arithmetic of every entry is the same as in the serial order).
namespace {
struct SpinBarrier {
  explicit SpinBarrier(int n) : n_(n) {}
  void wait() {
    const int gen = gen_.load(std::memory_order_acquire);
    if (count_.fetch_add(1, std::memory_order_acq_rel) + 1 == n_) {
      count_.store(0, std::memory_order_relaxed);
      gen_.store(gen + 1, std::memory_order_release);
    } else {
      while (gen_.load(std::memory_order_acquire) == gen) std::this_thread::yield();
    }
  }
  const int n_;
  std::atomic<int> count_{0}, gen_{0};
};
}  // namespace

static int small_factor(const std::vector<double>& G, int k, int cap, double noise, int64_t n, double* small,
                        std::vector<double>* inv) {
  std::vector<double> A((size_t)k * k), Lc((size_t)k * k, 0.0), Lt((size_t)k * k);
  for (int a = 0; a < k; ++a)
    for (int b = 0; b < k; ++b) A[a * k + b] = 0.5 * (G[a * k + b] + G[b * k + a]) + (a == b ? noise : 0.0);
  inv->assign((size_t)k * k, 0.0);
  int threads = 1;
  if (k >= 128) {
    const unsigned hw = std::thread::hardware_concurrency();
    threads = (int)(hw == 0 ? 4 : (hw > 16 ? 16 : hw));
    if (threads > k / 32) threads = k / 32;
    if (threads < 1) threads = 1;
  }
  std::atomic<int> bad_col{-1};
  SpinBarrier bar(threads);
  auto worker = [&](int tid) {
    // ---- Cholesky, column by column: the diagonal entry by thread 0, the rows below dealt round-robin ----
    for (int j = 0; j < k; ++j) {
      if (tid == 0) {
        double s = A[(size_t)j * k + j];
        for (int c = 0; c < j; ++c) s -= Lc[(size_t)j * k + c] * Lc[(size_t)j * k + c];
        if (!(s > 0.0)) bad_col.store(j);
        Lc[(size_t)j * k + j] = s > 0.0 ? sqrt(s) : 1.0;
      }
      if (threads > 1) bar.wait();
      if (bad_col.load() >= 0) return;
      const double dj = Lc[(size_t)j * k + j];
      const double* lj = &Lc[(size_t)j * k];
      for (int i = j + 1 + tid; i < k; i += threads) {
        double v = A[(size_t)i * k + j];
        const double* li = &Lc[(size_t)i * k];
        for (int c = 0; c < j; ++c) v -= li[c] * lj[c];
        Lc[(size_t)i * k + j] = v / dj;
      }
      if (threads > 1) bar.wait();
    }
    // ---- inverse: solve (Lc Lc^T) x = e_col, columns dealt round-robin ----
    for (int a = tid; a < k; a += threads)
      for (int b = 0; b < k; ++b) Lt[(size_t)b * k + a] = Lc[(size_t)a * k + b];      // contiguous rows for the back substitution
    if (threads > 1) bar.wait();
    std::vector<double> y(k), x(k);
    for (int col = tid; col < k; col += threads) {
      for (int i = 0; i < col; ++i) y[i] = 0.0;                                       // e_col starts with zeros
      for (int i = col; i < k; ++i) {
        double v = (i == col) ? 1.0 : 0.0;
        const double* li = &Lc[(size_t)i * k];
        for (int c = col; c < i; ++c) v -= li[c] * y[c];
        y[i] = v / li[i];
      }
      for (int i = k - 1; i >= 0; --i) {
        double v = y[i];
        const double* lt = &Lt[(size_t)i * k];
        for (int c = i + 1; c < k; ++c) v -= lt[c] * x[c];
        x[i] = v / lt[i];
      }
      for (int i = 0; i < k; ++i) (*inv)[(size_t)i * k + col] = x[i];
    }
  };
  if (threads > 1) {
    std::vector<std::thread> pool;
    for (int t = 1; t < threads; ++t) pool.emplace_back(worker, t);
    worker(0);
    for (std::thread& th : pool) th.join();
  } else {
    worker(0);
  }
  if (bad_col.load() >= 0)
    return fail(EGP_ERR_BREAKDOWN, "noise*I + L^T L is not positive definite at column %d", bad_col.load());
  double logdet = 0.0;
  for (int j = 0; j < k; ++j) logdet += 2.0 * log(Lc[(size_t)j * k + j]);
  logdet += (double)(n - k) * log(noise);
  for (int i = 0; i < cap * cap + 1; ++i) small[i] = 0.0;
  for (int a = 0; a < k; ++a)
    for (int b = 0; b < k; ++b) small[a * k + b] = Lc[a * k + b];
  small[(size_t)cap * cap] = logdet;
  return EGP_OK;
}

int pivchol_core(const float* X, int64_t n, const egp_hyper_t* h, float tol_abs, egp_precond_t* P, void* ws,
                 hipStream_t stream) {
  const int cap = P->rank;
  Prepared prep;
  int rc = prepare_points(X, n, h, ws, &prep, stream, EGP_KMM_FP32);      // kernel rows by direct differences: fp32 only
  if (rc != EGP_OK) return rc;
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
  double* Gp = reinterpret_cast<double*>(w);
  w += round_up(gram_partial_doubles(n, cap) * sizeof(double), 256);
  double* Gd = reinterpret_cast<double*>(w);

  int64_t nb = (n + 255) / 256;
  const int blocks = (int)(nb > kPcBlocks ? kPcBlocks : nb);
  {
    ProfScope prof(kProfPivChol, stream);
    hipLaunchKernelGGL(pc_init, dim3((unsigned)nb), dim3(256), 0, stream, diag, n, h->outputscale, st, cap);
    // 16-byte accesses to L and the residual diagonal where the layout allows them (four points per thread)
    const bool vec = (n & 3) == 0 && (reinterpret_cast<uintptr_t>(P->L) & 15) == 0 && n >= 4096;
    const int vblocks = (int)((n / 4 + 255) / 256 > kPcBlocks ? kPcBlocks : (n / 4 + 255) / 256);
    for (int m = 0; m < cap; ++m) {
      if (vec)
        hipLaunchKernelGGL(pc_step<true>, dim3(vblocks), dim3(256), 0, stream, prep.Xp, prep.ks, prep.d,
                           h->kernel_type, h->outputscale, n, P->L, diag, m, tol_abs, st);
      else
        hipLaunchKernelGGL(pc_step<false>, dim3(blocks), dim3(256), 0, stream, prep.Xp, prep.ks, prep.d,
                           h->kernel_type, h->outputscale, n, P->L, diag, m, tol_abs, st);
    }
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
  const int chunks = chunks_for(n, rank, rank);
  launch_gram(chunks, stream, P->L, rank, n, P->L, rank, n, n, Gp);
  hipLaunchKernelGGL(reduce_chunks, dim3((rank * rank + 3) / 4), dim3(256), 0, stream, Gp, chunks, rank * rank, Gd);
  EGP_HIP(hipGetLastError());
  std::vector<double> G((size_t)rank * rank);
  EGP_HIP(hipMemcpyAsync(G.data(), Gd, sizeof(double) * rank * rank, hipMemcpyDeviceToHost, stream));
  EGP_HIP(hipStreamSynchronize(stream));
  std::vector<double> inv;
  rc = small_factor(G, rank, cap, (double)h->noise, n, P->small, &inv);
  if (rc != EGP_OK) return rc;
  EGP_HIP(hipMemcpyAsync(P->small_dev, inv.data(), sizeof(double) * rank * rank, hipMemcpyHostToDevice, stream));
  EGP_HIP(hipStreamSynchronize(stream));
  return EGP_OK;
}

}  // namespace egp
