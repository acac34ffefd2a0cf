// Bilinear forms with the kernel derivatives, K never materialised and no n x t x d intermediate:
//   out[k] = sum_ij S_ij dK_ij/dl_k  (k < d),   out[d] = sum_ij S_ij K_ij / s,   S_ij = sum_c A[i][c] B[j][c].
//
// Paper, Eq. 2: every term of the marginal-likelihood gradient is such a form — u^T (dK/dtheta) u with
// A = B = u, and the probe estimate of tr(Khat^{-1} dK/dtheta) with A = Khat^{-1} z_c, B = P^{-1} z_c. Folding
// the column weights (+1/2 for y, -1/(2 t_p) for each probe) into A gives the whole gradient in one pass.
//
// Per 16 x 16 tile and wave: KS fp32 MFMA steps for the distance (as in kmm.hip, transposed accumulator
// layout), TS = ceil(t/4) MFMA steps for S^T[j][i] = sum_c B[j][c] A[i][c] (same layout, so S, h and the
// feature differences meet lane by lane), then on the VALU w = S h and for every lengthscale
// acc_k += w (x~_ik - x~_jk)^2. The accumulators are per lane (d + 1 registers per wave, not per row tile);
// they are reduced across the wave, the block and the grid at the end, the last step in fp64.
// Against materialising (dK/dl_k) V (4 d MFMA steps per tile) this needs TS MFMA steps per tile.
//
// dK/dtheta is symmetric, so only S + S^T matters: sum_ij S_ij D_ij = sum over tile pairs {I,J} of
// (S_IJ + S_JI^T) . D_IJ. A workgroup sweeps the column blocks (256 points) from its own to the half-way one,
// cyclically, and forms S_IJ + S_JI^T = Aw_I B_J^T + B_I Aw_J^T with 2 TS MFMA steps per tile; the own block and the
// half-way block (which both partners visit) carry the weight 1/2. Half of all tiles are never formed: the distance
// steps, the transform and above all the per-lengthscale VALU work are halved.

#include <math.h>

#include <vector>

#include "egp_internal.h"
#include "bilinear_detail.h"

namespace egp {

namespace {

using bilinear_detail::f4;
using bilinear_detail::hg;

// row tiles per wave: fewer when the per-tile registers (4 KS features, 2 TS operands of S + S^T) grow
constexpr int br_for(int ks, int ts) { return ks <= 5 ? ((ks == 3 && ts <= 5) ? 4 : 2) : 1; }
constexpr int BJT = 4;     // column tiles per LDS stage
constexpr int kBlk = 256;  // points per block of the symmetric sweep (a multiple of every workgroup's row count)
constexpr int kDMaxB = 31; // lengthscales handled by this kernel (d > 31: kmm_bilinear_wide.hip)

// M (n x t row-major) -> packed [tile][ts][64]: lane (q,p) of step s holds w[4s+q] * M[16 tile + p][4s + q]
__global__ __launch_bounds__(256) void pack_cols(const float* __restrict__ M, int64_t n, int64_t npad, int t, int ts,
                                                 const float* __restrict__ wcol, float* __restrict__ Mp) {
  int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t total = (npad >> 4) * ts * 64;
  if (g >= total) return;
  const int lane = (int)(g & 63);
  const int64_t rest = g >> 6;
  const int s = (int)(rest % ts);
  const int64_t tile = rest / ts;
  const int q = lane >> 4, p = lane & 15;
  const int c = 4 * s + q;
  const int64_t i = tile * 16 + p;
  float v = 0.f;
  if (c < t && i < n) v = M[i * t + c] * (wcol ? wcol[c] : 1.0f);
  Mp[g] = v;
}

template <int KS, int TS, int KIND>
__global__ __launch_bounds__(256, 2) void bilinear_kernel(const float* __restrict__ Xp, const float* __restrict__ nrm,
                                                          const float* __restrict__ Ap, const float* __restrict__ Bp,
                                                          float* __restrict__ part, int64_t npad, int d,
                                                          int stages_per_split) {
  constexpr int BR = br_for(KS, TS);
  constexpr int SB = kBlk / (16 * BJT);      // stages per block
  constexpr int XF4 = BJT * KS * 16;
  constexpr int BF4 = BJT * TS * 16;
  constexpr int NX = (XF4 + 255) / 256;
  constexpr int NB = (BF4 + 255) / 256;
  __shared__ f4 Xs[2][XF4];
  __shared__ f4 Bs[2][BF4];      // B of the column tiles
  __shared__ f4 As[2][BF4];      // A (weighted) of the column tiles
  __shared__ float red[4][kDMaxB + 1];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int q = lane >> 4, p = lane & 15;
  const int64_t row_tile0 = ((int64_t)blockIdx.x * 4 + wave) * BR;

  float b[BR][KS], a_op[BR][TS], b_op[BR][TS], xi[BR][KS * 4];
  f4 cq[BR];
  float acc_k[KS * 4];     // one accumulator per feature slot; slots >= d stay unused
  float acc_s = 0.f;
  const int ds = d >> 2, dq = d & 3;
#pragma unroll
  for (int k = 0; k < KS * 4; ++k) acc_k[k] = 0.f;
#pragma unroll
  for (int it = 0; it < BR; ++it) {
    const float* tile = Xp + (row_tile0 + it) * KS * 64;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      float v = -2.0f * tile[s * 64 + lane];
      if (s == ds && q == dq) v = 1.0f;
      b[it][s] = v;
    }
#pragma unroll
    for (int s = 0; s < TS; ++s) {
      a_op[it][s] = Ap[((row_tile0 + it) * TS + s) * 64 + lane];
      b_op[it][s] = Bp[((row_tile0 + it) * TS + s) * 64 + lane];
    }
    const float ni = nrm[(row_tile0 + it) * 16 + p];
    cq[it] = (f4){ni, ni, ni, ni};
#pragma unroll
    for (int k = 0; k < KS * 4; ++k) xi[it][k] = tile[(k >> 2) * 64 + (k & 3) * 16 + p];
  }

  // this workgroup's sweep: blocks own, own + 1, ..., own + half (cyclic), SB stages each
  const int nblk = (int)(npad / kBlk);      // even: npad is a multiple of 512
  const int half = nblk >> 1;
  const int own = (int)(((int64_t)blockIdx.x * 64 * BR) / kBlk);
  const int stages_all = (half + 1) * SB;
  const int s_total = nblk * SB;
  const int st_begin = blockIdx.y * stages_per_split;
  int st_end = st_begin + stages_per_split;
  if (st_end > stages_all) st_end = stages_all;
  auto abs_stage = [&](int k) {
    int st = own * SB + k;
    return st >= s_total ? st - s_total : st;
  };
  const f4* Xg = reinterpret_cast<const f4*>(Xp);
  const f4* Bg = reinterpret_cast<const f4*>(Bp);
  const f4* Ag = reinterpret_cast<const f4*>(Ap);
  f4 px[NX], pb[NB], pa[NB];
  auto fetch = [&](int k) {
    const int st = abs_stage(k);
    const int64_t xoff = (int64_t)st * XF4, boff = (int64_t)st * BF4;
#pragma unroll
    for (int i = 0; i < NX; ++i) {
      const int idx = tid + i * 256;
      if (XF4 % 256 == 0 || idx < XF4) px[i] = Xg[xoff + idx];
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      const int idx = tid + i * 256;
      if (BF4 % 256 == 0 || idx < BF4) {
        pb[i] = Bg[boff + idx];
        pa[i] = Ag[boff + idx];
      }
    }
  };
  auto stash = [&](int buf) {
#pragma unroll
    for (int i = 0; i < NX; ++i) {
      const int idx = tid + i * 256;
      if (XF4 % 256 == 0 || idx < XF4) Xs[buf][idx] = px[i];
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      const int idx = tid + i * 256;
      if (BF4 % 256 == 0 || idx < BF4) {
        Bs[buf][idx] = pb[i];
        As[buf][idx] = pa[i];
      }
    }
  };

  if (st_begin < st_end) {
    fetch(st_begin);
    stash(0);
  }
  __syncthreads();

  for (int st = st_begin; st < st_end; ++st) {
    const int buf = (st - st_begin) & 1;
    const bool more = st + 1 < st_end;
    if (more) fetch(st + 1);
    const float* xs = reinterpret_cast<const float*>(Xs[buf]);
    const float* bs = reinterpret_cast<const float*>(Bs[buf]);
    const float* as = reinterpret_cast<const float*>(As[buf]);
    const int delta = st / SB;
    const float wgt = (delta == 0 || delta == half) ? 0.5f : 1.0f;
    for (int jt = 0; jt < BJT; ++jt) {
      const float* xt = xs + jt * KS * 64;
      const float* bt = bs + jt * TS * 64;
      const float* at = as + jt * TS * 64;
      float a[KS], bo[TS], ao[TS];
#pragma unroll
      for (int s = 0; s < KS; ++s) a[s] = xt[s * 64 + lane];
#pragma unroll
      for (int s = 0; s < TS; ++s) {
        bo[s] = bt[s * 64 + lane];
        ao[s] = at[s * 64 + lane];
      }
      f4 w[BR];
#pragma unroll
      for (int it = 0; it < BR; ++it) {
        f4 acc = cq[it];
#pragma unroll
        for (int s = 0; s < KS; ++s) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[s], b[it][s], acc, 0, 0, 0);
        f4 sv = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < TS; ++s) sv = __builtin_amdgcn_mfma_f32_16x16x4f32(bo[s], a_op[it][s], sv, 0, 0, 0);
#pragma unroll
        for (int s = 0; s < TS; ++s) sv = __builtin_amdgcn_mfma_f32_16x16x4f32(ao[s], b_op[it][s], sv, 0, 0, 0);
        sv *= wgt;
        float g0, g1, g2, g3;
        const float h0 = hg<KIND>(acc.x, &g0), h1 = hg<KIND>(acc.y, &g1);
        const float h2 = hg<KIND>(acc.z, &g2), h3 = hg<KIND>(acc.w, &g3);
        acc_s = __builtin_fmaf(sv.x, g0, acc_s);
        acc_s = __builtin_fmaf(sv.y, g1, acc_s);
        acc_s = __builtin_fmaf(sv.z, g2, acc_s);
        acc_s = __builtin_fmaf(sv.w, g3, acc_s);
        w[it] = (f4){sv.x * h0, sv.y * h1, sv.z * h2, sv.w * h3};
      }
#pragma unroll
      for (int k = 0; k < KS * 4; ++k) {
        if (k < d) {
          // x~_jk of the four columns j = 4q + r of this lane group (broadcast read of the distance tile)
          const f4 xj = *reinterpret_cast<const f4*>(xt + (k >> 2) * 64 + (k & 3) * 16 + q * 4);
#pragma unroll
          for (int it = 0; it < BR; ++it) {
            const float d0 = xi[it][k] - xj.x, d1 = xi[it][k] - xj.y;
            const float d2 = xi[it][k] - xj.z, d3 = xi[it][k] - xj.w;
            acc_k[k] = __builtin_fmaf(w[it].x * d0, d0, acc_k[k]);
            acc_k[k] = __builtin_fmaf(w[it].y * d1, d1, acc_k[k]);
            acc_k[k] = __builtin_fmaf(w[it].z * d2, d2, acc_k[k]);
            acc_k[k] = __builtin_fmaf(w[it].w * d3, d3, acc_k[k]);
          }
        }
      }
    }
    if (more) stash(buf ^ 1);
    __syncthreads();
  }

  // ---- reduce: lanes -> wave -> block; one partial vector per block ----
#pragma unroll
  for (int k = 0; k < KS * 4; ++k) {
    float v = acc_k[k];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
    if (lane == 0 && k < d) red[wave][k] = v;
  }
  {
    float v = acc_s;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
    if (lane == 0) red[wave][d] = v;
  }
  __syncthreads();
  if (tid <= d) {
    const int64_t blk = (int64_t)blockIdx.y * gridDim.x + blockIdx.x;
    part[blk * (kDMaxB + 1) + tid] = (red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid]);
  }
}

struct BPlan { int row_blocks, splits, stages_per_split, stages_total; };
BPlan bilinear_plan(int64_t npad, int ks, int ts) {
  BPlan pl;
  pl.row_blocks = (int)(npad / (64 * br_for(ks, ts)));
  // one workgroup's sweep: its own block and the following npad / (2 kBlk) blocks, kBlk / (16 BJT) stages each
  pl.stages_total = (int)(npad / kBlk / 2 + 1) * (kBlk / (16 * BJT));
  int want = 1024 / pl.row_blocks;
  if (want < 1) want = 1;
  if (want > pl.stages_total) want = pl.stages_total;
  if (want > 64) want = 64;
  pl.stages_per_split = (pl.stages_total + want - 1) / want;
  pl.splits = (pl.stages_total + pl.stages_per_split - 1) / pl.stages_per_split;
  return pl;
}

template <int KS, int TS>
void launch_b(const Prepared& P, const BPlan& pl, const float* Ap, const float* Bp, float* part, hipStream_t stream) {
  dim3 grid(pl.row_blocks, pl.splits), block(256);
  switch (P.kernel_type) {
    case EGP_RBF:
      hipLaunchKernelGGL((bilinear_kernel<KS, TS, EGP_RBF>), grid, block, 0, stream, P.Xp, P.nrm, Ap, Bp, part, P.npad,
                         P.d, pl.stages_per_split);
      break;
    case EGP_MATERN32:
      hipLaunchKernelGGL((bilinear_kernel<KS, TS, EGP_MATERN32>), grid, block, 0, stream, P.Xp, P.nrm, Ap, Bp, part,
                         P.npad, P.d, pl.stages_per_split);
      break;
    case EGP_MATERN12:
      hipLaunchKernelGGL((bilinear_kernel<KS, TS, EGP_MATERN12>), grid, block, 0, stream, P.Xp, P.nrm, Ap, Bp, part,
                         P.npad, P.d, pl.stages_per_split);
      break;
    default:
      hipLaunchKernelGGL((bilinear_kernel<KS, TS, EGP_MATERN52>), grid, block, 0, stream, P.Xp, P.nrm, Ap, Bp, part,
                         P.npad, P.d, pl.stages_per_split);
  }
}

template <int KS>
int launch_ts(const Prepared& P, const BPlan& pl, int ts, const float* Ap, const float* Bp, float* part,
              hipStream_t stream) {
  switch (ts) {
    case 1: launch_b<KS, 1>(P, pl, Ap, Bp, part, stream); break;
    case 2: launch_b<KS, 2>(P, pl, Ap, Bp, part, stream); break;
    case 3: launch_b<KS, 3>(P, pl, Ap, Bp, part, stream); break;
    case 4: launch_b<KS, 4>(P, pl, Ap, Bp, part, stream); break;
    case 5: launch_b<KS, 5>(P, pl, Ap, Bp, part, stream); break;
    case 6: launch_b<KS, 6>(P, pl, Ap, Bp, part, stream); break;
    case 7: launch_b<KS, 7>(P, pl, Ap, Bp, part, stream); break;
    case 8: launch_b<KS, 8>(P, pl, Ap, Bp, part, stream); break;
    case 9: launch_b<KS, 9>(P, pl, Ap, Bp, part, stream); break;
    default: return fail(EGP_ERR_ARG, "bilinear forms support t <= 36");
  }
  EGP_HIP(hipGetLastError());
  return EGP_OK;
}

}  // namespace

size_t bilinear_core_ws_bytes(int64_t n, int d, int t) {
  if (ksteps_for(d) > 8) return bilinear_detail::bilinear_wide_ws_bytes(n, d, t);
  const int64_t npad = padded_points(n);
  const int ts = (t + 3) / 4;
  const BPlan pl = bilinear_plan(npad, ksteps_for(d), ts);
  size_t b = 2 * round_up((size_t)npad * ts * 4 * sizeof(float), 256);                                 // Ap, Bp
  b += round_up((size_t)pl.row_blocks * pl.splits * (kDMaxB + 1) * sizeof(float), 256);                // partials
  b += 256;                                                                                            // column weights
  return b;
}

// out[0..d-1] = sum_ij S_ij dK_ij/dl_k, out[d] = sum_ij S_ij K_ij / s with S = (A diag(wcol)) B^T.
// A, B: device n x t row-major; wcol: host t weights or NULL. Synchronises on the stream.
int bilinear_core(const Prepared& P, const egp_hyper_t* h, const float* A, const float* B, int t, const float* wcol,
                  double* out, void* ws2, hipStream_t stream) {
  if (P.ks > 8) return bilinear_detail::bilinear_wide_core(P, h, A, B, t, wcol, out, ws2, stream);
  const int64_t npad = P.npad;
  const int ts = (t + 3) / 4;
  if (ts > 9) return fail(EGP_ERR_ARG, "bilinear forms support t <= 36 (got %d)", t);
  const BPlan pl = bilinear_plan(npad, P.ks, ts);
  char* w = static_cast<char*>(ws2);
  const size_t pbytes = round_up((size_t)npad * ts * 4 * sizeof(float), 256);
  float* Ap = reinterpret_cast<float*>(w);
  float* Bp = reinterpret_cast<float*>(w + pbytes);
  w += 2 * pbytes;
  float* part = reinterpret_cast<float*>(w);
  const int64_t nblk = (int64_t)pl.row_blocks * pl.splits;
  w += round_up((size_t)nblk * (kDMaxB + 1) * sizeof(float), 256);
  float* wdev = reinterpret_cast<float*>(w);
  if (wcol) EGP_HIP(hipMemcpyAsync(wdev, wcol, sizeof(float) * t, hipMemcpyHostToDevice, stream));
  {
    ProfScope prof(kProfPack, stream);
    const int64_t total = (npad >> 4) * ts * 64;
    const unsigned blocks = (unsigned)((total + 255) / 256);
    hipLaunchKernelGGL(pack_cols, dim3(blocks), dim3(256), 0, stream, A, P.n, npad, t, ts, wcol ? wdev : nullptr, Ap);
    hipLaunchKernelGGL(pack_cols, dim3(blocks), dim3(256), 0, stream, B, P.n, npad, t, ts,
                       static_cast<const float*>(nullptr), Bp);
  }
  int rc;
  {
    ProfScope prof(kProfGrad, stream);
    switch (P.ks) {
      case 1: rc = launch_ts<1>(P, pl, ts, Ap, Bp, part, stream); break;
      case 2: rc = launch_ts<2>(P, pl, ts, Ap, Bp, part, stream); break;
      case 3: rc = launch_ts<3>(P, pl, ts, Ap, Bp, part, stream); break;
      case 4: rc = launch_ts<4>(P, pl, ts, Ap, Bp, part, stream); break;
      case 5: rc = launch_ts<5>(P, pl, ts, Ap, Bp, part, stream); break;
      case 6: rc = launch_ts<6>(P, pl, ts, Ap, Bp, part, stream); break;
      case 7: rc = launch_ts<7>(P, pl, ts, Ap, Bp, part, stream); break;
      case 8: rc = launch_ts<8>(P, pl, ts, Ap, Bp, part, stream); break;
      default: rc = fail(EGP_ERR_ARG, "d = %d: the bilinear kernel supports d <= 31", P.d);
    }
  }
  if (rc != EGP_OK) return rc;
  std::vector<float> hp((size_t)nblk * (kDMaxB + 1));
  EGP_HIP(hipMemcpyAsync(hp.data(), part, hp.size() * sizeof(float), hipMemcpyDeviceToHost, stream));
  EGP_HIP(hipStreamSynchronize(stream));
  const double c2 = h->kernel_type == EGP_RBF ? 0.5 * 1.4426950408889634
                    : (h->kernel_type == EGP_MATERN32 ? 3.0 : (h->kernel_type == EGP_MATERN52 ? 5.0 : 1.0)) *
                          1.4426950408889634 * 1.4426950408889634;
  // Matern-1/2: h = exp(-r) / r = log2(e) exp2(-a) / a with a = r log2(e)
  const double hfac = h->kernel_type == EGP_RBF ? 1.0
                      : (h->kernel_type == EGP_MATERN32 ? 3.0 : (h->kernel_type == EGP_MATERN52 ? 5.0 / 3.0 : 1.4426950408889634));
  for (int k = 0; k <= P.d; ++k) {
    double s = 0.0;
    for (int64_t bidx = 0; bidx < nblk; ++bidx) s += (double)hp[(size_t)bidx * (kDMaxB + 1) + k];
    // lengthscales: (x_ik - x_jk)^2 / l_k^3 = (x~_ik - x~_jk)^2 / (l_k c^2), h carries 1, 3 or 5/3;
    // slot d: sum S g = sum S K / s
    out[k] = k < P.d ? s * (double)h->outputscale * hfac / ((double)h->lengthscales[k] * c2) : s;
  }
  return EGP_OK;
}

}  // namespace egp
