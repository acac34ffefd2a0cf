// Fused derivative products dout[k] = (dK/dl_k) V for all lengthscales, K never materialised.
//
// Paper, Eq. 2: the marginal-likelihood gradient needs products with dKhat/dtheta. For the ARD
// lengthscales dK/dl_k [i,j] = s h(r_ij) (x_ik - x_jk)^2 / l_k^3 (chain rule on the kernels of kmm.hip).
//
// Per 16x16 tile the distance step is the one of kmm.hip (fp32 MFMA, transposed accumulator layout);
// then h(r) is evaluated once and, for every lengthscale k of the current pass, the tile
// w_k = h .* (x~_ik - x~_jk)^2 is formed on the VALU (3 operations per entry and k) and contracted with
// the V tile on the MFMA (4 steps per k). Lengthscales are processed in passes of at most DK so that the
// 4 * DK * R accumulator registers fit; each pass recomputes the distance tile (KS MFMA steps against
// 4 * DK). Column-side x~_jk are read from the same LDS tile that feeds the distance MFMA.

#include "egp_internal.h"

namespace egp {

typedef float f4 __attribute__((ext_vector_type(4)));

namespace {

constexpr float kLn2 = 0.6931471805599453f;
constexpr int DK = 13;   // lengthscales per pass
constexpr int GR = 2;    // row tiles per wave
constexpr int GJT = 8;   // column tiles per LDS stage

// h(r) up to a constant factor that the output scale carries (1, 3, 5/3; log2 e for Matern-1/2)
template <int KIND>
__device__ __forceinline__ float htransform(float acc) {
  if constexpr (KIND == EGP_RBF) {
    return __builtin_amdgcn_exp2f(-acc);
  } else if constexpr (KIND == EGP_MATERN32) {
    float a = __builtin_amdgcn_sqrtf(__builtin_fabsf(acc));
    return __builtin_amdgcn_exp2f(-a);
  } else if constexpr (KIND == EGP_MATERN12) {
    const float m = __builtin_fabsf(acc);      // exp(-r) / r, 0 for a point against itself
    return m > 0.f ? __builtin_amdgcn_exp2f(-__builtin_amdgcn_sqrtf(m)) * __builtin_amdgcn_rsqf(m) : 0.f;
  } else {
    float a = __builtin_amdgcn_sqrtf(__builtin_fabsf(acc));
    return __builtin_fmaf(a, kLn2, 1.0f) * __builtin_amdgcn_exp2f(-a);
  }
}

struct GradScale { float v[EGP_D_MAX + 1]; };

// Vp: [tile][lane] f4 (16 columns).  Part: [split][dk][npad][16] raw sums, or (direct = 1) the final
// dout[k0 + kk][row][c0 + c] with stride t, scaled.
template <int KS, int KIND>
__global__ __launch_bounds__(256, 2) void kmm_grad_kernel(const float* __restrict__ Xp,
                                                          const float* __restrict__ nrm,
                                                          const f4* __restrict__ Vp, float* __restrict__ dst,
                                                          int64_t npad, int64_t n, int d, int k0, int dk,
                                                          int stages_per_split, int stages_total, int direct,
                                                          int t, int c0, int tg, GradScale sc) {
  constexpr int XF4 = GJT * KS * 16;
  constexpr int VF4 = GJT * 64;
  constexpr int NX = (XF4 + 255) / 256;
  constexpr int NV = (VF4 + 255) / 256;
  __shared__ f4 Xs[2][XF4];
  __shared__ f4 Vs[2][VF4];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int q = lane >> 4, p = lane & 15;
  const int64_t row_tile0 = ((int64_t)blockIdx.x * 4 + wave) * GR;

  float b[GR][KS];
  f4 cq[GR];
  float xi[GR][DK];
  f4 o[GR][DK];
  const int ds = d >> 2, dq = d & 3;
#pragma unroll
  for (int it = 0; it < GR; ++it) {
    const float* tile = Xp + (row_tile0 + it) * KS * 64;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      float v = -2.0f * tile[s * 64 + lane];
      if (s == ds && q == dq) v = 1.0f;
      b[it][s] = v;
    }
    const float ni = nrm[(row_tile0 + it) * 16 + p];
    cq[it] = (f4){ni, ni, ni, ni};
#pragma unroll
    for (int kk = 0; kk < DK; ++kk) {
      const int f = k0 + kk;
      xi[it][kk] = (kk < dk) ? tile[(f >> 2) * 64 + (f & 3) * 16 + p] : 0.f;
      o[it][kk] = (f4){0.f, 0.f, 0.f, 0.f};
    }
  }

  const int st_begin = blockIdx.y * stages_per_split;
  int st_end = st_begin + stages_per_split;
  if (st_end > stages_total) st_end = stages_total;
  const f4* Xg = reinterpret_cast<const f4*>(Xp);
  f4 px[NX], pv[NV];
  auto fetch = [&](int st) {
    const int64_t xoff = (int64_t)st * XF4, voff = (int64_t)st * VF4;
#pragma unroll
    for (int k = 0; k < NX; ++k) {
      const int idx = tid + k * 256;
      if (XF4 % 256 == 0 || idx < XF4) px[k] = Xg[xoff + idx];
    }
#pragma unroll
    for (int k = 0; k < NV; ++k) pv[k] = Vp[voff + tid + k * 256];
  };
  auto stash = [&](int buf) {
#pragma unroll
    for (int k = 0; k < NX; ++k) {
      const int idx = tid + k * 256;
      if (XF4 % 256 == 0 || idx < XF4) Xs[buf][idx] = px[k];
    }
#pragma unroll
    for (int k = 0; k < NV; ++k) Vs[buf][tid + k * 256] = pv[k];
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
    for (int jt = 0; jt < GJT; ++jt) {
      const float* xt = xs + jt * KS * 64;
      float a[KS];
#pragma unroll
      for (int s = 0; s < KS; ++s) a[s] = xt[s * 64 + lane];
      const f4 v = Vs[buf][jt * 64 + lane];
      f4 h[GR];
#pragma unroll
      for (int it = 0; it < GR; ++it) {
        f4 acc = cq[it];
#pragma unroll
        for (int s = 0; s < KS; ++s) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[s], b[it][s], acc, 0, 0, 0);
        h[it].x = htransform<KIND>(acc.x);
        h[it].y = htransform<KIND>(acc.y);
        h[it].z = htransform<KIND>(acc.z);
        h[it].w = htransform<KIND>(acc.w);
      }
#pragma unroll
      for (int kk = 0; kk < DK; ++kk) {
        if (kk < dk) {
          const int f = k0 + kk;
          // x~_jk for the four columns j = 4q + r of this lane group (broadcast read)
          const f4 xj = *reinterpret_cast<const f4*>(xt + (f >> 2) * 64 + (f & 3) * 16 + q * 4);
#pragma unroll
          for (int it = 0; it < GR; ++it) {
            const float d0 = xi[it][kk] - xj.x, d1 = xi[it][kk] - xj.y;
            const float d2 = xi[it][kk] - xj.z, d3 = xi[it][kk] - xj.w;
            o[it][kk] = __builtin_amdgcn_mfma_f32_16x16x4f32(h[it].x * d0 * d0, v.x, o[it][kk], 0, 0, 0);
            o[it][kk] = __builtin_amdgcn_mfma_f32_16x16x4f32(h[it].y * d1 * d1, v.y, o[it][kk], 0, 0, 0);
            o[it][kk] = __builtin_amdgcn_mfma_f32_16x16x4f32(h[it].z * d2 * d2, v.z, o[it][kk], 0, 0, 0);
            o[it][kk] = __builtin_amdgcn_mfma_f32_16x16x4f32(h[it].w * d3 * d3, v.w, o[it][kk], 0, 0, 0);
          }
        }
      }
    }
    if (more) stash(buf ^ 1);
    __syncthreads();
  }

#pragma unroll
  for (int it = 0; it < GR; ++it) {
    const int64_t row0 = (row_tile0 + it) * 16 + q * 4;
#pragma unroll
    for (int kk = 0; kk < DK; ++kk) {
      if (kk < dk) {
        const float vals[4] = {o[it][kk].x, o[it][kk].y, o[it][kk].z, o[it][kk].w};
        if (direct) {
          const float scale = sc.v[k0 + kk];
          if (p < tg) {
#pragma unroll
            for (int r = 0; r < 4; ++r)
              if (row0 + r < n) dst[((int64_t)(k0 + kk) * n + row0 + r) * t + c0 + p] = scale * vals[r];
          }
        } else {
          float* base = dst + (((int64_t)blockIdx.y * dk + kk) * npad + row0) * 16 + p;
#pragma unroll
          for (int r = 0; r < 4; ++r) base[r * 16] = vals[r];
        }
      }
    }
  }
}

__global__ __launch_bounds__(256) void grad_epilogue(const float* __restrict__ Part, int splits, int dk,
                                                     int64_t npad, int64_t n, int t, int c0, int tg, int k0,
                                                     GradScale sc, float* __restrict__ dout) {
  int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;   // (kk, row, c)
  const int64_t total = (int64_t)dk * n * tg;
  if (g >= total) return;
  const int c = (int)(g % tg);
  const int64_t row = (g / tg) % n;
  const int kk = (int)(g / ((int64_t)tg * n));
  float acc = 0.f;
  for (int sp = 0; sp < splits; ++sp) acc += Part[(((int64_t)sp * dk + kk) * npad + row) * 16 + c];
  dout[((int64_t)(k0 + kk) * n + row) * t + c0 + c] = sc.v[k0 + kk] * acc;
}


struct GPlan { int row_blocks, splits, stages_per_split, stages_total; };
GPlan grad_plan(int64_t npad) {
  GPlan pl;
  pl.row_blocks = (int)(npad / (64 * GR));
  pl.stages_total = (int)(npad / (16 * GJT));
  int want = 1024 / pl.row_blocks;
  if (want < 1) want = 1;
  if (want > pl.stages_total) want = pl.stages_total;
  if (want > 32) want = 32;
  pl.stages_per_split = (pl.stages_total + want - 1) / want;
  pl.splits = (pl.stages_total + pl.stages_per_split - 1) / pl.stages_per_split;
  return pl;
}

template <int KS>
int launch_grad(const Prepared& P, const GPlan& pl, const f4* Vp, float* dst, int k0, int dk, int direct, int t,
                int c0, int tg, const GradScale& sc, hipStream_t stream) {
  dim3 grid(pl.row_blocks, pl.splits), block(256);
  switch (P.kernel_type) {
    case EGP_RBF:
      hipLaunchKernelGGL((kmm_grad_kernel<KS, EGP_RBF>), grid, block, 0, stream, P.Xp, P.nrm, Vp, dst, P.npad, P.n,
                         P.d, k0, dk, pl.stages_per_split, pl.stages_total, direct, t, c0, tg, sc);
      break;
    case EGP_MATERN32:
      hipLaunchKernelGGL((kmm_grad_kernel<KS, EGP_MATERN32>), grid, block, 0, stream, P.Xp, P.nrm, Vp, dst, P.npad,
                         P.n, P.d, k0, dk, pl.stages_per_split, pl.stages_total, direct, t, c0, tg, sc);
      break;
    case EGP_MATERN12:
      hipLaunchKernelGGL((kmm_grad_kernel<KS, EGP_MATERN12>), grid, block, 0, stream, P.Xp, P.nrm, Vp, dst, P.npad,
                         P.n, P.d, k0, dk, pl.stages_per_split, pl.stages_total, direct, t, c0, tg, sc);
      break;
    default:
      hipLaunchKernelGGL((kmm_grad_kernel<KS, EGP_MATERN52>), grid, block, 0, stream, P.Xp, P.nrm, Vp, dst, P.npad,
                         P.n, P.d, k0, dk, pl.stages_per_split, pl.stages_total, direct, t, c0, tg, sc);
  }
  EGP_HIP(hipGetLastError());
  return EGP_OK;
}

}  // namespace

size_t kmm_grad_core_ws_bytes(int64_t n, int d, int t) {
  const int64_t npad = padded_points(n);
  const GPlan pl = grad_plan(npad);
  size_t b = round_up((size_t)npad * 16 * sizeof(float), 256);   // Vp
  if (pl.splits > 1) b += round_up((size_t)pl.splits * DK * npad * 16 * sizeof(float), 256);
  return b;
}

int kmm_grad_core(const Prepared& P, const egp_hyper_t* h, const float* V, int t, float* dout, void* ws2,
                  hipStream_t stream) {
  const int64_t npad = P.npad;
  const GPlan pl = grad_plan(npad);
  char* w = static_cast<char*>(ws2);
  f4* Vp = reinterpret_cast<f4*>(w);
  w += round_up((size_t)npad * 16 * sizeof(float), 256);
  float* Part = reinterpret_cast<float*>(w);

  // x~ = c x / l  =>  (x_ik - x_jk)^2 / l_k^3 = (x~_ik - x~_jk)^2 / (l_k c^2); Matern h carries 3 resp. 5/3
  const double c2 = h->kernel_type == EGP_RBF ? 0.5 * 1.4426950408889634
                    : (h->kernel_type == EGP_MATERN32 ? 3.0 : (h->kernel_type == EGP_MATERN52 ? 5.0 : 1.0)) *
                          1.4426950408889634 * 1.4426950408889634;
  // Matern-1/2: h = exp(-r) / r = log2(e) exp2(-a) / a with a = r log2(e)
  const double hfac = h->kernel_type == EGP_RBF ? 1.0
                      : (h->kernel_type == EGP_MATERN32 ? 3.0 : (h->kernel_type == EGP_MATERN52 ? 5.0 / 3.0 : 1.4426950408889634));
  GradScale sc;
  for (int k = 0; k <= EGP_D_MAX; ++k)
    sc.v[k] = k < P.d ? (float)((double)h->outputscale * hfac / ((double)h->lengthscales[k] * c2)) : 0.f;

  const int passes = (P.d + DK - 1) / DK;
  const int per = (P.d + passes - 1) / passes;
  const int direct = pl.splits == 1 ? 1 : 0;
  for (int c0 = 0; c0 < t; c0 += 16) {
    const int tg = t - c0 < 16 ? t - c0 : 16;
    {
      ProfScope prof(kProfPack, stream);
      launch_pack_rhs(V, P.n, npad, t, c0, 1, 0, Vp, nullptr, stream);
    }
    for (int k0 = 0; k0 < P.d; k0 += per) {
      const int dk = P.d - k0 < per ? P.d - k0 : per;
      float* dst = direct ? dout : Part;
      int rc;
      {
        ProfScope prof(kProfGrad, stream);
        switch (P.ks) {
          case 1: rc = launch_grad<1>(P, pl, Vp, dst, k0, dk, direct, t, c0, tg, sc, stream); break;
          case 2: rc = launch_grad<2>(P, pl, Vp, dst, k0, dk, direct, t, c0, tg, sc, stream); break;
          case 3: rc = launch_grad<3>(P, pl, Vp, dst, k0, dk, direct, t, c0, tg, sc, stream); break;
          case 4: rc = launch_grad<4>(P, pl, Vp, dst, k0, dk, direct, t, c0, tg, sc, stream); break;
          case 5: rc = launch_grad<5>(P, pl, Vp, dst, k0, dk, direct, t, c0, tg, sc, stream); break;
          case 6: rc = launch_grad<6>(P, pl, Vp, dst, k0, dk, direct, t, c0, tg, sc, stream); break;
          case 7: rc = launch_grad<7>(P, pl, Vp, dst, k0, dk, direct, t, c0, tg, sc, stream); break;
          case 8: rc = launch_grad<8>(P, pl, Vp, dst, k0, dk, direct, t, c0, tg, sc, stream); break;
          default: rc = fail(EGP_ERR_ARG, "d = %d: the derivative kernel supports d <= 31", P.d);
        }
      }
      if (rc != EGP_OK) return rc;
      if (!direct) {
        ProfScope prof(kProfPack, stream);
        const int64_t total = (int64_t)dk * P.n * tg;
        hipLaunchKernelGGL(grad_epilogue, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, Part,
                           pl.splits, dk, npad, P.n, t, c0, tg, k0, sc, dout);
        EGP_HIP(hipGetLastError());
      }
    }
  }
  return EGP_OK;
}

}  // namespace egp
