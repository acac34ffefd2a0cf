// Fused kernel-matrix multiply for inputs of more than 31 dimensions (up to EGP_D_WIDE_MAX).
//
// Same tile algebra as kmm_kernel.h, but the distance step needs KS = ceil((d+1)/4) > 8 MFMA k-steps and the
// per-row-tile operands no longer fit in registers: both distance operands are read from LDS inside a
// run-time loop over the k-steps. A workgroup keeps the packed rows of its 4 x RW row tiles in LDS for the
// whole column sweep (KS KB per row tile) and streams column tiles through a double-buffered stage. The
// kernel stays bound by the fp32 MFMA: KS + 4 steps per tile against two 256-byte LDS reads per step.

#include "kmm_kernel.h"

namespace egp {

namespace {

template <int RW, int KIND, int NB, int EXTRA>
__global__ __launch_bounds__(256) void kmm_kernel_wide(const float* __restrict__ XpRow, const float* __restrict__ nrm,
                                                       const float* __restrict__ Xp, const f4* __restrict__ Vp,
                                                       const float* __restrict__ Ep, float* __restrict__ Part,
                                                       int64_t npad, int d, int ks, int jt_stage,
                                                       int stages_per_split, int stages_total, int cm) {
  constexpr int TS = 16 * NB + EXTRA;
  extern __shared__ __align__(16) unsigned char smem[];
  // layout: rows [4*RW][ks][64] floats | 2 x column stage [jt_stage][ks][64] floats | 2 x V stage | 2 x extra stage
  float* Rs = reinterpret_cast<float*>(smem);
  float* Xs = Rs + 4 * RW * ks * 64;
  f4* Vs = reinterpret_cast<f4*>(Xs + 2 * jt_stage * ks * 64);
  f4* Es = Vs + 2 * jt_stage * NB * 64;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int q = lane >> 4, p = lane & 15;
  const int64_t row_tile0 = ((int64_t)blockIdx.x * 4 + wave) * RW;
  const int ds = d >> 2, dq = d & 3;

  // rows of this wave: -2 x~ with the norm slot set to 1, same element order as the packed tiles
  const int ks4 = ks >> 2, kt = ks & 3;      // groups of four k-steps, left-over steps
  for (int it = 0; it < RW; ++it) {
    const float* src = XpRow + (row_tile0 + it) * ks * 64;
    float* dstr = Rs + (wave * RW + it) * ks * 64;
    for (int e = lane; e < ks * 64; e += 64) {
      int s_, l_;
      if (e < ks4 * 256) {
        s_ = (e >> 8) * 4 + (e & 3);
        l_ = (e >> 2) & 63;
      } else {
        s_ = e >> 6;
        l_ = e & 63;
      }
      dstr[e] = (s_ == ds && (l_ >> 4) == dq) ? 1.0f : -2.0f * src[e];
    }
  }
  f4 cq[RW], o[RW][NB], o2[RW][NB];      // o: current block of 4096 column points, o2: sum of the blocks
  float eacc[RW], eacc2[RW];
#pragma unroll
  for (int it = 0; it < RW; ++it) {
    const float ni = nrm[(row_tile0 + it) * 16 + p];
    cq[it] = (f4){ni, ni, ni, ni};
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      o[it][nb] = (f4){0.f, 0.f, 0.f, 0.f};
      o2[it][nb] = (f4){0.f, 0.f, 0.f, 0.f};
    }
    eacc[it] = 0.f;
    eacc2[it] = 0.f;
  }
  auto fold = [&]() {      // two-level accumulation, see kmm_kernel.h
#pragma unroll
    for (int it = 0; it < RW; ++it) {
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        o2[it][nb] += o[it][nb];
        o[it][nb] = (f4){0.f, 0.f, 0.f, 0.f};
      }
      if (EXTRA) {
        eacc2[it] += eacc[it];
        eacc[it] = 0.f;
      }
    }
  };
  const int flush_stages = 256 / jt_stage;

  const int st_begin = blockIdx.y * stages_per_split;
  int st_end = st_begin + stages_per_split;
  if (st_end > stages_total) st_end = stages_total;
  const int xf4 = jt_stage * ks * 16, vf4 = jt_stage * NB * 64, ef4 = jt_stage * 4;
  const f4* Xg = reinterpret_cast<const f4*>(Xp);
  const f4* Eg = reinterpret_cast<const f4*>(Ep);
  auto issue = [&](int st, int buf) {
    const int64_t xoff = (int64_t)st * xf4, voff = (int64_t)st * vf4, eoff = (int64_t)st * ef4;
    f4* xs4 = reinterpret_cast<f4*>(Xs + buf * jt_stage * ks * 64);
    for (int k = wave * 64; k < xf4; k += 256)
      if (k + lane < xf4)      // xf4 is a multiple of 16, not of 64
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Xg + xoff + k + lane),
                                         (__attribute__((address_space(3))) void*)(xs4 + k), 16, 0, 0);
    for (int k = wave * 64; k < vf4; k += 256)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Vp + voff + k + lane),
                                       (__attribute__((address_space(3))) void*)(Vs + buf * vf4 + k), 16, 0, 0);
    if (EXTRA && tid < ef4)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Eg + eoff + tid),
                                       (__attribute__((address_space(3))) void*)(Es + buf * ef4), 16, 0, 0);
  };
  if (st_begin < st_end) issue(st_begin, 0);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();

  f4 rfirst[RW];      // row operands of the first group of four k-steps: resident in registers
#pragma unroll
  for (int it = 0; it < RW; ++it) rfirst[it] = reinterpret_cast<const f4*>(Rs + (wave * RW + it) * ks * 64)[lane];

  for (int st = st_begin; st < st_end; ++st) {
    const int buf = (st - st_begin) & 1;
    const bool more = st + 1 < st_end;
    if (more) issue(st + 1, buf ^ 1);
    const float* xs = Xs + buf * jt_stage * ks * 64;
    for (int jt = 0; jt < jt_stage; ++jt) {
      const float* xt = xs + jt * ks * 64;
      const f4* xg = reinterpret_cast<const f4*>(xt) + lane;
      f4 acc[RW];
      const f4* rg[RW];
#pragma unroll
      for (int it = 0; it < RW; ++it) rg[it] = reinterpret_cast<const f4*>(Rs + (wave * RW + it) * ks * 64) + lane;
      // left-over steps first (index clamped, so the loads need no branch): in flight while the groups run
      float ta[3], tr[RW][3];
#pragma unroll
      for (int k = 0; k < 3; ++k) {
        const int sk = ks4 * 4 + k < ks ? ks4 * 4 + k : ks - 1;
        ta[k] = xt[sk * 64 + lane];
#pragma unroll
        for (int it = 0; it < RW; ++it) tr[it][k] = Rs[((wave * RW + it) * ks + sk) * 64 + lane];
      }
      // groups of four steps, two groups per trip with the operands of the next group loaded ahead (ping-pong)
      auto four = [&](const f4& a, const f4 (&r)[RW]) {
#pragma unroll
        for (int it = 0; it < RW; ++it) acc[it] = __builtin_amdgcn_mfma_f32_16x16x4f32(a.x, r[it].x, acc[it], 0, 0, 0);
#pragma unroll
        for (int it = 0; it < RW; ++it) acc[it] = __builtin_amdgcn_mfma_f32_16x16x4f32(a.y, r[it].y, acc[it], 0, 0, 0);
#pragma unroll
        for (int it = 0; it < RW; ++it) acc[it] = __builtin_amdgcn_mfma_f32_16x16x4f32(a.z, r[it].z, acc[it], 0, 0, 0);
#pragma unroll
        for (int it = 0; it < RW; ++it) acc[it] = __builtin_amdgcn_mfma_f32_16x16x4f32(a.w, r[it].w, acc[it], 0, 0, 0);
      };
      // Group 0 is peeled: its row operands never change (rfirst, loaded once per kernel) and its first MFMA takes
      // the row norms as the accumulator input, so a tile starts without any register copy. There are at least
      // two groups (KS >= 9).
      f4 a0 = xg[0], a1 = xg[64], r1[RW], r0[RW];
#pragma unroll
      for (int it = 0; it < RW; ++it) r1[it] = rg[it][64];
#pragma unroll
      for (int it = 0; it < RW; ++it) acc[it] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0.x, rfirst[it].x, cq[it], 0, 0, 0);
#pragma unroll
      for (int it = 0; it < RW; ++it) acc[it] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0.y, rfirst[it].y, acc[it], 0, 0, 0);
#pragma unroll
      for (int it = 0; it < RW; ++it) acc[it] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0.z, rfirst[it].z, acc[it], 0, 0, 0);
#pragma unroll
      for (int it = 0; it < RW; ++it) acc[it] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0.w, rfirst[it].w, acc[it], 0, 0, 0);
      int g = 1;
      for (; g + 2 <= ks4; g += 2) {
        a0 = xg[(g + 1) * 64];
#pragma unroll
        for (int it = 0; it < RW; ++it) r0[it] = rg[it][(g + 1) * 64];
        four(a1, r1);
        const int gn = g + 2 < ks4 ? g + 2 : ks4 - 1;
        a1 = xg[gn * 64];
#pragma unroll
        for (int it = 0; it < RW; ++it) r1[it] = rg[it][gn * 64];
        four(a0, r0);
      }
      if (g < ks4) four(a1, r1);
#pragma unroll
      for (int k = 0; k < 3; ++k)
        if (k < kt) {
#pragma unroll
          for (int it = 0; it < RW; ++it) acc[it] = __builtin_amdgcn_mfma_f32_16x16x4f32(ta[k], tr[it][k], acc[it], 0, 0, 0);
        }
      f4 v[NB];
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) v[nb] = Vs[buf * vf4 + (jt * NB + nb) * 64 + lane];
      f4 e = {0.f, 0.f, 0.f, 0.f};
      if (EXTRA) e = Es[buf * ef4 + jt * 4 + q];
#pragma unroll
      for (int it = 0; it < RW; ++it) {
        f4 k;
        k.x = transform<KIND>(acc[it].x);
        k.y = transform<KIND>(acc[it].y);
        k.z = transform<KIND>(acc[it].z);
        k.w = transform<KIND>(acc[it].w);
        if constexpr (KIND == EGP_MATERN12) {      // exact k(x, x) on the diagonal of a square product (see kmm_kernel.h)
          if (XpRow == Xp && row_tile0 + it == (int64_t)st * jt_stage + jt) set_unit_diagonal(k, q, p);
        }
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          o[it][nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(k.x, v[nb].x, o[it][nb], 0, 0, 0);
          o[it][nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(k.y, v[nb].y, o[it][nb], 0, 0, 0);
          o[it][nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(k.z, v[nb].z, o[it][nb], 0, 0, 0);
          o[it][nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(k.w, v[nb].w, o[it][nb], 0, 0, 0);
        }
        if (EXTRA) {
          eacc[it] = __builtin_fmaf(k.x, e.x, eacc[it]);
          eacc[it] = __builtin_fmaf(k.y, e.y, eacc[it]);
          eacc[it] = __builtin_fmaf(k.z, e.z, eacc[it]);
          eacc[it] = __builtin_fmaf(k.w, e.w, eacc[it]);
        }
      }
    }
    if ((st - st_begin) % flush_stages == flush_stages - 1) fold();
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
  }
  fold();

  float* dst = Part + (int64_t)blockIdx.y * npad * TS;
#pragma unroll
  for (int it = 0; it < RW; ++it) {
    const int64_t row0 = (row_tile0 + it) * 16;
    if (cm) {
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
        *reinterpret_cast<f4*>(dst + (int64_t)(nb * 16 + p) * npad + row0 + q * 4) = o2[it][nb];
    } else {
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        float* r0 = dst + (row0 + q * 4) * TS + nb * 16 + p;
        r0[0 * TS] = o2[it][nb].x;
        r0[1 * TS] = o2[it][nb].y;
        r0[2 * TS] = o2[it][nb].z;
        r0[3 * TS] = o2[it][nb].w;
      }
    }
    if (EXTRA) {
      float s = eacc2[it];
      s += __shfl_xor(s, 16);
      s += __shfl_xor(s, 32);
      if (q == 0) {
        if (cm) dst[(int64_t)(16 * NB) * npad + row0 + p] = s;
        else dst[(row0 + p) * TS + 16 * NB] = s;
      }
    }
  }
}

struct WideShape { int rw, jt; size_t lds; };
// rows: 4 * rw * ks KB; a column stage: jt * (ks KB / 4 ... ) -- sized to stay within ~150 KB
WideShape wide_shape(int ks, int nb, int extra) {
  WideShape w;
  w.rw = ks <= 40 ? 2 : 1;
  const size_t rows = (size_t)4 * w.rw * ks * 256;
  const size_t budget = 150 * 1024 - rows;
  int jt = 4;
  while (jt > 1 && (size_t)2 * jt * ((size_t)ks * 256 + (size_t)nb * 1024 + (extra ? 64 : 0)) > budget) jt /= 2;
  w.jt = jt;
  w.lds = rows + (size_t)2 * jt * ((size_t)ks * 256 + (size_t)nb * 1024 + (extra ? 64 : 0));
  return w;
}

template <int RW, int KIND, int NB, int EXTRA>
int launch_wide_one(const Prepared& P, const Prepared& Q, const kmm_detail::Plan& pl, const WideShape& sh, const f4* Vp,
                    const float* Ep, float* Part, int cm, hipStream_t stream) {
  auto kern = kmm_kernel_wide<RW, KIND, NB, EXTRA>;
  EGP_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)sh.lds));
  hipLaunchKernelGGL(kern, dim3(pl.row_blocks, pl.splits), dim3(256), sh.lds, stream, Q.Xp, Q.nrm, P.Xp, Vp, Ep, Part,
                     Q.npad, P.d, P.ks, sh.jt, pl.stages_per_split, pl.stages_total, cm);
  EGP_HIP(hipGetLastError());
  return EGP_OK;
}

template <int RW, int KIND>
int launch_wide_cols(const Prepared& P, const Prepared& Q, const kmm_detail::Plan& pl, const WideShape& sh, int nb,
                     int extra, const f4* Vp, const float* Ep, float* Part, int cm, hipStream_t stream) {
  if (nb == 1 && !extra) return launch_wide_one<RW, KIND, 1, 0>(P, Q, pl, sh, Vp, Ep, Part, cm, stream);
  if (nb == 1 && extra) return launch_wide_one<RW, KIND, 1, 1>(P, Q, pl, sh, Vp, Ep, Part, cm, stream);
  if (nb == 2 && !extra) return launch_wide_one<RW, KIND, 2, 0>(P, Q, pl, sh, Vp, Ep, Part, cm, stream);
  return launch_wide_one<RW, KIND, 2, 1>(P, Q, pl, sh, Vp, Ep, Part, cm, stream);
}

template <int RW>
int launch_wide_kind(const Prepared& P, const Prepared& Q, const kmm_detail::Plan& pl, const WideShape& sh, int nb,
                     int extra, const f4* Vp, const float* Ep, float* Part, int cm, hipStream_t stream) {
  switch (P.kernel_type) {
    case EGP_RBF: return launch_wide_cols<RW, EGP_RBF>(P, Q, pl, sh, nb, extra, Vp, Ep, Part, cm, stream);
    case EGP_MATERN32: return launch_wide_cols<RW, EGP_MATERN32>(P, Q, pl, sh, nb, extra, Vp, Ep, Part, cm, stream);
    case EGP_MATERN12: return launch_wide_cols<RW, EGP_MATERN12>(P, Q, pl, sh, nb, extra, Vp, Ep, Part, cm, stream);
    default: return launch_wide_cols<RW, EGP_MATERN52>(P, Q, pl, sh, nb, extra, Vp, Ep, Part, cm, stream);
  }
}

}  // namespace

namespace kmm_detail {

Plan make_plan_wide(int64_t npad_rows, int64_t npad_cols, int ks, int nb, int extra) {
  const WideShape sh = wide_shape(ks, nb, extra);
  Plan pl;
  pl.big = true;
  pl.row_blocks = (int)(npad_rows / (64 * sh.rw));
  pl.stages_total = (int)(npad_cols / (16 * sh.jt));
  int want = 1024 / pl.row_blocks;
  if (want < 1) want = 1;
  if (want > pl.stages_total) want = pl.stages_total;
  if (want > 64) want = 64;
  pl.stages_per_split = (pl.stages_total + want - 1) / want;
  pl.splits = (pl.stages_total + pl.stages_per_split - 1) / pl.stages_per_split;
  return pl;
}

int launch_wide(const Prepared& P, const Prepared& Q, const Plan& pl, int nb, int extra, const f4* Vp, const float* Ep,
                float* Part, int cm, hipStream_t stream) {
  const WideShape sh = wide_shape(P.ks, nb, extra);
  ProfScope prof(kProfKmm, stream);
  if (sh.rw == 2) return launch_wide_kind<2>(P, Q, pl, sh, nb, extra, Vp, Ep, Part, cm, stream);
  return launch_wide_kind<1>(P, Q, pl, sh, nb, extra, Vp, Ep, Part, cm, stream);
}

}  // namespace kmm_detail
}  // namespace egp
