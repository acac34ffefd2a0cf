// Bilinear forms with the kernel derivatives for inputs of more than 31 dimensions:
//   out[k] = sum_ij S_ij dK_ij/dl_k  (k < d),   out[d] = sum_ij S_ij K_ij / s,   S = (A diag w) B^T.
//
// Paper, Eq. 2 (every term of the marginal-likelihood gradient is such a form, see kmm_bilinear.hip). With d in
// the hundreds the per-lengthscale VALU work of the d <= 31 kernel (three operations per entry and lengthscale)
// would dwarf the MFMA work, so the squared difference is expanded and contracted on the matrix cores instead.
// The weight (x_ik - x_jk)^2 is symmetric in (i, j), so S may be replaced by its symmetric part
// S' = (S + S^T)/2 = [A w/2 | B w/2] [B | A]^T (twice the columns). With W_ij = S'_ij h_ij symmetric,
//   sum_ij W_ij (x~_ik - x~_jk)^2 = 2 sum_i x~_ik ( x~_ik r_i - Y_ik ),   Y = W X~,  r = W 1,
// and Y, r come from one more MFMA contraction of the tile with the column points [X~ | 1] laid out with the
// features as columns (the layout of a right-hand side). Per 16 x 16 tile: KS distance steps, ceil(2t/4) steps
// for S'^T, 4 ceil((d+1)/16) steps for [Y | r]; VALU work is the transform only. The norm expansion in the
// derivative weight is acceptable here because the points are centred and lengthscales at these d are of the
// order of the data's spread (|x~| is of the order of the differences).
//
// Row operands (scaled points and the A side of S') live in LDS for the whole column sweep; column tiles stream
// through a single- or double-buffered stage of one tile. The [Y | r] accumulators (4 NBF registers per row
// tile) stay in registers across the sweep, which is why NBF is a template parameter (d is rounded up to the
// next instantiated block count with zero features).

#include <math.h>

#include <vector>

#include "bilinear_detail.h"

namespace egp {

namespace {

using bilinear_detail::f4;
using bilinear_detail::hg;

constexpr int kWLd = EGP_D_WIDE_MAX + 1;      // leading dimension of the per-block partial vectors
constexpr size_t kLdsBudget = 158 * 1024;

// [A w/2 | B w/2] (a_side) or [B | A] packed per 16-point tile as [tg][64][4]: step s = 4 g + e, lane (q, p)
// holds column c = 4 s + q of point 16 tile + p (zero beyond 2 t columns and beyond n)
__global__ __launch_bounds__(256) void pack_sym(const float* __restrict__ A, const float* __restrict__ B, int64_t n,
                                                int64_t npad, int t, int tg, const float* __restrict__ wcol,
                                                int a_side, float* __restrict__ out) {
  const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int per = tg * 256;
  if (g >= (npad >> 4) * per) return;
  const int e = (int)(g % per);
  const int64_t tile = g / per;
  const int lane = (e >> 2) & 63;
  const int s = (e >> 8) * 4 + (e & 3);
  const int q = lane >> 4, p = lane & 15;
  const int c = 4 * s + q;
  const int64_t i = tile * 16 + p;
  float v = 0.f;
  if (i < n && c < 2 * t) {
    const int cc = c < t ? c : c - t;
    const bool from_a = (c < t) == (a_side != 0);
    v = (from_a ? A : B)[i * t + cc];
    if (a_side) v *= 0.5f * (wcol ? wcol[cc] : 1.0f);
  }
  out[g] = v;
}

// Scaled points with the features as columns: Xf[tile][fb][lane (q,p)] = x~[16 tile + 4q + r][16 fb + p], r = 0..3;
// feature slot d is 1 for real points (its column of Y is the row sum r), later slots are 0
__global__ __launch_bounds__(256) void pack_feat(const float* __restrict__ Xp, int64_t n, int64_t npad, int d, int ks,
                                                 int nbf, f4* __restrict__ Xf) {
  const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (g >= (npad >> 4) * nbf * 64) return;
  const int lane = (int)(g & 63);
  const int64_t rest = g >> 6;
  const int fb = (int)(rest % nbf);
  const int64_t tile = rest / nbf;
  const int q = lane >> 4, p = lane & 15;
  const int f = 16 * fb + p;
  const float* base = Xp + tile * ks * 64;
  float v[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int pp = 4 * q + r;
    if (f < d) v[r] = base[xp_offset(ks, f, pp)];
    else v[r] = (f == d && tile * 16 + pp < n) ? 1.0f : 0.f;
  }
  Xf[g] = (f4){v[0], v[1], v[2], v[3]};
}

template <int RW, int NBF, int KIND>
__global__ __launch_bounds__(256) void bilinear_wide_kernel(const float* __restrict__ Xp, const float* __restrict__ nrm,
                                                            const float* __restrict__ Ap, const float* __restrict__ Bp,
                                                            const f4* __restrict__ Xf, float* __restrict__ part,
                                                            int64_t npad, int d, int ks, int tg, int nbuf,
                                                            int tiles_per_split, int tiles_total) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int nw = blockDim.x >> 6;
  const int rowf = ks * 64 + tg * 256;                 // floats of one row-tile record: x part, then A part
  const int stagef = ks * 64 + tg * 256 + NBF * 256;   // floats of one column-tile stage: x, B part, features
  float* Rs = reinterpret_cast<float*>(smem);          // [nw * RW][rowf]
  float* St = Rs + nw * RW * rowf;                     // [nbuf][stagef]

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int q = lane >> 4, p = lane & 15;
  const int64_t row_tile0 = ((int64_t)blockIdx.x * nw + wave) * RW;
  const int ds = d >> 2, dq = d & 3;
  const int ks4 = ks >> 2, kt = ks & 3;

  for (int it = 0; it < RW; ++it) {
    const float* src = Xp + (row_tile0 + it) * ks * 64;
    float* dst = Rs + (wave * RW + it) * rowf;
    for (int e = lane; e < ks * 64; e += 64) {
      int s_, l_;
      if (e < ks4 * 256) {
        s_ = (e >> 8) * 4 + (e & 3);
        l_ = (e >> 2) & 63;
      } else {
        s_ = e >> 6;
        l_ = e & 63;
      }
      dst[e] = (s_ == ds && (l_ >> 4) == dq) ? 1.0f : -2.0f * src[e];
    }
    const float* asrc = Ap + (row_tile0 + it) * tg * 256;
    for (int e = lane; e < tg * 256; e += 64) dst[ks * 64 + e] = asrc[e];
  }
  f4 cq[RW], yacc[RW][NBF];
  float acc_s = 0.f;
#pragma unroll
  for (int it = 0; it < RW; ++it) {
    const float ni = nrm[(row_tile0 + it) * 16 + p];
    cq[it] = (f4){ni, ni, ni, ni};
#pragma unroll
    for (int fb = 0; fb < NBF; ++fb) yacc[it][fb] = (f4){0.f, 0.f, 0.f, 0.f};
  }

  const int ct_begin = blockIdx.y * tiles_per_split;
  int ct_end = ct_begin + tiles_per_split;
  if (ct_end > tiles_total) ct_end = tiles_total;
  const f4* Xg = reinterpret_cast<const f4*>(Xp);
  const f4* Bg = reinterpret_cast<const f4*>(Bp);
  const int xf4 = ks * 16, bf4 = tg * 64, ff4 = NBF * 64;
  auto issue = [&](int ct, int buf) {
    f4* s4 = reinterpret_cast<f4*>(St + buf * stagef);
    for (int k = wave * 64; k < xf4; k += nw * 64)
      if (k + lane < xf4)     // xf4 is a multiple of 16, not of 64
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Xg + (int64_t)ct * xf4 + k + lane),
                                         (__attribute__((address_space(3))) void*)(s4 + k), 16, 0, 0);
    for (int k = wave * 64; k < bf4; k += nw * 64)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Bg + (int64_t)ct * bf4 + k + lane),
                                       (__attribute__((address_space(3))) void*)(s4 + xf4 + k), 16, 0, 0);
    for (int k = wave * 64; k < ff4; k += nw * 64)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Xf + (int64_t)ct * ff4 + k + lane),
                                       (__attribute__((address_space(3))) void*)(s4 + xf4 + bf4 + k), 16, 0, 0);
  };
  if (ct_begin < ct_end) issue(ct_begin, 0);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();

  f4 rfirst[RW];      // row operands of the first group of four k-steps: resident in registers
#pragma unroll
  for (int it = 0; it < RW; ++it) rfirst[it] = reinterpret_cast<const f4*>(Rs + (wave * RW + it) * rowf)[lane];

  for (int ct = ct_begin; ct < ct_end; ++ct) {
    const int buf = nbuf == 2 ? ((ct - ct_begin) & 1) : 0;
    const bool more = ct + 1 < ct_end;
    if (nbuf == 2 && more) issue(ct + 1, buf ^ 1);
    const float* xt = St + buf * stagef;
    const f4* xg = reinterpret_cast<const f4*>(xt) + lane;
    const f4* bg = reinterpret_cast<const f4*>(xt + ks * 64) + lane;
    const f4* fg = reinterpret_cast<const f4*>(xt + ks * 64 + tg * 256) + lane;
    const f4* rg[RW];
    const f4* ag[RW];
    f4 acc[RW], sv[RW];
#pragma unroll
    for (int it = 0; it < RW; ++it) {
      sv[it] = (f4){0.f, 0.f, 0.f, 0.f};
      rg[it] = reinterpret_cast<const f4*>(Rs + (wave * RW + it) * rowf) + lane;
      ag[it] = reinterpret_cast<const f4*>(Rs + (wave * RW + it) * rowf + ks * 64) + lane;
    }
    // ---- squared distances, transposed: acc[j][i] ----
    float ta[3], tr[RW][3];
#pragma unroll
    for (int k = 0; k < 3; ++k) {
      const int sk = ks4 * 4 + k < ks ? ks4 * 4 + k : ks - 1;
      ta[k] = xt[sk * 64 + lane];
#pragma unroll
      for (int it = 0; it < RW; ++it) tr[it][k] = Rs[(wave * RW + it) * rowf + sk * 64 + lane];
    }
    auto four = [&](f4 (&dstacc)[RW], const f4& a, const f4 (&r)[RW]) {
#pragma unroll
      for (int it = 0; it < RW; ++it) dstacc[it] = __builtin_amdgcn_mfma_f32_16x16x4f32(a.x, r[it].x, dstacc[it], 0, 0, 0);
#pragma unroll
      for (int it = 0; it < RW; ++it) dstacc[it] = __builtin_amdgcn_mfma_f32_16x16x4f32(a.y, r[it].y, dstacc[it], 0, 0, 0);
#pragma unroll
      for (int it = 0; it < RW; ++it) dstacc[it] = __builtin_amdgcn_mfma_f32_16x16x4f32(a.z, r[it].z, dstacc[it], 0, 0, 0);
#pragma unroll
      for (int it = 0; it < RW; ++it) dstacc[it] = __builtin_amdgcn_mfma_f32_16x16x4f32(a.w, r[it].w, dstacc[it], 0, 0, 0);
    };
    {
      // group 0 peeled: resident row operands, the row norms enter as the first MFMA's accumulator input
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
        four(acc, a1, r1);
        const int gn = g + 2 < ks4 ? g + 2 : ks4 - 1;
        a1 = xg[gn * 64];
#pragma unroll
        for (int it = 0; it < RW; ++it) r1[it] = rg[it][gn * 64];
        four(acc, a0, r0);
      }
      if (g < ks4) four(acc, a1, r1);
#pragma unroll
      for (int k = 0; k < 3; ++k)
        if (k < kt) {
#pragma unroll
          for (int it = 0; it < RW; ++it) acc[it] = __builtin_amdgcn_mfma_f32_16x16x4f32(ta[k], tr[it][k], acc[it], 0, 0, 0);
        }
    }
    // ---- S'^T[j][i] in the same layout ----
    for (int g = 0; g < tg; ++g) {
      const f4 b = bg[g * 64];
      f4 a[RW];
#pragma unroll
      for (int it = 0; it < RW; ++it) a[it] = ag[it][g * 64];
      four(sv, b, a);
    }
    // ---- W = S' h; outputscale term sum S' g ----
    f4 w[RW];
#pragma unroll
    for (int it = 0; it < RW; ++it) {
      float g0, g1, g2, g3;
      float h0 = hg<KIND>(acc[it].x, &g0), h1 = hg<KIND>(acc[it].y, &g1);
      float h2 = hg<KIND>(acc[it].z, &g2), h3 = hg<KIND>(acc[it].w, &g3);
      if constexpr (KIND == EGP_MATERN12) {
        // A point against itself: the expanded squared difference is rounding noise, not 0, and h = exp(-r)/r is
        // huge at a computed r ~ 3e-4; the entry does not depend on the lengthscales, so its weight is 0.
        if (row_tile0 + it == ct) {
          const int r = p - 4 * q;
          if (r == 0) h0 = 0.f;
          if (r == 1) h1 = 0.f;
          if (r == 2) h2 = 0.f;
          if (r == 3) h3 = 0.f;
        }
      }
      acc_s = __builtin_fmaf(sv[it].x, g0, acc_s);
      acc_s = __builtin_fmaf(sv[it].y, g1, acc_s);
      acc_s = __builtin_fmaf(sv[it].z, g2, acc_s);
      acc_s = __builtin_fmaf(sv[it].w, g3, acc_s);
      w[it] = (f4){sv[it].x * h0, sv[it].y * h1, sv[it].z * h2, sv[it].w * h3};
    }
    // ---- [Y | r] += W [X~ | 1] ----
#pragma unroll
    for (int fb = 0; fb < NBF; ++fb) {
      const f4 xf = fg[fb * 64];
#pragma unroll
      for (int it = 0; it < RW; ++it) {
        yacc[it][fb] = __builtin_amdgcn_mfma_f32_16x16x4f32(w[it].x, xf.x, yacc[it][fb], 0, 0, 0);
        yacc[it][fb] = __builtin_amdgcn_mfma_f32_16x16x4f32(w[it].y, xf.y, yacc[it][fb], 0, 0, 0);
        yacc[it][fb] = __builtin_amdgcn_mfma_f32_16x16x4f32(w[it].z, xf.z, yacc[it][fb], 0, 0, 0);
        yacc[it][fb] = __builtin_amdgcn_mfma_f32_16x16x4f32(w[it].w, xf.w, yacc[it][fb], 0, 0, 0);
      }
    }
    if (nbuf == 1 && more) {
      __syncthreads();          // every wave has finished reading the only buffer
      issue(ct + 1, 0);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
  }

  // ---- per feature f = 16 fb + p: sum over this wave's rows of x~_if (x~_if r_i - Y_if) ----
  float gsum[NBF];
#pragma unroll
  for (int fb = 0; fb < NBF; ++fb) gsum[fb] = 0.f;
  const int fbd = d >> 4, src_lane = q * 16 + (d & 15);
#pragma unroll
  for (int it = 0; it < RW; ++it) {
    f4 ysel = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int fb = 0; fb < NBF; ++fb)
      if (fb == fbd) ysel = yacc[it][fb];
    f4 ri;      // r_i of the four rows i = 4q + r of this lane group
    ri.x = __shfl(ysel.x, src_lane);
    ri.y = __shfl(ysel.y, src_lane);
    ri.z = __shfl(ysel.z, src_lane);
    ri.w = __shfl(ysel.w, src_lane);
#pragma unroll
    for (int fb = 0; fb < NBF; ++fb) {
      const f4 x = Xf[((row_tile0 + it) * NBF + fb) * 64 + lane];
      const f4 y = yacc[it][fb];
      float a = gsum[fb];
      a = __builtin_fmaf(x.x, __builtin_fmaf(x.x, ri.x, -y.x), a);
      a = __builtin_fmaf(x.y, __builtin_fmaf(x.y, ri.y, -y.y), a);
      a = __builtin_fmaf(x.z, __builtin_fmaf(x.z, ri.z, -y.z), a);
      a = __builtin_fmaf(x.w, __builtin_fmaf(x.w, ri.w, -y.w), a);
      gsum[fb] = a;
    }
  }
  // the stage is free now (the loop ended with a barrier): reuse it for the cross-wave sums
  float* red = St;                       // [nw][NBF * 16 + 1]
  constexpr int RL = NBF * 16 + 1;
#pragma unroll
  for (int fb = 0; fb < NBF; ++fb) {
    float v = gsum[fb];
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 32);
    if (q == 0) red[wave * RL + fb * 16 + p] = v;
  }
  {
    float v = acc_s;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
    if (lane == 0) red[wave * RL + NBF * 16] = v;
  }
  __syncthreads();
  const int64_t blk = (int64_t)blockIdx.y * gridDim.x + blockIdx.x;
  for (int f = tid; f <= d; f += blockDim.x) {
    const int slot = f < d ? f : NBF * 16;
    float v = 0.f;
    for (int wv = 0; wv < nw; ++wv) v += red[wv * RL + slot];
    part[blk * kWLd + f] = v;
  }
}

struct WPlan {
  int nbf, rw, nw, nbuf, tg;
  size_t lds;
  int row_blocks, splits, tiles_per_split, tiles_total;
};

constexpr int kBuckets[] = {3, 4, 5, 6, 7, 8, 10, 12, 16, 20, 25};

WPlan wide_plan(int64_t npad, int d, int t) {
  WPlan pl;
  const int ks = ksteps_for(d);
  const int need = (d + 1 + 15) / 16;
  pl.nbf = 25;
  for (int b : kBuckets)
    if (b >= need) {
      pl.nbf = b;
      break;
    }
  pl.rw = pl.nbf <= 12 ? 2 : 1;
  pl.tg = ((2 * t + 3) / 4 + 3) / 4;
  const size_t rowb = (size_t)(ks * 64 + pl.tg * 256) * 4;
  const size_t stageb = (size_t)(ks * 64 + pl.tg * 256 + pl.nbf * 256) * 4;
  pl.nw = 4;
  if (4 * pl.rw * rowb + stageb > kLdsBudget && pl.rw == 2) pl.rw = 1;
  if (4 * pl.rw * rowb + stageb > kLdsBudget) pl.nw = 2;
  pl.nbuf = (size_t)pl.nw * pl.rw * rowb + 2 * stageb <= kLdsBudget ? 2 : 1;
  pl.lds = (size_t)pl.nw * pl.rw * rowb + pl.nbuf * stageb;
  pl.row_blocks = (int)(npad / (16 * pl.nw * pl.rw));
  pl.tiles_total = (int)(npad / 16);
  int want = 1024 / pl.row_blocks;
  if (want < 1) want = 1;
  if (want > pl.tiles_total) want = pl.tiles_total;
  if (want > 64) want = 64;
  pl.tiles_per_split = (pl.tiles_total + want - 1) / want;
  pl.splits = (pl.tiles_total + pl.tiles_per_split - 1) / pl.tiles_per_split;
  return pl;
}

template <int RW, int NBF, int KIND>
int launch_one(const Prepared& P, const WPlan& pl, const float* Ap, const float* Bp, const f4* Xf, float* part,
               hipStream_t stream) {
  auto kern = bilinear_wide_kernel<RW, NBF, KIND>;
  EGP_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)pl.lds));
  hipLaunchKernelGGL(kern, dim3(pl.row_blocks, pl.splits), dim3(64 * pl.nw), pl.lds, stream, P.Xp, P.nrm, Ap, Bp, Xf,
                     part, P.npad, P.d, P.ks, pl.tg, pl.nbuf, pl.tiles_per_split, pl.tiles_total);
  EGP_HIP(hipGetLastError());
  return EGP_OK;
}

template <int NBF, int KIND>
int launch_rw(const Prepared& P, const WPlan& pl, const float* Ap, const float* Bp, const f4* Xf, float* part,
              hipStream_t stream) {
  if constexpr (NBF <= 12) {
    if (pl.rw == 2) return launch_one<2, NBF, KIND>(P, pl, Ap, Bp, Xf, part, stream);
  }
  return launch_one<1, NBF, KIND>(P, pl, Ap, Bp, Xf, part, stream);
}

template <int KIND>
int launch_nbf(const Prepared& P, const WPlan& pl, const float* Ap, const float* Bp, const f4* Xf, float* part,
               hipStream_t stream) {
  switch (pl.nbf) {
    case 3: return launch_rw<3, KIND>(P, pl, Ap, Bp, Xf, part, stream);
    case 4: return launch_rw<4, KIND>(P, pl, Ap, Bp, Xf, part, stream);
    case 5: return launch_rw<5, KIND>(P, pl, Ap, Bp, Xf, part, stream);
    case 6: return launch_rw<6, KIND>(P, pl, Ap, Bp, Xf, part, stream);
    case 7: return launch_rw<7, KIND>(P, pl, Ap, Bp, Xf, part, stream);
    case 8: return launch_rw<8, KIND>(P, pl, Ap, Bp, Xf, part, stream);
    case 10: return launch_rw<10, KIND>(P, pl, Ap, Bp, Xf, part, stream);
    case 12: return launch_rw<12, KIND>(P, pl, Ap, Bp, Xf, part, stream);
    case 16: return launch_rw<16, KIND>(P, pl, Ap, Bp, Xf, part, stream);
    case 20: return launch_rw<20, KIND>(P, pl, Ap, Bp, Xf, part, stream);
    default: return launch_rw<25, KIND>(P, pl, Ap, Bp, Xf, part, stream);
  }
}

struct WWs { size_t ab, xf, part, wdev; };
WWs wide_ws(int64_t npad, const WPlan& pl) {
  WWs w;
  w.ab = round_up((size_t)(npad >> 4) * pl.tg * 256 * sizeof(float), 256);
  w.xf = round_up((size_t)(npad >> 4) * pl.nbf * 64 * sizeof(f4), 256);
  w.part = round_up((size_t)pl.row_blocks * pl.splits * kWLd * sizeof(float), 256);
  w.wdev = 256;
  return w;
}

}  // namespace

namespace bilinear_detail {

size_t bilinear_wide_ws_bytes(int64_t n, int d, int t) {
  const int64_t npad = padded_points(n);
  const WWs w = wide_ws(npad, wide_plan(npad, d, t));
  return 2 * w.ab + w.xf + w.part + w.wdev;
}

int bilinear_wide_core(const Prepared& P, const egp_hyper_t* h, const float* A, const float* B, int t,
                       const float* wcol, double* out, void* ws2, hipStream_t stream) {
  if (t > 36) return fail(EGP_ERR_ARG, "bilinear forms support t <= 36 (got %d)", t);
  const int64_t npad = P.npad;
  const WPlan pl = wide_plan(npad, P.d, t);
  if (pl.lds > 160 * 1024) return fail(EGP_ERR_ARG, "d = %d, t = %d: the bilinear kernel's LDS need exceeds 160 KB", P.d, t);
  const WWs lay = wide_ws(npad, pl);
  char* w = static_cast<char*>(ws2);
  float* Ap = reinterpret_cast<float*>(w);
  float* Bp = reinterpret_cast<float*>(w + lay.ab);
  f4* Xf = reinterpret_cast<f4*>(w + 2 * lay.ab);
  float* part = reinterpret_cast<float*>(w + 2 * lay.ab + lay.xf);
  float* wdev = reinterpret_cast<float*>(w + 2 * lay.ab + lay.xf + lay.part);
  if (wcol) EGP_HIP(hipMemcpyAsync(wdev, wcol, sizeof(float) * t, hipMemcpyHostToDevice, stream));
  {
    ProfScope prof(kProfPack, stream);
    const int64_t tot_ab = (npad >> 4) * pl.tg * 256;
    const unsigned b1 = (unsigned)((tot_ab + 255) / 256);
    hipLaunchKernelGGL(pack_sym, dim3(b1), dim3(256), 0, stream, A, B, P.n, npad, t, pl.tg, wcol ? wdev : nullptr, 1, Ap);
    hipLaunchKernelGGL(pack_sym, dim3(b1), dim3(256), 0, stream, A, B, P.n, npad, t, pl.tg,
                       static_cast<const float*>(nullptr), 0, Bp);
    const int64_t tot_f = (npad >> 4) * pl.nbf * 64;
    hipLaunchKernelGGL(pack_feat, dim3((unsigned)((tot_f + 255) / 256)), dim3(256), 0, stream, P.Xp, P.n, npad, P.d,
                       P.ks, pl.nbf, Xf);
    EGP_HIP(hipGetLastError());
  }
  int rc;
  {
    ProfScope prof(kProfGrad, stream);
    switch (P.kernel_type) {
      case EGP_RBF: rc = launch_nbf<EGP_RBF>(P, pl, Ap, Bp, Xf, part, stream); break;
      case EGP_MATERN32: rc = launch_nbf<EGP_MATERN32>(P, pl, Ap, Bp, Xf, part, stream); break;
      case EGP_MATERN12: rc = launch_nbf<EGP_MATERN12>(P, pl, Ap, Bp, Xf, part, stream); break;
      default: rc = launch_nbf<EGP_MATERN52>(P, pl, Ap, Bp, Xf, part, stream);
    }
  }
  if (rc != EGP_OK) return rc;
  const int64_t nblk = (int64_t)pl.row_blocks * pl.splits;
  std::vector<float> hp((size_t)nblk * kWLd);
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
    for (int64_t bidx = 0; bidx < nblk; ++bidx) s += (double)hp[(size_t)bidx * kWLd + k];
    // the kernel leaves half of sum W (x~_ik - x~_jk)^2 per lengthscale; slot d: sum S g = sum S K / s
    out[k] = k < P.d ? 2.0 * s * (double)h->outputscale * hfac / ((double)h->lengthscales[k] * c2) : s;
  }
  return EGP_OK;
}

}  // namespace bilinear_detail
}  // namespace egp
