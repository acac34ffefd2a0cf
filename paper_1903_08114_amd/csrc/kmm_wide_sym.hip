// Symmetric variant of the fused multiply for inputs of more than 31 dimensions (square products, 16 or 17
// right-hand sides): kmm_wide.hip's tile loop (row operands in LDS, grouped k-steps) with kmm_sym.hip's two-sided use of every
// tile off the block diagonal. With KS distance steps per tile against 4 contraction steps per side, forming a tile
// once instead of twice saves the larger share the larger d is (d = 90: 23 + 8 MFMA per tile pair against 54).
//
// A wave works on its RW row tiles of one column tile at a time, so the software pipeline runs over the column
// tiles: the tiles of column tile jt go to the wave's LDS patches (two sets, alternating), are read back transposed
// at the start of column tile jt + 1 and contracted with the packed V of the wave's own rows after that tile's
// distance steps.
#include "kmm_kernel.h"

namespace egp {
namespace kmm_detail {

namespace {

constexpr int kPatchW = 280;      // floats of one transposition patch (layout: kmm_sym.hip)

// Sum over the 16 lanes of a DPP row (all lanes receive it), as in kmm_sym.hip.
__device__ __forceinline__ float row_sum16w(float x) {
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xf, 0xf, false));
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xf, 0xf, false));
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x141, 0xf, 0xf, false));
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x140, 0xf, 0xf, false));
  return x;
}

template <int RW, int KIND, int EXTRA>
__global__ __launch_bounds__(256) void kmm_kernel_wide_sym(const float* __restrict__ Xp, const float* __restrict__ nrm,
                                                           const f4* __restrict__ Vp, const float* __restrict__ Ep,
                                                           float* __restrict__ Part, int64_t npad, int d, int ks,
                                                           int jt_stage, int nblk, int stages_per_split, int cm) {
  constexpr int TS = 16 + EXTRA;
  extern __shared__ __align__(16) unsigned char smem[];
  // rows [4 RW][ks][64] | 2 x column stage [jt_stage][ks][64] | 2 x V stage [jt_stage][64] f4 |
  // patches [4 waves][2][RW][kPatchW] | column-side sums [4 waves][jt_stage][64] f4 |
  // with a 17th column: 2 x its stage [jt_stage][4] f4 | its column-side sums [4 waves][jt_stage][64] f4
  float* Rs = reinterpret_cast<float*>(smem);
  float* Xs = Rs + 4 * RW * ks * 64;
  f4* Vs = reinterpret_cast<f4*>(Xs + 2 * jt_stage * ks * 64);
  float* Ts = reinterpret_cast<float*>(Vs + 2 * jt_stage * 64);
  f4* CJ = reinterpret_cast<f4*>(Ts + 4 * 2 * RW * kPatchW);
  f4* Es = CJ + 4 * jt_stage * 64;
  f4* CJE = Es + 2 * jt_stage * 4;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int q = lane >> 4, p = lane & 15;
  const int bi = (nblk & 7) == 0 ? (int)(blockIdx.x & 7) * (nblk >> 3) + (int)(blockIdx.x >> 3) : (int)blockIdx.x;
  const int sb = 4 * RW / jt_stage;            // stages per block of 64 RW points
  const int half = nblk >> 1;
  const int stages_all = (half + 1) * sb;
  const int s_total = nblk * sb;
  const int64_t row_tile0 = ((int64_t)bi * 4 + wave) * RW;
  const int ds = d >> 2, dq = d & 3;
  const int ks4 = ks >> 2, kt = ks & 3;

  for (int it = 0; it < RW; ++it) {
    const float* src = Xp + (row_tile0 + it) * ks * 64;
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
  f4 cq[RW], o[RW], o2[RW], vrow[RW];
  float eacc[RW], eacc2[RW], erow[RW];
#pragma unroll
  for (int it = 0; it < RW; ++it) {
    const float ni = nrm[(row_tile0 + it) * 16 + p];
    cq[it] = (f4){ni, ni, ni, ni};
    o[it] = (f4){0.f, 0.f, 0.f, 0.f};
    o2[it] = (f4){0.f, 0.f, 0.f, 0.f};
    vrow[it] = Vp[(row_tile0 + it) * 64 + lane];
    eacc[it] = 0.f;
    eacc2[it] = 0.f;
    erow[it] = EXTRA ? Ep[(row_tile0 + it) * 16 + p] : 0.f;
  }
  auto fold = [&]() {
#pragma unroll
    for (int it = 0; it < RW; ++it) {
      o2[it] += o[it];
      o[it] = (f4){0.f, 0.f, 0.f, 0.f};
      if (EXTRA) {
        eacc2[it] += eacc[it];
        eacc[it] = 0.f;
      }
    }
  };
  const int flush_stages = 256 / jt_stage;

  float* patch = Ts + wave * 2 * RW * kPatchW;      // [2][RW][kPatchW]
  const int woff = 4 * (18 * q + ((p >> 2) & 1) + 8 * (p >> 3) + 2 * (p & 3));
  const int roff = 72 * (p >> 2) + 4 * (q & 1) + 32 * (q >> 1) + (p & 3);

  const int k_begin = blockIdx.y * stages_per_split;
  int k_end = k_begin + stages_per_split;
  if (k_end > stages_all) k_end = stages_all;
  const int xf4 = jt_stage * ks * 16, vf4 = jt_stage * 64, ef4 = jt_stage * 4;
  const f4* Xg = reinterpret_cast<const f4*>(Xp);
  const f4* Eg = reinterpret_cast<const f4*>(Ep);
  auto abs_stage = [&](int k) {
    int st = bi * sb + k;
    return st >= s_total ? st - s_total : st;
  };
  auto is_dual = [&](int k) {
    const int delta = k / sb;
    return delta != 0 && !(delta == half && (nblk & 1) == 0);
  };
  auto issue = [&](int st, int buf) {
    const int64_t xoff = (int64_t)st * xf4, voff = (int64_t)st * vf4;
    f4* xs4 = reinterpret_cast<f4*>(Xs + buf * jt_stage * ks * 64);
    for (int k = wave * 64; k < xf4; k += 256)
      if (k + lane < xf4)      // xf4 is a multiple of 16, not of 64
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Xg + xoff + k + lane),
                                         (__attribute__((address_space(3))) void*)(xs4 + k), 16, 0, 0);
    for (int k = wave * 64; k < vf4; k += 256)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Vp + voff + k + lane),
                                       (__attribute__((address_space(3))) void*)(Vs + buf * vf4 + k), 16, 0, 0);
    if (EXTRA && tid < ef4)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Eg + (int64_t)st * ef4 + tid),
                                       (__attribute__((address_space(3))) void*)(Es + buf * ef4), 16, 0, 0);
  };
  // column-side sums leave as 64-bit fixed-point atomic adds (colside_add, kmm_kernel.h): order-independent
  __shared__ float cscale[18];
  long long* slab = reinterpret_cast<long long*>(Part + (int64_t)gridDim.y * npad * TS);
  if (tid < TS)
    cscale[tid] = colside_scale(colside_exp(reinterpret_cast<const unsigned*>(slab + npad * TS)[tid]));
  auto flush = [&](int st) {
    if (cm) {
      const int c = tid >> 4, jrow = tid & 15;
      const float* cf = reinterpret_cast<const float*>(CJ);
      const int off = ((jrow >> 2) * 16 + c) * 4 + (jrow & 3);
      const float sc = cscale[c];
      for (int jt = 0; jt < jt_stage; ++jt) {
        const float v = (cf[(0 * jt_stage + jt) * 256 + off] + cf[(1 * jt_stage + jt) * 256 + off]) +
                        (cf[(2 * jt_stage + jt) * 256 + off] + cf[(3 * jt_stage + jt) * 256 + off]);
        colside_add(slab + (int64_t)c * npad + ((int64_t)st * jt_stage + jt) * 16 + jrow, v, sc);
      }
    } else {
      for (int e = tid; e < jt_stage * 64; e += 256) {      // (tile, lane)
        const int jt = e >> 6, l = e & 63;
        f4 v = CJ[(0 * jt_stage + jt) * 64 + l];
        v += CJ[(1 * jt_stage + jt) * 64 + l];
        v += CJ[(2 * jt_stage + jt) * 64 + l];
        v += CJ[(3 * jt_stage + jt) * 64 + l];
        long long* dst = slab + (((int64_t)st * jt_stage + jt) * 16 + 4 * (l >> 4)) * TS + (l & 15);
        const float sc = cscale[l & 15];
        colside_add(dst + 0 * TS, v.x, sc);
        colside_add(dst + 1 * TS, v.y, sc);
        colside_add(dst + 2 * TS, v.z, sc);
        colside_add(dst + 3 * TS, v.w, sc);
      }
    }
    if (EXTRA) {
      // per tile: sum over the four waves, then over the 16 lanes of the DPP row (point index p); lanes p < 4 add
      // component p
      for (int jt = wave; jt < jt_stage; jt += 4) {      // wave-uniform
        f4 v = CJE[(0 * jt_stage + jt) * 64 + lane];
        v += CJE[(1 * jt_stage + jt) * 64 + lane];
        v += CJE[(2 * jt_stage + jt) * 64 + lane];
        v += CJE[(3 * jt_stage + jt) * 64 + lane];
        v.x = row_sum16w(v.x);
        v.y = row_sum16w(v.y);
        v.z = row_sum16w(v.z);
        v.w = row_sum16w(v.w);
        const int r = p & 3;
        float add = r == 0 ? v.x : (r == 1 ? v.y : (r == 2 ? v.z : v.w));
        const int col = 16;
        const int64_t j = ((int64_t)st * jt_stage + jt) * 16 + 4 * q + r;
        if (p < 4) colside_add(cm ? slab + (int64_t)col * npad + j : slab + j * TS + col, add, cscale[16]);
      }
    }
  };

  if (k_begin < k_end) issue(abs_stage(k_begin), 0);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();

  f4 rfirst[RW];
#pragma unroll
  for (int it = 0; it < RW; ++it) rfirst[it] = reinterpret_cast<const f4*>(Rs + (wave * RW + it) * ks * 64)[lane];

  // squared distances of one column tile against the wave's RW row tiles (transposed accumulator layout), as in
  // kmm_kernel_wide: left-over steps loaded first, groups of four steps ping-pong, first group from registers
  auto distances = [&](const float* xt, f4 (&acc)[RW]) {
    const f4* xg = reinterpret_cast<const f4*>(xt) + lane;
    const f4* rg[RW];
#pragma unroll
    for (int it = 0; it < RW; ++it) rg[it] = reinterpret_cast<const f4*>(Rs + (wave * RW + it) * ks * 64) + lane;
    float ta[3], tr[RW][3];
#pragma unroll
    for (int k = 0; k < 3; ++k) {
      const int sk = ks4 * 4 + k < ks ? ks4 * 4 + k : ks - 1;
      ta[k] = xt[sk * 64 + lane];
#pragma unroll
      for (int it = 0; it < RW; ++it) tr[it][k] = Rs[((wave * RW + it) * ks + sk) * 64 + lane];
    }
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
  };
  // transform and row-side contraction of the RW tiles of one column tile; returns the tiles in kk
  auto row_side = [&](const f4 (&acc)[RW], const f4& v, const f4& e, bool diag_stage, int64_t col_tile, f4 (&kk)[RW]) {
#pragma unroll
    for (int it = 0; it < RW; ++it) {
      kk[it].x = transform<KIND>(acc[it].x);
      kk[it].y = transform<KIND>(acc[it].y);
      kk[it].z = transform<KIND>(acc[it].z);
      kk[it].w = transform<KIND>(acc[it].w);
      if constexpr (KIND == EGP_MATERN12) {      // exact k(x, x) on the diagonal (see kmm_kernel.h)
        if (diag_stage && row_tile0 + it == col_tile) set_unit_diagonal(kk[it], q, p);
      }
      o[it] = __builtin_amdgcn_mfma_f32_16x16x4f32(kk[it].x, v.x, o[it], 0, 0, 0);
      o[it] = __builtin_amdgcn_mfma_f32_16x16x4f32(kk[it].y, v.y, o[it], 0, 0, 0);
      o[it] = __builtin_amdgcn_mfma_f32_16x16x4f32(kk[it].z, v.z, o[it], 0, 0, 0);
      o[it] = __builtin_amdgcn_mfma_f32_16x16x4f32(kk[it].w, v.w, o[it], 0, 0, 0);
      if (EXTRA) {
        eacc[it] = __builtin_fmaf(kk[it].x, e.x, eacc[it]);
        eacc[it] = __builtin_fmaf(kk[it].y, e.y, eacc[it]);
        eacc[it] = __builtin_fmaf(kk[it].z, e.z, eacc[it]);
        eacc[it] = __builtin_fmaf(kk[it].w, e.w, eacc[it]);
      }
    }
  };
  // read back the RW tiles of patch set `set`, transposed
  auto read_patches = [&](int set, f4 (&ktr)[RW]) {
#pragma unroll
    for (int it = 0; it < RW; ++it) {
      const float* rp = patch + (set * RW + it) * kPatchW + roff;
      ktr[it].x = rp[0];
      ktr[it].y = rp[8];
      ktr[it].z = rp[16];
      ktr[it].w = rp[24];
    }
  };
  // column side of one column tile: the wave's RW row tiles contracted with the packed V of those rows
  auto col_side = [&](const f4 (&ktr)[RW], int jt) {
    f4 oj = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int it = 0; it < RW; ++it) {
      oj = __builtin_amdgcn_mfma_f32_16x16x4f32(ktr[it].x, vrow[it].x, oj, 0, 0, 0);
      oj = __builtin_amdgcn_mfma_f32_16x16x4f32(ktr[it].y, vrow[it].y, oj, 0, 0, 0);
      oj = __builtin_amdgcn_mfma_f32_16x16x4f32(ktr[it].z, vrow[it].z, oj, 0, 0, 0);
      oj = __builtin_amdgcn_mfma_f32_16x16x4f32(ktr[it].w, vrow[it].w, oj, 0, 0, 0);
    }
    CJ[(wave * jt_stage + jt) * 64 + lane] = oj;
  };

  for (int k = k_begin; k < k_end; ++k) {
    const int buf = (k - k_begin) & 1;
    const int st = abs_stage(k);
    if (k + 1 < k_end) issue(abs_stage(k + 1), buf ^ 1);
    const bool dual = is_dual(k);
    const bool diag_stage = k / sb == 0;
    const float* xs = Xs + buf * jt_stage * ks * 64;
    if (!dual) {
      for (int jt = 0; jt < jt_stage; ++jt) {
        f4 acc[RW], kk[RW];
        distances(xs + jt * ks * 64, acc);
        f4 e = {0.f, 0.f, 0.f, 0.f};
        if (EXTRA) e = Es[buf * ef4 + jt * 4 + q];
        row_side(acc, Vs[buf * vf4 + jt * 64 + lane], e, diag_stage, (int64_t)st * jt_stage + jt, kk);
      }
    } else {
      for (int jt = 0; jt < jt_stage; ++jt) {
        f4 ktr[RW];
        if (jt > 0) read_patches((jt - 1) & 1, ktr);      // in flight during this tile's distance steps
        __builtin_amdgcn_sched_barrier(0);
        f4 acc[RW], kk[RW];
        distances(xs + jt * ks * 64, acc);
        __builtin_amdgcn_sched_barrier(0);
        if (jt > 0) col_side(ktr, jt - 1);
        f4 e = {0.f, 0.f, 0.f, 0.f};
        if (EXTRA) e = Es[buf * ef4 + jt * 4 + q];
        row_side(acc, Vs[buf * vf4 + jt * 64 + lane], e, false, 0, kk);
#pragma unroll
        for (int it = 0; it < RW; ++it)
          *reinterpret_cast<f4*>(patch + ((jt & 1) * RW + it) * kPatchW + woff) = kk[it];
        if (EXTRA) {
          // column side of the 17th column from the untransposed tiles: kk.r = k(column 4q + r, row p); the sum over
          // the lanes p is taken in the flush
          f4 ej = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int it = 0; it < RW; ++it) {
            ej.x = __builtin_fmaf(kk[it].x, erow[it], ej.x);
            ej.y = __builtin_fmaf(kk[it].y, erow[it], ej.y);
            ej.z = __builtin_fmaf(kk[it].z, erow[it], ej.z);
            ej.w = __builtin_fmaf(kk[it].w, erow[it], ej.w);
          }
          CJE[(wave * jt_stage + jt) * 64 + lane] = ej;
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      {
        f4 ktr[RW];
        read_patches((jt_stage - 1) & 1, ktr);
        col_side(ktr, jt_stage - 1);
      }
    }
    if ((k - k_begin) % flush_stages == flush_stages - 1) fold();
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (dual) {      // uniform over the workgroup
      flush(st);
      __syncthreads();
    }
  }
  fold();

  float* dst = Part + (int64_t)blockIdx.y * npad * TS;
#pragma unroll
  for (int it = 0; it < RW; ++it) {
    const int64_t row0 = (row_tile0 + it) * 16;
    if (cm) {
      *reinterpret_cast<f4*>(dst + (int64_t)p * npad + row0 + q * 4) = o2[it];
    } else {
      float* r0 = dst + (row0 + q * 4) * TS + p;
      r0[0 * TS] = o2[it].x;
      r0[1 * TS] = o2[it].y;
      r0[2 * TS] = o2[it].z;
      r0[3 * TS] = o2[it].w;
    }
    if (EXTRA) {
      float sum = eacc2[it];
      sum += __shfl_xor(sum, 16);
      sum += __shfl_xor(sum, 32);
      if (q == 0) {
        if (cm) dst[(int64_t)16 * npad + row0 + p] = sum;
        else dst[(row0 + p) * TS + 16] = sum;
      }
    }
  }
}

struct WideSymShape { int rw, jt; size_t lds; };
// LDS: rows 4 rw ks 256 B | patches 4 x 2 x rw x 1120 B | per column tile of a stage: 2 x (ks 256 + 1024) B of
// operands and 4 x 1024 B of column-side sums (a 17th column: 2 x 64 B and 4 x 1024 B more). jt = 0: does not fit.
WideSymShape wide_sym_shape(int ks, int extra) {
  WideSymShape w;
  w.rw = ks <= 40 ? 2 : 1;
  const size_t fixed = (size_t)4 * w.rw * ks * 256 + (size_t)4 * 2 * w.rw * kPatchW * 4;
  const size_t per_jt = (size_t)2 * (ks * 256 + 1024) + 4 * 1024 + (extra ? 2 * 64 + 4 * 1024 : 0);
  const size_t budget = 150 * 1024;
  int jt = 4;
  while (jt >= 1 && fixed + jt * per_jt > budget) jt /= 2;
  w.jt = jt;
  w.lds = fixed + (size_t)(jt > 0 ? jt : 0) * per_jt;
  return w;
}

template <int RW, int KIND, int EXTRA>
int launch_wide_sym_one(const Prepared& P, const Plan& pl, const WideSymShape& sh, const f4* Vp, const float* Ep,
                        float* Part, int cm, hipStream_t stream) {
  auto kern = kmm_kernel_wide_sym<RW, KIND, EXTRA>;
  EGP_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)sh.lds));
  const int nblk = (int)(P.npad / (64 * RW));
  hipLaunchKernelGGL(kern, dim3(nblk, pl.splits), dim3(256), sh.lds, stream, P.Xp, P.nrm, Vp, Ep, Part, P.npad, P.d,
                     P.ks, sh.jt, nblk, pl.stages_per_split, cm);
  EGP_HIP(hipGetLastError());
  return EGP_OK;
}

template <int RW, int EXTRA>
int launch_wide_sym_kind(const Prepared& P, const Plan& pl, const WideSymShape& sh, const f4* Vp, const float* Ep,
                         float* Part, int cm, hipStream_t stream) {
  switch (P.kernel_type) {
    case EGP_RBF: return launch_wide_sym_one<RW, EGP_RBF, EXTRA>(P, pl, sh, Vp, Ep, Part, cm, stream);
    case EGP_MATERN32: return launch_wide_sym_one<RW, EGP_MATERN32, EXTRA>(P, pl, sh, Vp, Ep, Part, cm, stream);
    case EGP_MATERN12: return launch_wide_sym_one<RW, EGP_MATERN12, EXTRA>(P, pl, sh, Vp, Ep, Part, cm, stream);
    default: return launch_wide_sym_one<RW, EGP_MATERN52, EXTRA>(P, pl, sh, Vp, Ep, Part, cm, stream);
  }
}

}  // namespace

bool wide_sym_applies(int64_t npad_rows, int64_t npad_cols, int ks, int nb, int extra) {
  return npad_rows == npad_cols && ks > 8 && nb == 1 && npad_rows / (64 * 8) >= 64 &&
         wide_sym_shape(ks, extra).jt >= 1;
}

Plan make_plan_wide_sym(int64_t npad, int ks, int extra) {
  const WideSymShape sh = wide_sym_shape(ks, extra);
  Plan pl;
  pl.big = true;
  pl.sym = true;
  pl.extra_slabs = 2;      // the int64 column-side slab
  const int nblk = (int)(npad / (64 * sh.rw));
  const int sb = 4 * sh.rw / sh.jt;
  pl.row_blocks = nblk;
  pl.stages_total = (nblk / 2 + 1) * sb;
  int want = 1024 / nblk;
  if (want < 1) want = 1;
  if (want > pl.stages_total) want = pl.stages_total;
  if (want > 64) want = 64;
  pl.stages_per_split = (pl.stages_total + want - 1) / want;
  pl.splits = (pl.stages_total + pl.stages_per_split - 1) / pl.stages_per_split;
  return pl;
}

// Part must hold pl.splits + 2 slabs of npad x (16 + extra) floats and kColsideAuxFloats more: the int64 column-side
// slab, cleared here, and the column sums of |V|, computed here (as in launch_sym).
int launch_wide_sym(const Prepared& P, const Plan& pl, int extra, const f4* Vp, const float* Ep, float* Part, int cm,
                    hipStream_t stream) {
  const WideSymShape sh = wide_sym_shape(P.ks, extra);
  if (sh.jt < 1) return fail(EGP_ERR_ARG, "the symmetric wide kernel does not fit d = %d", P.d);
  ProfScope prof(kProfKmm, stream);
  const size_t slab = (size_t)P.npad * (16 + extra);
  float* cside = Part + (size_t)pl.splits * slab;
  launch_zero_slab(cside, 2 * slab, stream);
  launch_col_abs_sums(Vp, Ep, P.npad, 1, extra, cside + 2 * slab, stream);
  if (sh.rw == 2) {
    if (extra) return launch_wide_sym_kind<2, 1>(P, pl, sh, Vp, Ep, Part, cm, stream);
    return launch_wide_sym_kind<2, 0>(P, pl, sh, Vp, Ep, Part, cm, stream);
  }
  if (extra) return launch_wide_sym_kind<1, 1>(P, pl, sh, Vp, Ep, Part, cm, stream);
  return launch_wide_sym_kind<1, 0>(P, pl, sh, Vp, Ep, Part, cm, stream);
}

}  // namespace kmm_detail
}  // namespace egp
