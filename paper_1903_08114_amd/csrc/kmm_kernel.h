// The fused kernel-matrix-multiply kernel template and its launch plumbing, shared by the translation
// units that instantiate it (kmm.hip: d <= 31, kmm_wide.hip: 32 <= d <= 63).
#pragma once

#include "egp_internal.h"

namespace egp {

typedef float f4 __attribute__((ext_vector_type(4)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

template <int KIND>
__device__ __forceinline__ float transform(float acc) {
  if constexpr (KIND == EGP_RBF) {
    return __builtin_amdgcn_exp2f(-acc);
  } else if constexpr (KIND == EGP_MATERN32) {
    float a = __builtin_amdgcn_sqrtf(__builtin_fabsf(acc));
    return __builtin_fmaf(a, kLn2, 1.0f) * __builtin_amdgcn_exp2f(-a);
  } else if constexpr (KIND == EGP_MATERN12) {
    return __builtin_amdgcn_exp2f(-__builtin_amdgcn_sqrtf(__builtin_fabsf(acc)));
  } else {
    float a = __builtin_amdgcn_sqrtf(__builtin_fabsf(acc));
    float poly = __builtin_fmaf(__builtin_fmaf(a, kLn2 * kLn2 / 3.0f, kLn2), a, 1.0f);
    return poly * __builtin_amdgcn_exp2f(-a);
  }
}

// Matern-1/2 has a cusp at r = 0: g = exp(-r) has slope -1 there, so the rounding error of the norm expansion
// (|x~_i|^2 + |x~_j|^2 - 2 x~_i.x~_j ~ 1e-7 instead of 0 for a point against itself) becomes an error of ~3e-4 in
// k(x, x), on every diagonal entry of a square product. On diagonal tiles of square products those entries are set
// to their exact value 1 (lane (q, p), register r holds k(column 4q + r, row p)). The other families are flat at 0.
template <typename V4>
__device__ __forceinline__ void set_unit_diagonal(V4& k, int q, int p) {
  const int r = p - 4 * q;
  if (r == 0) k.x = 1.0f;
  if (r == 1) k.y = 1.0f;
  if (r == 2) k.z = 1.0f;
  if (r == 3) k.w = 1.0f;
}

// Column-side sums of the symmetric kernels: 64-bit fixed point, so that the atomic adds from different workgroups
// commute exactly and the result does not depend on their order (float atomics would make the last bits vary from
// run to run). Column c of the right-hand sides gets the scale 2^e_c with e_c chosen from S_c = sum_i |V_ic| (colsum,
// a float computed in a fixed order) such that S_c * 2^e_c <= 2^61: kernel values are at most 1, so no sum of
// contributions can leave the int64 range, and one unit is 2^-61 of that bound. A column-side sum of ~2000
// contributions is therefore exact to 2^-50 S_c, against the 2^-24 sum_i |k_ij V_ic| of an fp32 accumulation.
__device__ __forceinline__ int colside_exp(unsigned sumbits) {
  int eb = (int)((sumbits >> 23) & 0xffu) - 127;      // S_c < 2^(eb + 1)
  if (eb < -126) eb = -126;
  const int e = 60 - eb;
  return e > 120 ? 120 : e;      // never below -68: a float scale exists either way
}
__device__ __forceinline__ float colside_scale(int e) { return __uint_as_float((unsigned)(e + 127) << 23); }
__device__ __forceinline__ float colside_value(long long sum, int e) {      // sum * 2^-e, rounded once to fp32
  return (float)((double)sum * __builtin_bit_cast(double, (unsigned long long)(1023 - e) << 52));
}
__device__ __forceinline__ void colside_add(long long* dst, float v, float scale) {
  const float a = __builtin_fabsf(v) * scale;                    // exact: a power of two
  const float ah = __builtin_floorf(a * 0x1p-32f);
  const float al = __builtin_fmaf(-ah, 0x1p32f, a);              // exact: the low bits of a, in [0, 2^32)
  unsigned long long m = ((unsigned long long)(unsigned)ah << 32) | (unsigned long long)(unsigned)al;
  if (v < 0.f) m = 0ull - m;
  atomicAdd(reinterpret_cast<unsigned long long*>(dst), m);
}

// ------------------------------------------------------------------------------------------------
// The fused kernel.
//   grid.x = row blocks (4 waves x R row tiles x 16 rows), grid.y = column splits
//   block  = 256 threads; each wave owns R row tiles for the whole column sweep of its split
//   LDS    = double-buffered stage of JT column tiles: packed points, packed V, extra column
//   Part   = [split][npad][TS] raw accumulators (TS = 16 NB + EXTRA); the epilogue kernel reduces
//            splits in a fixed order, scales by the outputscale and adds noise * V.
// ------------------------------------------------------------------------------------------------
typedef short s4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
typedef float f2 __attribute__((ext_vector_type(2)));

// SPLIT = 1: the tile x V contraction runs on the bf16 MFMA with both operands split into a high and a low
// bf16 part (k = k_hi + k_lo, v = v_hi + v_lo; k_hi v_hi + k_hi v_lo + k_lo v_hi, fp32 accumulation): 16
// significant bits per factor, relative error ~2^-16 per product, and three 16x16x16 steps in place of four
// fp32 16x16x4 steps. Unlike the fp32 MFMA, the bf16 MFMA co-executes with the VALU work of the transform.
// The distance step stays in fp32 (it cancels). V arrives pre-split: dwords 0,1 of a packed quad hold the four
// high parts, dwords 2,3 the four low parts.
template <int KS, int R, int KIND, int NB, int EXTRA, int JT, int SPLIT>
__global__ __launch_bounds__(256, 2) void kmm_kernel(const float* __restrict__ XpRow,
                                                     const float* __restrict__ nrm,
                                                     const float* __restrict__ Xp,
                                                     const f4* __restrict__ Vp,
                                                     const float* __restrict__ Ep,
                                                     float* __restrict__ Part, int64_t npad, int d,
                                                     int stages_per_split, int stages_total, int cm) {
  constexpr int TS = 16 * NB + EXTRA;
  constexpr int NBA = NB > 0 ? NB : 1;    // array extents when there is no 16-column block (single column: NB = 0, EXTRA = 1)
  static_assert(NB > 0 || EXTRA, "a launch carries at least one column");
  constexpr int XF4 = JT * KS * 16;       // f4 elements of packed points per stage
  constexpr int VF4 = JT * NB * 64;       // f4 elements of packed V per stage
  constexpr int EF4 = JT * 4;             // f4 elements of the extra column per stage
  constexpr int NX = (XF4 + 255) / 256;
  constexpr int NV = (VF4 + 255) / 256;

  __shared__ f4 Xs[2][XF4];
  __shared__ f4 Vs[2][VF4 > 0 ? VF4 : 1];
  __shared__ f4 Es[2][EXTRA ? EF4 : 1];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int q = lane >> 4, p = lane & 15;

  // ---- resident row operands ----
  const int64_t row_tile0 = ((int64_t)blockIdx.x * 4 + wave) * R;
  float b[R][KS];
  f4 cq[R];
  f4 o[R][NBA];
  float eacc[R];
  // Two-level accumulation: `o` sums a block of kFlushCols column points and is then folded into `o2`. A single
  // fp32 accumulator over n = 10^6 terms carries a rounding error of ~2^-24 sqrt(n) relative to the sum of
  // magnitudes (2e-5 of the result for random-sign right-hand sides at n = 2^20); with blocks of 4096 column
  // points the two levels carry ~3e-6 together.
  f4 o2[R][NBA];
  float eacc2[R];
  constexpr int kFlushStages = 4096 / (16 * JT);     // blocks of 4096 column points
  const int ds = d >> 2, dq = d & 3;
#pragma unroll
  for (int it = 0; it < R; ++it) {
    const float* src = XpRow + (row_tile0 + it) * KS * 64 + lane;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      float v = -2.0f * src[s * 64];
      if (s == ds && q == dq) v = 1.0f;     // the slot that multiplies the column point's norm
      b[it][s] = v;
    }
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
  auto fold = [&]() {
#pragma unroll
    for (int it = 0; it < R; ++it) {
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

  const int st_begin = blockIdx.y * stages_per_split;
  int st_end = st_begin + stages_per_split;
  if (st_end > stages_total) st_end = stages_total;

  const f4* Xg = reinterpret_cast<const f4*>(Xp);
  const f4* Eg = reinterpret_cast<const f4*>(Ep);
  // Stage copy global -> LDS without passing through registers: the 64 lanes of a wave deposit 16 bytes each
  // at consecutive LDS addresses from a wave-uniform base (the packed arrays are already in operand order, so
  // a stage is a straight copy).
  auto issue = [&](int st, int buf) {
    const int64_t xoff = (int64_t)st * XF4, voff = (int64_t)st * VF4, eoff = (int64_t)st * EF4;
#pragma unroll
    for (int k = 0; k < NX; ++k)
      if (XF4 % 256 == 0 || k * 256 + wave * 64 < XF4)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Xg + xoff + tid + k * 256),
                                         (__attribute__((address_space(3))) void*)(&Xs[buf][k * 256 + wave * 64]), 16, 0, 0);
#pragma unroll
    for (int k = 0; k < NV; ++k)
      if (VF4 % 256 == 0 || k * 256 + wave * 64 < VF4)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Vp + voff + tid + k * 256),
                                         (__attribute__((address_space(3))) void*)(&Vs[buf][k * 256 + wave * 64]), 16, 0, 0);
    if (EXTRA && tid < EF4)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Eg + eoff + tid),
                                       (__attribute__((address_space(3))) void*)(&Es[buf][0]), 16, 0, 0);
  };

  if (st_begin < st_end) issue(st_begin, 0);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();

  for (int st = st_begin; st < st_end; ++st) {
    const int buf = (st - st_begin) & 1;
    const bool more = st + 1 < st_end;
    if (more) issue(st + 1, buf ^ 1);

    const float* xs = reinterpret_cast<const float*>(Xs[buf]);
#pragma unroll 2
    for (int jt = 0; jt < JT; ++jt) {
      float a[KS];
#pragma unroll
      for (int s = 0; s < KS; ++s) a[s] = xs[(jt * KS + s) * 64 + lane];
      f4 v[NBA];
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) v[nb] = Vs[buf][(jt * NB + nb) * 64 + lane];
      f4 e = {0.f, 0.f, 0.f, 0.f};
      if (EXTRA) e = Es[buf][jt * 4 + q];
#pragma unroll
      for (int it = 0; it < R; ++it) {
        f4 acc = cq[it];
#pragma unroll
        for (int s = 0; s < KS; ++s) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[s], b[it][s], acc, 0, 0, 0);
        f4 k;
        k.x = transform<KIND>(acc.x);
        k.y = transform<KIND>(acc.y);
        k.z = transform<KIND>(acc.z);
        k.w = transform<KIND>(acc.w);
        if constexpr (KIND == EGP_MATERN12) {
          if (XpRow == Xp && row_tile0 + it == (int64_t)st * JT + jt) set_unit_diagonal(k, q, p);
        }
        if constexpr (SPLIT) {
          // high parts by truncation (taken straight from the upper halves), low parts = exact remainders
          const unsigned u0 = __float_as_uint(k.x), u1 = __float_as_uint(k.y);
          const unsigned u2 = __float_as_uint(k.z), u3 = __float_as_uint(k.w);
          const unsigned hi01 = __builtin_amdgcn_perm(u1, u0, 0x07060302u);
          const unsigned hi23 = __builtin_amdgcn_perm(u3, u2, 0x07060302u);
          const f2 l01 = {k.x - __uint_as_float(u0 & 0xffff0000u), k.y - __uint_as_float(u1 & 0xffff0000u)};
          const f2 l23 = {k.z - __uint_as_float(u2 & 0xffff0000u), k.w - __uint_as_float(u3 & 0xffff0000u)};
          const unsigned lo01 = __builtin_bit_cast(unsigned, __builtin_convertvector(l01, bf2));
          const unsigned lo23 = __builtin_bit_cast(unsigned, __builtin_convertvector(l23, bf2));
          typedef unsigned u2v __attribute__((ext_vector_type(2)));
          const s4 khi = __builtin_bit_cast(s4, (u2v){hi01, hi23});
          const s4 klo = __builtin_bit_cast(s4, (u2v){lo01, lo23});
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) {
            const s4 vhi = __builtin_bit_cast(s4, (f2){v[nb].x, v[nb].y});
            const s4 vlo = __builtin_bit_cast(s4, (f2){v[nb].z, v[nb].w});
            o[it][nb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(khi, vhi, o[it][nb], 0, 0, 0);
            o[it][nb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(khi, vlo, o[it][nb], 0, 0, 0);
            o[it][nb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(klo, vhi, o[it][nb], 0, 0, 0);
          }
        } else {
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) {
            o[it][nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(k.x, v[nb].x, o[it][nb], 0, 0, 0);
            o[it][nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(k.y, v[nb].y, o[it][nb], 0, 0, 0);
            o[it][nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(k.z, v[nb].z, o[it][nb], 0, 0, 0);
            o[it][nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(k.w, v[nb].w, o[it][nb], 0, 0, 0);
          }
        }
        if (EXTRA) {
          eacc[it] = __builtin_fmaf(k.x, e.x, eacc[it]);
          eacc[it] = __builtin_fmaf(k.y, e.y, eacc[it]);
          eacc[it] = __builtin_fmaf(k.z, e.z, eacc[it]);
          eacc[it] = __builtin_fmaf(k.w, e.w, eacc[it]);
        }
      }
    }
    if ((st - st_begin) % kFlushStages == kFlushStages - 1) fold();
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
  }
  fold();

  // ---- write raw accumulators: lane (q,p), register r holds out[row 4q + r][column p] ----
  float* dst = Part + (int64_t)blockIdx.y * npad * TS;
  if (cm) {
    // column-major partials [TS][npad]: the four rows of a lane are one 16-byte store
#pragma unroll
    for (int it = 0; it < R; ++it) {
      const int64_t row0 = (row_tile0 + it) * 16;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
        *reinterpret_cast<f4*>(dst + (int64_t)(nb * 16 + p) * npad + row0 + q * 4) = o2[it][nb];
      if (EXTRA) {
        float s = eacc2[it];
        s += __shfl_xor(s, 16);
        s += __shfl_xor(s, 32);
        if (q == 0) dst[(int64_t)(16 * NB) * npad + row0 + p] = s;
      }
    }
    return;
  }
#pragma unroll
  for (int it = 0; it < R; ++it) {
    const int64_t row0 = (row_tile0 + it) * 16;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      float* r0 = dst + (row0 + q * 4) * TS + nb * 16 + p;
      r0[0 * TS] = o2[it][nb].x;
      r0[1 * TS] = o2[it][nb].y;
      r0[2 * TS] = o2[it][nb].z;
      r0[3 * TS] = o2[it][nb].w;
    }
    if (EXTRA) {
      float s = eacc2[it];
      s += __shfl_xor(s, 16);
      s += __shfl_xor(s, 32);
      if (q == 0) dst[(row0 + p) * TS + 16 * NB] = s;
    }
  }
}

namespace kmm_detail {

struct Plan {
  bool big;
  int splits, stages_per_split, stages_total, row_blocks;
  int extra_slabs = 0;      // float slabs of room behind the per-split ones (symmetric kernels: 2, one int64 slab)
  bool sym = false;         // launch the symmetric kernel
  int waves = 4;            // waves per workgroup of the symmetric kernel (4 or 8)
};

// Launch shapes (row tiles per wave, column tiles per LDS stage). Up to 8 k-steps (d <= 31) the wide shape
// keeps 8 row tiles per wave; beyond that the row operands (R * KS registers) allow 4.
constexpr int kSmallR = 2, kSmallJT = 4;
// (with two column blocks AND a 33rd column the two accumulator levels of 8 tiles exceed 256 registers: 4 tiles)
constexpr int big_r(int ks, int nb = 1, int extra = 0) { return (ks <= 8 && !(nb == 2 && extra)) ? 8 : 4; }
// column tiles per stage: the largest of 16, 8, 4 whose double-buffered stage stays within 80 KB of LDS, so that
// two workgroups share a CU (a 90 KB stage at KS = 7 or at 32 columns left one wave per SIMD)
constexpr int big_jt(int ks, int nb = 1) {
  return 2 * 16 * (ks * 256 + nb * 1024 + 16) <= 80 * 1024 ? 16 : (2 * 8 * (ks * 256 + nb * 1024 + 16) <= 80 * 1024 ? 8 : 4);
}

inline Plan make_plan(int64_t npad_rows, int64_t npad_cols, int ks, int nb = 1, int extra = 0) {
  Plan pl;
  const int64_t big_rows = 64 * 8;
  pl.big = npad_rows / big_rows >= 64;     // enough row blocks for the wide shape to be worthwhile
  const int R = pl.big ? big_r(ks, nb, extra) : kSmallR, JT = pl.big ? big_jt(ks, nb) : kSmallJT;
  pl.row_blocks = (int)(npad_rows / (64 * R));
  pl.stages_total = (int)(npad_cols / (16 * JT));
  int want = 1024 / pl.row_blocks;
  if (want < 1) want = 1;
  if (want > pl.stages_total) want = pl.stages_total;
  if (want > 64) want = 64;
  pl.stages_per_split = (pl.stages_total + want - 1) / want;
  pl.splits = (pl.stages_total + pl.stages_per_split - 1) / pl.stages_per_split;
  return pl;
}

template <int KS, int KIND, int NB, int EXTRA, int SPLIT>
int launch_shape(const Prepared& P, const Prepared& Q, const Plan& pl, const f4* Vp, const float* Ep, float* Part,
                 int cm, hipStream_t stream) {   // P: column points, Q: row points
  dim3 grid(pl.row_blocks, pl.splits), block(256);
  if (pl.big) {
    hipLaunchKernelGGL((kmm_kernel<KS, big_r(KS, NB, EXTRA), KIND, NB, EXTRA, big_jt(KS, NB), SPLIT>), grid, block, 0, stream, Q.Xp, Q.nrm,
                       P.Xp, Vp, Ep, Part, Q.npad, P.d, pl.stages_per_split, pl.stages_total, cm);
  } else {
    hipLaunchKernelGGL((kmm_kernel<KS, kSmallR, KIND, NB, EXTRA, kSmallJT, SPLIT>), grid, block, 0, stream, Q.Xp,
                       Q.nrm, P.Xp, Vp, Ep, Part, Q.npad, P.d, pl.stages_per_split, pl.stages_total, cm);
  }
  EGP_HIP(hipGetLastError());
  return EGP_OK;
}

template <int KS, int KIND, int SPLIT>
int launch_cols(const Prepared& P, const Prepared& Q, const Plan& pl, int nb, int extra, const f4* Vp,
                const float* Ep, float* Part, int cm, hipStream_t stream) {
  if (nb == 0) return launch_shape<KS, KIND, 0, 1, SPLIT>(P, Q, pl, Vp, Ep, Part, cm, stream);      // one column, on the VALU
  if (nb == 1 && !extra) return launch_shape<KS, KIND, 1, 0, SPLIT>(P, Q, pl, Vp, Ep, Part, cm, stream);
  if (nb == 1 && extra) return launch_shape<KS, KIND, 1, 1, SPLIT>(P, Q, pl, Vp, Ep, Part, cm, stream);
  if (nb == 2 && !extra) return launch_shape<KS, KIND, 2, 0, SPLIT>(P, Q, pl, Vp, Ep, Part, cm, stream);
  return launch_shape<KS, KIND, 2, 1, SPLIT>(P, Q, pl, Vp, Ep, Part, cm, stream);
}

template <int KS, int SPLIT>
int launch_kind(const Prepared& P, const Prepared& Q, const Plan& pl, int nb, int extra, const f4* Vp,
                const float* Ep, float* Part, int cm, hipStream_t stream) {
  switch (P.kernel_type) {
    case EGP_RBF: return launch_cols<KS, EGP_RBF, SPLIT>(P, Q, pl, nb, extra, Vp, Ep, Part, cm, stream);
    case EGP_MATERN32: return launch_cols<KS, EGP_MATERN32, SPLIT>(P, Q, pl, nb, extra, Vp, Ep, Part, cm, stream);
    case EGP_MATERN12: return launch_cols<KS, EGP_MATERN12, SPLIT>(P, Q, pl, nb, extra, Vp, Ep, Part, cm, stream);
    default: return launch_cols<KS, EGP_MATERN52, SPLIT>(P, Q, pl, nb, extra, Vp, Ep, Part, cm, stream);
  }
}

template <int SPLIT>
int launch_all_ks(const Prepared& P, const Prepared& Q, const Plan& pl, int nb, int extra, const f4* Vp,
                  const float* Ep, float* Part, int cm, hipStream_t stream) {
  switch (P.ks) {
    case 1: return launch_kind<1, SPLIT>(P, Q, pl, nb, extra, Vp, Ep, Part, cm, stream);
    case 2: return launch_kind<2, SPLIT>(P, Q, pl, nb, extra, Vp, Ep, Part, cm, stream);
    case 3: return launch_kind<3, SPLIT>(P, Q, pl, nb, extra, Vp, Ep, Part, cm, stream);
    case 4: return launch_kind<4, SPLIT>(P, Q, pl, nb, extra, Vp, Ep, Part, cm, stream);
    case 5: return launch_kind<5, SPLIT>(P, Q, pl, nb, extra, Vp, Ep, Part, cm, stream);
    case 6: return launch_kind<6, SPLIT>(P, Q, pl, nb, extra, Vp, Ep, Part, cm, stream);
    case 7: return launch_kind<7, SPLIT>(P, Q, pl, nb, extra, Vp, Ep, Part, cm, stream);
    case 8: return launch_kind<8, SPLIT>(P, Q, pl, nb, extra, Vp, Ep, Part, cm, stream);
    default: return fail(EGP_ERR_ARG, "d = %d needs %d k-steps; this build supports d <= 31", P.d, P.ks);
  }
}

// defined in kmm_split.hip: the SPLIT = 1 instantiations and the in-place split of a packed V
int launch_all_ks_split(const Prepared& P, const Prepared& Q, const Plan& pl, int nb, int extra, const f4* Vp,
                        const float* Ep, float* Part, int cm, hipStream_t stream);
void launch_split_vp(f4* Vp, int64_t count, hipStream_t stream);
// defined in kmm_wide.hip: more than 8 distance k-steps (d > 31), operands from LDS
Plan make_plan_wide(int64_t npad_rows, int64_t npad_cols, int ks, int nb, int extra);
int launch_wide(const Prepared& P, const Prepared& Q, const Plan& pl, int nb, int extra, const f4* Vp, const float* Ep,
                float* Part, int cm, hipStream_t stream);
// defined in kmm_sym.hip: square products that use every off-diagonal tile twice
void launch_zero_slab(float* slab, size_t floats, hipStream_t stream);
void launch_col_abs_sums(const f4* Vp, const float* Ep, int64_t npad, int nb, int extra, float* aux,
                         hipStream_t stream);
// The column-side region of the partial-sum buffer, after the pl.splits row-side slabs: an int64 slab (the room of
// two float slabs) followed by kColsideAuxFloats floats: the per-column sums of |V| (first 64) and the per-wave
// partial sums they are reduced from (kColsumBlocks blocks x 4 waves x 17).
constexpr int kColsumBlocks = 256;
constexpr int kColsideAuxFloats = 64 + kColsumBlocks * 4 * 17;
int sym_row_tiles(int64_t npad_rows, int64_t npad_cols, int ks, int nb, int extra);
Plan make_plan_sym(int64_t npad, int r, int ks, int nb, int extra);
int launch_sym(const Prepared& P, const Plan& pl, int nb, int extra, const f4* Vp, const float* Ep, float* Part, int cm,
               hipStream_t stream);
// defined in kmm_wide_sym.hip: the same for d > 31 (groups of 16 or 17 columns)
bool wide_sym_applies(int64_t npad_rows, int64_t npad_cols, int ks, int nb, int extra);
Plan make_plan_wide_sym(int64_t npad, int ks, int extra);
int launch_wide_sym(const Prepared& P, const Plan& pl, int extra, const f4* Vp, const float* Ep, float* Part, int cm,
                    hipStream_t stream);
// defined in kmm_bf.hip: every contraction on the bf16 MFMA
Plan make_plan_bf(int64_t npad_rows, int64_t npad_cols, int d, int nb, int extra);
void launch_pack_points_bf(const Prepared& P, hipStream_t stream);
int launch_all_bf(const Prepared& P, const Prepared& Q, const Plan& pl, int nb, int extra, const f4* Vp, void* Vb,
                  const float* Ep, float* Part, int cm, hipStream_t stream);

}  // namespace kmm_detail

}  // namespace egp
