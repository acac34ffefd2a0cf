// Fused kernel-matrix multiply with every contraction on the bf16 MFMA (mode EGP_KMM_SPLIT_BF16_ALL).
//
// Same tile algebra as kmm_kernel.h (paper, Method, "Partitioned kernel MVMs": tiles formed, multiplied,
// discarded), but each fp32 operand is carried as a sum of bf16 parts and the products that matter are
// accumulated in fp32 by v_mfma_f32_16x16x32_bf16:
//   distance  x~ = x0 + x1 + x2 exactly (three 8-bit parts of the 24-bit significand), both for the column
//             operand A = (-2 x~_j, |x~_j|^2) and the row operand B = (x~_i, 1); the six products
//             A0B0, A0B1, A1B0, A1B1, A2B0, A0B2 are kept (what is dropped is below 2^-24 |A||B|, the fp32
//             rounding level), stacked two per instruction along the K = 32 axis:
//             [A0|A0].[B0|B1] + [A1|A1].[B0|B1] + [A2|A0].[B0|B2]            (3 MFMA per 16 feature slots)
//   tile x V  k = k_hi + k_lo, v = v_hi + v_lo:  [k_hi|k_lo].[v_hi|v_hi] + [k_hi|k_lo].[v_lo|0]     (2 MFMA)
// Every MFMA of the kernel is the same instruction, so each accumulator sees one opcode only (a chain that
// mixed the 16x16x16 and 16x16x32 forms on one accumulator lost the first product on this toolchain).
// The reason to do this on gfx950: the bf16 MFMA overlaps (partly) with the VALU work of the transform and of
// the splitting, while the fp32 MFMA does not overlap with it at all.

#include "kmm_kernel.h"

namespace egp {

typedef __bf16 b8 __attribute__((ext_vector_type(8)));
typedef unsigned u4 __attribute__((ext_vector_type(4)));
typedef unsigned u2 __attribute__((ext_vector_type(2)));

namespace {

// x = p0 + p1 + p2 exactly, each part a bf16 (returned in the upper 16 bits of a dword)
__device__ __forceinline__ void split3(float x, unsigned* p0, unsigned* p1, unsigned* p2) {
  const unsigned b0 = __float_as_uint(x) & 0xffff0000u;
  const float r1 = x - __uint_as_float(b0);
  const unsigned b1 = __float_as_uint(r1) & 0xffff0000u;
  const float r2 = r1 - __uint_as_float(b1);
  *p0 = b0;
  *p1 = b1;
  *p2 = __float_as_uint(r2) & 0xffff0000u;
}
__device__ __forceinline__ unsigned pack2(unsigned lo_elem, unsigned hi_elem) {   // two upper halves -> one dword
  return (lo_elem >> 16) | hi_elem;
}

// Packed fp32 points -> split operands.
//   XbC[(tile*ks16 + g)*3 + op][lane]: op0 = [A0|A0], op1 = [A1|A1], op2 = [A2|A0]   (column operand)
//   XbR[(tile*ks16 + g)*2 + op][lane]: op0 = [B0|B1], op1 = [B0|B2]                  (row operand)
// Lane (q,p) carries feature slots 16 g + 4 q + e (e = 0..3) of point p.
__global__ __launch_bounds__(256) void pack_points_bf(const float* __restrict__ Xp, int64_t npad, int d, int ks,
                                                      int ks16, u4* __restrict__ XbC, u4* __restrict__ XbR) {
  const int64_t gidx = (int64_t)blockIdx.x * 256 + threadIdx.x;     // (tile, g, lane)
  const int64_t total = (npad >> 4) * ks16 * 64;
  if (gidx >= total) return;
  const int lane = (int)(gidx & 63);
  const int64_t tg = gidx >> 6;
  const int g = (int)(tg % ks16);
  const int64_t tile = tg / ks16;
  const int q = lane >> 4, p = lane & 15;
  unsigned a[3][4], b[3][4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int f = 16 * g + 4 * q + e;
    float xv = 0.f;
    if (f < ks * 4) xv = Xp[(tile * ks + (f >> 2)) * 64 + (f & 3) * 16 + p];   // slot d holds the squared norm
    const float av = (f < d) ? -2.0f * xv : (f == d ? xv : 0.f);
    const float bv = (f < d) ? xv : (f == d ? 1.0f : 0.f);
    split3(av, &a[0][e], &a[1][e], &a[2][e]);
    split3(bv, &b[0][e], &b[1][e], &b[2][e]);
  }
  unsigned A[3][2], B[3][2];
#pragma unroll
  for (int s = 0; s < 3; ++s) {
    A[s][0] = pack2(a[s][0], a[s][1]);
    A[s][1] = pack2(a[s][2], a[s][3]);
    B[s][0] = pack2(b[s][0], b[s][1]);
    B[s][1] = pack2(b[s][2], b[s][3]);
  }
  u4* c = XbC + (tg * 3) * 64 + lane;
  c[0] = (u4){A[0][0], A[0][1], A[0][0], A[0][1]};
  c[64] = (u4){A[1][0], A[1][1], A[1][0], A[1][1]};
  c[128] = (u4){A[2][0], A[2][1], A[0][0], A[0][1]};
  u4* r = XbR + (tg * 2) * 64 + lane;
  r[0] = (u4){B[0][0], B[0][1], B[1][0], B[1][1]};
  r[64] = (u4){B[0][0], B[0][1], B[2][0], B[2][1]};
}

// fp32 packed V quads -> VbA = [v_hi|v_hi] (16 bytes per lane), VbB = v_lo (8 bytes per lane)
__global__ __launch_bounds__(256) void split_v_bf(const f4* __restrict__ Vp, int64_t count, u4* __restrict__ VbA,
                                                  u2* __restrict__ VbB) {
  const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (g >= count) return;
  const f4 v = Vp[g];
  const unsigned u0 = __float_as_uint(v.x), u1 = __float_as_uint(v.y);
  const unsigned u2_ = __float_as_uint(v.z), u3 = __float_as_uint(v.w);
  const f2 l01 = {v.x - __uint_as_float(u0 & 0xffff0000u), v.y - __uint_as_float(u1 & 0xffff0000u)};
  const f2 l23 = {v.z - __uint_as_float(u2_ & 0xffff0000u), v.w - __uint_as_float(u3 & 0xffff0000u)};
  const unsigned h01 = __builtin_amdgcn_perm(u1, u0, 0x07060302u), h23 = __builtin_amdgcn_perm(u3, u2_, 0x07060302u);
  VbA[g] = (u4){h01, h23, h01, h23};
  VbB[g] = (u2){__builtin_bit_cast(unsigned, __builtin_convertvector(l01, bf2)),
                __builtin_bit_cast(unsigned, __builtin_convertvector(l23, bf2))};
}

template <int KS16, int R, int KIND, int NB, int EXTRA, int JT>
__global__ __launch_bounds__(256, 2) void kmm_kernel_bf(const u4* __restrict__ XbR, const float* __restrict__ nrm,
                                                        const u4* __restrict__ XbC, const u4* __restrict__ VbA,
                                                        const u2* __restrict__ VbB, const float* __restrict__ Ep,
                                                        float* __restrict__ Part, int64_t npad,
                                                        int stages_per_split, int stages_total, int cm,
                                                        int square) {
  constexpr int TS = 16 * NB + EXTRA;
  constexpr int NBA = NB > 0 ? NB : 1;       // array extents of the single-column shape (NB = 0, EXTRA = 1)
  static_assert(NB > 0 || EXTRA, "a launch carries at least one column");
  constexpr int XU4 = JT * KS16 * 3 * 64;    // u4 elements of column operands per stage
  constexpr int AU4 = JT * NB * 64;          // u4 elements of [v_hi|v_hi] (and of [v_lo|0]) per stage
  constexpr int EF4 = JT * 4;
  constexpr int NX = XU4 / 256, NA = (AU4 + 255) / 256;
  static_assert(XU4 % 256 == 0, "stage size");

  __shared__ u4 Xs[2][XU4];
  __shared__ u4 As[2][AU4 > 0 ? AU4 : 1];
  __shared__ u2 Bs[2][AU4 > 0 ? AU4 : 1];
  __shared__ f4 Es[2][EXTRA ? EF4 : 1];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int q = lane >> 4, p = lane & 15;
  const int64_t row_tile0 = ((int64_t)blockIdx.x * 4 + wave) * R;

  b8 br[R][KS16][2];
  f4 cq[R];
  f4 o[R][NBA];
  float eacc[R];
#pragma unroll
  for (int it = 0; it < R; ++it) {
#pragma unroll
    for (int g = 0; g < KS16; ++g) {
      const u4* src = XbR + (((row_tile0 + it) * KS16 + g) * 2) * 64 + lane;
      br[it][g][0] = __builtin_bit_cast(b8, src[0]);
      br[it][g][1] = __builtin_bit_cast(b8, src[64]);
    }
    const float ni = nrm[(row_tile0 + it) * 16 + p];
    cq[it] = (f4){ni, ni, ni, ni};
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) o[it][nb] = (f4){0.f, 0.f, 0.f, 0.f};
    eacc[it] = 0.f;
  }

  const int st_begin = blockIdx.y * stages_per_split;
  int st_end = st_begin + stages_per_split;
  if (st_end > stages_total) st_end = stages_total;
  const f4* Eg = reinterpret_cast<const f4*>(Ep);
  // Stage copy global -> LDS without passing through registers: each wave's 64 lanes deposit 16 bytes each at
  // consecutive LDS addresses from a wave-uniform base (the packed arrays are already in operand order, so a
  // stage is a straight copy).
  auto issue = [&](int st, int buf) {
    const int64_t xoff = (int64_t)st * XU4, aoff = (int64_t)st * AU4, eoff = (int64_t)st * EF4;
#pragma unroll
    for (int k = 0; k < NX; ++k)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(XbC + xoff + tid + k * 256),
                                       (__attribute__((address_space(3))) void*)(&Xs[buf][k * 256 + wave * 64]), 16, 0, 0);
#pragma unroll
    for (int k = 0; k < NA; ++k) {
      if (AU4 % 256 == 0 || k * 256 + wave * 64 < AU4) {
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(VbA + aoff + tid + k * 256),
                                         (__attribute__((address_space(3))) void*)(&As[buf][k * 256 + wave * 64]), 16, 0, 0);
      }
    }
    // v_lo is 8 bytes per lane: copied as 16-byte chunks, two lanes' worth each
    {
      const u4* VbB4 = reinterpret_cast<const u4*>(VbB + aoff);
      u4* Bs4 = reinterpret_cast<u4*>(&Bs[buf][0]);
#pragma unroll
      for (int k = 0; k < (AU4 / 2 + 255) / 256; ++k)
        if ((AU4 / 2) % 256 == 0 || k * 256 + wave * 64 < AU4 / 2)
          __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(VbB4 + tid + k * 256),
                                           (__attribute__((address_space(3))) void*)(&Bs4[k * 256 + wave * 64]), 16, 0, 0);
    }
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
#pragma unroll 2
    for (int jt = 0; jt < JT; ++jt) {
      b8 ac[KS16][3];
#pragma unroll
      for (int g = 0; g < KS16; ++g)
#pragma unroll
        for (int op = 0; op < 3; ++op) ac[g][op] = __builtin_bit_cast(b8, Xs[buf][((jt * KS16 + g) * 3 + op) * 64 + lane]);
      b8 va[NBA], vl[NBA];
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        va[nb] = __builtin_bit_cast(b8, As[buf][(jt * NB + nb) * 64 + lane]);
        const u2 lo = Bs[buf][(jt * NB + nb) * 64 + lane];
        vl[nb] = __builtin_bit_cast(b8, (u4){lo.x, lo.y, 0u, 0u});            // [v_lo|0]
      }
      f4 e = {0.f, 0.f, 0.f, 0.f};
      if (EXTRA) e = Es[buf][jt * 4 + q];
#pragma unroll
      for (int it = 0; it < R; ++it) {
        f4 acc = cq[it];
#pragma unroll
        for (int g = 0; g < KS16; ++g) {
          // smallest contributions first
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ac[g][2], br[it][g][1], acc, 0, 0, 0);   // A2B0 + A0B2
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ac[g][1], br[it][g][0], acc, 0, 0, 0);   // A1B0 + A1B1
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ac[g][0], br[it][g][0], acc, 0, 0, 0);   // A0B0 + A0B1
        }
        f4 k;
        k.x = transform<KIND>(acc.x);
        k.y = transform<KIND>(acc.y);
        k.z = transform<KIND>(acc.z);
        k.w = transform<KIND>(acc.w);
        if constexpr (KIND == EGP_MATERN12) {      // exact k(x, x) on the diagonal of a square product (see kmm_kernel.h)
          if (square && row_tile0 + it == (int64_t)st * JT + jt) set_unit_diagonal(k, q, p);
        }
        const unsigned u0 = __float_as_uint(k.x), u1 = __float_as_uint(k.y);
        const unsigned u2_ = __float_as_uint(k.z), u3 = __float_as_uint(k.w);
        const unsigned hi01 = __builtin_amdgcn_perm(u1, u0, 0x07060302u);
        const unsigned hi23 = __builtin_amdgcn_perm(u3, u2_, 0x07060302u);
        const f2 l01 = {k.x - __uint_as_float(u0 & 0xffff0000u), k.y - __uint_as_float(u1 & 0xffff0000u)};
        const f2 l23 = {k.z - __uint_as_float(u2_ & 0xffff0000u), k.w - __uint_as_float(u3 & 0xffff0000u)};
        const unsigned lo01 = __builtin_bit_cast(unsigned, __builtin_convertvector(l01, bf2));
        const unsigned lo23 = __builtin_bit_cast(unsigned, __builtin_convertvector(l23, bf2));
        const b8 khl = __builtin_bit_cast(b8, (u4){hi01, hi23, lo01, lo23});
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          o[it][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(khl, vl[nb], o[it][nb], 0, 0, 0);       // k_hi v_lo
          o[it][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(khl, va[nb], o[it][nb], 0, 0, 0);       // (k_hi + k_lo) v_hi
        }
        if (EXTRA) {
          eacc[it] = __builtin_fmaf(k.x, e.x, eacc[it]);
          eacc[it] = __builtin_fmaf(k.y, e.y, eacc[it]);
          eacc[it] = __builtin_fmaf(k.z, e.z, eacc[it]);
          eacc[it] = __builtin_fmaf(k.w, e.w, eacc[it]);
        }
      }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
  }

  float* dst = Part + (int64_t)blockIdx.y * npad * TS;
#pragma unroll
  for (int it = 0; it < R; ++it) {
    const int64_t row0 = (row_tile0 + it) * 16;
    if (cm) {
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
        *reinterpret_cast<f4*>(dst + (int64_t)(nb * 16 + p) * npad + row0 + q * 4) = o[it][nb];
    } else {
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        float* r0 = dst + (row0 + q * 4) * TS + nb * 16 + p;
        r0[0 * TS] = o[it][nb].x;
        r0[1 * TS] = o[it][nb].y;
        r0[2 * TS] = o[it][nb].z;
        r0[3 * TS] = o[it][nb].w;
      }
    }
    if (EXTRA) {
      float s = eacc[it];
      s += __shfl_xor(s, 16);
      s += __shfl_xor(s, 32);
      if (q == 0) {
        if (cm) dst[(int64_t)(16 * NB) * npad + row0 + p] = s;
        else dst[(row0 + p) * TS + 16 * NB] = s;
      }
    }
  }
}

// 8 row tiles per wave; 4 when two 16-feature groups (d >= 16) meet a 17th column or a second column block,
// where 8 tiles' operands and accumulators no longer fit 256 registers without spilling
constexpr int kBfSmallR = 2;
constexpr int bf_big_r(int ks16, int nb, int extra) { return (ks16 >= 2 && (nb == 2 || extra)) ? 4 : 8; }
constexpr int bf_big_jt(int ks16, int nb = 1) { return 8 / ks16 / (nb > 0 ? nb : 1); }   // keeps a stage near 36 KB
constexpr int bf_small_jt(int ks16) { return 4 / ks16; }

template <int KS16, int KIND, int NB, int EXTRA>
int launch_bf_shape(const Prepared& P, const Prepared& Q, const kmm_detail::Plan& pl, const u4* VbA, const u2* VbB,
                    const float* Ep, float* Part, int cm, hipStream_t stream) {
  dim3 grid(pl.row_blocks, pl.splits), block(256);
  const u4* xr = reinterpret_cast<const u4*>(Q.XbR);
  const u4* xc = reinterpret_cast<const u4*>(P.XbC);
  if (pl.big)
    hipLaunchKernelGGL((kmm_kernel_bf<KS16, bf_big_r(KS16, NB, EXTRA), KIND, NB, EXTRA, bf_big_jt(KS16, NB)>), grid, block, 0, stream, xr, Q.nrm, xc,
                       VbA, VbB, Ep, Part, Q.npad, pl.stages_per_split, pl.stages_total, cm, (int)(Q.Xp == P.Xp));
  else
    hipLaunchKernelGGL((kmm_kernel_bf<KS16, kBfSmallR, KIND, NB, EXTRA, bf_small_jt(KS16)>), grid, block, 0, stream, xr, Q.nrm,
                       xc, VbA, VbB, Ep, Part, Q.npad, pl.stages_per_split, pl.stages_total, cm, (int)(Q.Xp == P.Xp));
  EGP_HIP(hipGetLastError());
  return EGP_OK;
}

template <int KS16, int KIND>
int launch_bf_cols(const Prepared& P, const Prepared& Q, const kmm_detail::Plan& pl, int nb, int extra, const u4* VbA,
                   const u2* VbB, const float* Ep, float* Part, int cm, hipStream_t stream) {
  if (nb == 0) return launch_bf_shape<KS16, KIND, 0, 1>(P, Q, pl, VbA, VbB, Ep, Part, cm, stream);      // one column, on the VALU
  if (nb == 1 && !extra) return launch_bf_shape<KS16, KIND, 1, 0>(P, Q, pl, VbA, VbB, Ep, Part, cm, stream);
  if (nb == 1 && extra) return launch_bf_shape<KS16, KIND, 1, 1>(P, Q, pl, VbA, VbB, Ep, Part, cm, stream);
  if (nb == 2 && !extra) return launch_bf_shape<KS16, KIND, 2, 0>(P, Q, pl, VbA, VbB, Ep, Part, cm, stream);
  return launch_bf_shape<KS16, KIND, 2, 1>(P, Q, pl, VbA, VbB, Ep, Part, cm, stream);
}

template <int KS16>
int launch_bf_kind(const Prepared& P, const Prepared& Q, const kmm_detail::Plan& pl, int nb, int extra, const u4* VbA,
                   const u2* VbB, const float* Ep, float* Part, int cm, hipStream_t stream) {
  switch (P.kernel_type) {
    case EGP_RBF: return launch_bf_cols<KS16, EGP_RBF>(P, Q, pl, nb, extra, VbA, VbB, Ep, Part, cm, stream);
    case EGP_MATERN32: return launch_bf_cols<KS16, EGP_MATERN32>(P, Q, pl, nb, extra, VbA, VbB, Ep, Part, cm, stream);
    case EGP_MATERN12: return launch_bf_cols<KS16, EGP_MATERN12>(P, Q, pl, nb, extra, VbA, VbB, Ep, Part, cm, stream);
    default: return launch_bf_cols<KS16, EGP_MATERN52>(P, Q, pl, nb, extra, VbA, VbB, Ep, Part, cm, stream);
  }
}

}  // namespace

namespace kmm_detail {

Plan make_plan_bf(int64_t npad_rows, int64_t npad_cols, int d, int nb, int extra) {
  Plan pl;
  const int ks16 = (d + 1 + 15) / 16;
  pl.big = npad_rows / (64 * 8) >= 64;
  const int R = pl.big ? bf_big_r(ks16, nb, extra) : kBfSmallR, JT = pl.big ? bf_big_jt(ks16, nb) : bf_small_jt(ks16);
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

void launch_pack_points_bf(const Prepared& P, hipStream_t stream) {
  const int ks16 = (P.d + 1 + 15) / 16;
  const int64_t total = (P.npad >> 4) * ks16 * 64;
  hipLaunchKernelGGL(pack_points_bf, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, P.Xp, P.npad, P.d,
                     P.ks, ks16, reinterpret_cast<u4*>(P.XbC), reinterpret_cast<u4*>(P.XbR));
}

// Vp: fp32 packed quads (count of them); Vb: room for 2 x the bytes of Vp
int launch_all_bf(const Prepared& P, const Prepared& Q, const Plan& pl, int nb, int extra, const f4* Vp, void* Vb,
                  const float* Ep, float* Part, int cm, hipStream_t stream) {
  const int64_t count = (P.npad >> 4) * nb * 64;
  u4* VbA = static_cast<u4*>(Vb);
  u2* VbB = reinterpret_cast<u2*>(VbA + count);
  if (count > 0) {
    ProfScope prof(kProfPack, stream);
    hipLaunchKernelGGL(split_v_bf, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, stream, Vp, count, VbA, VbB);
  }
  ProfScope prof(kProfKmm, stream);
  const int ks16 = (P.d + 1 + 15) / 16;
  if (ks16 == 1) return launch_bf_kind<1>(P, Q, pl, nb, extra, VbA, VbB, Ep, Part, cm, stream);
  return launch_bf_kind<2>(P, Q, pl, nb, extra, VbA, VbB, Ep, Part, cm, stream);
}

}  // namespace kmm_detail
}  // namespace egp
