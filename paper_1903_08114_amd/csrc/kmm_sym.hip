// Symmetric variant of the fused kernel-matrix multiply (square products, d <= 31; 1, 16, 17, 32 or 33 right-hand
// sides per launch).
//
// The kernel matrix is symmetric (paper, Background: k(x, x') is a covariance), so the tile K[I,J] that serves
// out[I] += K[I,J] V[J] also serves out[J] += K[I,J]^T V[I]. A workgroup owns 64 R rows (row block b) and sweeps
// the column blocks b, b+1, ..., b + floor(nblk/2) (cyclically). On the blocks strictly between the diagonal one
// and the half-way one every tile is used twice, so the distance steps and the transform of half of all tiles are
// never computed:
//   row side     as in kmm_kernel: the tile feeds the contraction with V[J] straight from the accumulator layout;
//   column side  needs the tile transposed relative to that layout. Each wave passes the tile through a private
//                LDS patch (one 16-byte write, four 4-byte reads per lane, both free of bank conflicts), and
//                contracts it with the packed V of its own row tiles (resident in registers). The column-side sums
//                of a wave's R row tiles go to LDS; at the end of a stage the waves' sums are added up and
//                leave the workgroup as 64-bit fixed-point atomic adds (colside_add, kmm_kernel.h) into an extra slab
//                of the partial-sum buffer.
//                (LDS float atomics were measured far too slow for the first step: plain stores, one patch per wave.)
// Row-side accumulation has two levels, as in kmm_kernel. Where both fit the register file with eight row tiles per
// wave (16 columns up to 4 distance k-steps, a single column) or the shape runs four row tiles anyway (32 / 33 columns),
// the second level is a register set; for 17 columns (up to 4 k-steps) and for 16 columns beyond 4 k-steps it lives in
// device memory instead: after every block of 4096 column points a wave adds its register accumulators to its own rows
// of the partial-sum slab (plain loads and stores: a wave owns its rows of its split's slab) and clears them. That
// frees R * 16 NB registers, which is what lets those shapes keep eight row tiles per wave.
// The diagonal block and (for an even block count) the half-way block are computed one-sided, as in kmm_kernel.
// Results differ from kmm_kernel's only in summation order. Within a workgroup that order is fixed, and the integer
// atomic adds between workgroups commute exactly: results are reproducible bit for bit.
#include "kmm_kernel.h"

namespace egp {
namespace kmm_detail {

namespace {

// column tiles per stage: 8 up to 4 distance k-steps with one 16-column block and no 17th column, else 4 (keeps the
// workgroup's LDS under 80 KB: two per CU)
constexpr int sym_jt(int ks, int nb, int extra) { return (ks <= 4 && nb <= 1 && !extra) ? 8 : 4; }
constexpr int kPatch = 280;      // floats of one transposition patch: 70 slots of 16 bytes

// Sum over the 16 lanes of a DPP row (all lanes receive it): two quad permutations, half-row mirror, row mirror.
__device__ __forceinline__ float row_sum16(float x) {
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xf, 0xf, false));
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xf, 0xf, false));
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x141, 0xf, 0xf, false));
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x140, 0xf, 0xf, false));
  return x;
}

// LDS of one workgroup (static arrays in the kernel; this struct mirrors their sizes for the launch-time checks).
//   Xs, Vs, Es  double-buffered stage: packed column points, packed V, the extra column
//   Ts          per wave: two transposition patches
//   CJ          column-side sums of one stage, per wave: [wave][tile][block][slot], register r = component
//   CJE         the same for the 17th column: lane (q, p), component r holds the sum over the wave's rows with point
//               index p of k(column 4q + r, row) e[row]; the sum over p is left to the flush
//   cscale      fixed-point scale of each right-hand-side column (colside_exp)
//   Er          the 17th column's entries at the wave's own rows (the column-side weights of its tiles), read back one
//               value per row-tile step instead of being held in R registers (R = 8 only: the 33-column shape has the
//               registers, and no LDS to spare)
template <int KS, int R, int NB, int EXTRA, int NW>
struct SymLds {
  static constexpr int JT = sym_jt(KS, NB, EXTRA);
  static constexpr int NBA = NB > 0 ? NB : 1;
  static constexpr int XF4 = JT * KS * 16, VF4 = JT * NBA * 64, EF4 = JT * 4;
  static constexpr bool kErLds = EXTRA && R == 8;
  static constexpr size_t xs = 0;
  static constexpr size_t vs = xs + (size_t)2 * XF4 * 16;
  static constexpr size_t ts = vs + (NB ? (size_t)2 * VF4 * 16 : 16);
  static constexpr size_t es = ts + (NB ? (size_t)NW * 2 * kPatch * 4 : 16);
  static constexpr size_t cj = es + (EXTRA ? (size_t)2 * EF4 * 16 : 16);
  static constexpr size_t cje = cj + (NB ? (size_t)NW * JT * NBA * 64 * 16 : 16);
  static constexpr size_t csc = cje + (EXTRA ? (size_t)NW * JT * 64 * 16 : 16);
  static constexpr size_t er = csc + 144;      // 34 floats, rounded up to 16 bytes
  static constexpr size_t total = er + (kErLds ? (size_t)NW * R * 16 * 4 : 16);
  static_assert((kPatch * 4) % 16 == 0, "patches keep the 16-byte alignment of what follows");
};

// NW waves per workgroup: 4 (two workgroups per CU) or 8 (one). A workgroup owns 16 R NW rows; its NW waves' column-
// side sums of a column tile are added in LDS before they leave as atomic adds, so eight waves halve the adds.
template <int KS, int R, int KIND, int NB, int EXTRA, int NW>
__global__ __launch_bounds__(64 * NW, NW == 4 ? 2 : 1) void kmm_kernel_sym(
    const float* __restrict__ Xp, const float* __restrict__ nrm, const f4* __restrict__ Vp,
    const float* __restrict__ Ep, float* __restrict__ Part, int64_t npad, int d, int nblk, int stages_per_split,
    int cm) {
  // (the int64 column-side slab and the column maxima follow the gridDim.y row-side slabs of Part)
  using L = SymLds<KS, R, NB, EXTRA, NW>;
  constexpr int JT = L::JT;
  constexpr int TS = 16 * NB + EXTRA;      // NB = 0, EXTRA = 1: a single column, everything on the VALU
  static_assert(NB == 1 || NB == 2 || (NB == 0 && EXTRA == 1), "1, 16, 17, 32 or 33 columns");
  static_assert(NW == 4 || NW == 8, "four or eight waves");
  static_assert(JT % (NW / 4) == 0 && (JT % NW == 0 || NW == 2 * JT), "the flush deals whole column tiles to thread groups");
  constexpr int NT = 64 * NW;
  constexpr int NBA = L::NBA;      // array extents
  constexpr int SB = R * NW / JT;      // stages per block of 16 R NW points
  constexpr int XF4 = L::XF4, VF4 = L::VF4, EF4 = L::EF4;
  constexpr int NX = (XF4 + NT - 1) / NT, NV = (VF4 + NT - 1) / NT;
  constexpr bool kErLds = L::kErLds;
  constexpr bool kLateRhs = EXTRA && NB == 1 && R == 8;      // see the two-sided loop

  __shared__ f4 Xs[2][XF4];
  __shared__ f4 Vs[2][NB ? VF4 : 1];
  __shared__ __attribute__((aligned(16))) float Ts[NB ? NW : 1][2][NB ? kPatch : 4];
  __shared__ f4 Es[2][EXTRA ? EF4 : 1];
  __shared__ f4 CJ[NB ? NW : 1][NB ? JT : 1][NBA][NB ? 64 : 1];
  __shared__ f4 CJE[EXTRA ? NW : 1][EXTRA ? JT : 1][EXTRA ? 64 : 1];
  __shared__ float cscale[34];
  __shared__ float Er[kErLds ? NW : 1][kErLds ? R : 1][16];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int q = lane >> 4, p = lane & 15;
  // Workgroups are dealt to the 8 XCDs round-robin. Row blocks are renumbered so that the workgroups resident on one
  // XCD own neighbouring row blocks: their sweeps then run a few stages apart over the same column tiles and share
  // them through that XCD's L2 (with the plain numbering every workgroup of an XCD streamed a range of its own).
  const int bi = (nblk & 7) == 0 ? (int)(blockIdx.x & 7) * (nblk >> 3) + (int)(blockIdx.x >> 3) : (int)blockIdx.x;
  const int half = nblk >> 1;
  const int stages_all = (half + 1) * SB;      // this workgroup's whole sweep, in stages
  const int s_total = nblk * SB;

  const int64_t row_tile0 = ((int64_t)bi * NW + wave) * R;
  float b[R][KS];
  f4 cq[R], o[R][NBA], vrow[R][NBA];
  float eacc[R], erow[kErLds ? 1 : R];
  // Second accumulation level: in device memory for the shapes that only fit eight row tiles without it (17 columns;
  // 16 columns beyond 4 distance k-steps), in registers for the others (no extra traffic).
  constexpr bool kFoldMem = NB == 1 && R == 8 && (EXTRA || KS > 4);
  f4 o2[kFoldMem ? 1 : R][NBA];
  float eacc2[kFoldMem ? 1 : R];
  constexpr int kFlushStages = 4096 / (16 * JT);
  const int ds = d >> 2, dq = d & 3;
#pragma unroll
  for (int it = 0; it < R; ++it) {
    const float* src = Xp + (row_tile0 + it) * KS * 64 + lane;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      float v = -2.0f * src[s * 64];
      if (s == ds && q == dq) v = 1.0f;
      b[it][s] = v;
    }
    const float ni = nrm[(row_tile0 + it) * 16 + p];
    cq[it] = (f4){ni, ni, ni, ni};
#pragma unroll
    for (int nb = 0; nb < NBA; ++nb) {
      o[it][nb] = (f4){0.f, 0.f, 0.f, 0.f};
      if constexpr (!kFoldMem) o2[it][nb] = (f4){0.f, 0.f, 0.f, 0.f};
      vrow[it][nb] = NB ? Vp[((row_tile0 + it) * NBA + nb) * 64 + lane] : (f4){0.f, 0.f, 0.f, 0.f};
    }
    eacc[it] = 0.f;
    if constexpr (!kFoldMem) eacc2[it] = 0.f;
    if constexpr (kErLds) {
      if (q == 0) Er[wave][it][p] = Ep[(row_tile0 + it) * 16 + p];      // (read by this wave only, after the barrier below)
    } else {
      erow[it] = EXTRA ? Ep[(row_tile0 + it) * 16 + p] : 0.f;
    }
  }
  // Adding the register sums to this wave's rows of the row-side slab of its split. Lane (q, p), register r of
  // o[it][nb] is out[row 4q + r of tile it][column 16 nb + p]; the slab's content on entry is not read (the first
  // call stores). The same lanes touch the same addresses at every call, so program order is all the ordering this
  // needs. With kFoldMem this is the second accumulation level itself; otherwise it runs once, at the end.
  float* const rdst = Part + (int64_t)blockIdx.y * npad * TS;
  bool first_fold = true;
  auto fold_to_slab = [&]() {
#pragma unroll
    for (int it = 0; it < R; ++it) {
      const int64_t row0 = (row_tile0 + it) * 16;
      if constexpr (NB > 0) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          if (cm) {      // column-major slab [TS][npad]: the four rows of a lane are one 16-byte access
            f4* ptr = reinterpret_cast<f4*>(rdst + (int64_t)(16 * nb + p) * npad + row0 + q * 4);
            f4 prev = {0.f, 0.f, 0.f, 0.f};
            if (!first_fold) prev = *ptr;
            *ptr = prev + o[it][nb];
          } else {
            float* r0 = rdst + (row0 + q * 4) * TS + 16 * nb + p;
            f4 prev = {0.f, 0.f, 0.f, 0.f};
            if (!first_fold) prev = (f4){r0[0 * TS], r0[1 * TS], r0[2 * TS], r0[3 * TS]};
            prev += o[it][nb];
            r0[0 * TS] = prev.x;
            r0[1 * TS] = prev.y;
            r0[2 * TS] = prev.z;
            r0[3 * TS] = prev.w;
          }
          o[it][nb] = (f4){0.f, 0.f, 0.f, 0.f};
        }
      }
      if (EXTRA) {      // the 17th / single column: the four lane groups hold partial sums over the column points
        float sum = eacc[it];
        sum += __shfl_xor(sum, 16);
        sum += __shfl_xor(sum, 32);
        if (q == 0) {
          float* ptr = cm ? rdst + (int64_t)(16 * NB) * npad + row0 + p : rdst + (row0 + p) * TS + 16 * NB;
          *ptr = first_fold ? sum : *ptr + sum;
        }
        eacc[it] = 0.f;
      }
    }
    first_fold = false;
  };
  auto fold_to_regs = [&]() {
    if constexpr (!kFoldMem) {
#pragma unroll
      for (int it = 0; it < R; ++it) {
#pragma unroll
        for (int nb = 0; nb < NBA; ++nb) {
          o2[it][nb] += o[it][nb];
          o[it][nb] = (f4){0.f, 0.f, 0.f, 0.f};
        }
        if (EXTRA) {
          eacc2[it] += eacc[it];
          eacc[it] = 0.f;
        }
      }
    }
  };
  // transposition patch: lane (q,p) holds M[4q + r][p] in register r and wants M[p][4q + r]
  float* patch = &Ts[NB ? wave : 0][0][0];
  // 16-byte slot of writer (q, p = 4a + b): 18 q + (a & 1) + 8 (a >> 1) + 2 b. Free of bank conflicts for 32 banks
  // with 8 lanes per write pass / 32 per read pass as well as for 64 banks with 16 / 64 (checked by enumeration).
  // Slot of lane (q, p) in a per-wave tile of column-side sums: q 16 + (p ^ f(q)), f = {0, 10, 4, 14}. The plain slot
  // q 16 + p made the column-major flush below (a thread reads row 4q + r of column c across the waves) hit each bank
  // four times; with the swizzle both that read and the 16-byte writes are conflict-free for 32 and for 64 banks
  // (enumerated on the CPU).
  const int cjslot = cm ? q * 16 + (p ^ ((q & 1) * 10 ^ (q >> 1) * 4)) : lane;      // (the row-major flush reads its own slot)
  const int woff = 4 * (18 * q + ((p >> 2) & 1) + 8 * (p >> 3) + 2 * (p & 3));
  const int roff = 72 * (p >> 2) + 4 * (q & 1) + 32 * (q >> 1) + (p & 3);      // + 8 r: the value for step r

  const int k_begin = blockIdx.y * stages_per_split;
  int k_end = k_begin + stages_per_split;
  if (k_end > stages_all) k_end = stages_all;

  const f4* Xg = reinterpret_cast<const f4*>(Xp);
  const f4* Eg = reinterpret_cast<const f4*>(Ep);
  auto abs_stage = [&](int k) {
    int st = bi * SB + k;
    return st >= s_total ? st - s_total : st;
  };
  auto is_dual = [&](int k) {
    const int delta = k / SB;
    return delta != 0 && !(delta == half && (nblk & 1) == 0);
  };
  auto issue = [&](int st, int buf) {
    const int64_t xoff = (int64_t)st * XF4, voff = (int64_t)st * VF4;
#pragma unroll
    for (int k = 0; k < NX; ++k)
      if (XF4 % NT == 0 || k * NT + wave * 64 < XF4)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Xg + xoff + tid + k * NT),
                                         (__attribute__((address_space(3))) void*)(&Xs[buf][k * NT + wave * 64]), 16, 0, 0);
    if constexpr (NB > 0) {
#pragma unroll
      for (int k = 0; k < NV; ++k)
        if (VF4 % NT == 0 || k * NT + wave * 64 < VF4)
          __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Vp + voff + tid + k * NT),
                                           (__attribute__((address_space(3))) void*)(&Vs[buf][k * NT + wave * 64]), 16, 0, 0);
    }
    if (EXTRA && tid < EF4)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Eg + (int64_t)st * EF4 + tid),
                                       (__attribute__((address_space(3))) void*)(&Es[buf][0]), 16, 0, 0);
  };
  // the column-side sums of stage st (absolute), one partial per wave in CJ, leave as atomic adds into the extra slab
  long long* slab = reinterpret_cast<long long*>(Part + (int64_t)gridDim.y * npad * TS);
  if (tid < TS)
    cscale[tid] = colside_scale(colside_exp(reinterpret_cast<const unsigned*>(slab + npad * TS)[tid]));
  // (visible to every thread after the barrier that follows the first stage's loads)
  auto flush = [&](int st) {
    if constexpr (NB == 0) {
    } else if (cm) {
      // column-major slab [column][row]: a thread takes (column c, row jrow) of the tiles of its thread group (256
      // threads per group: group g takes tiles g, g + NW/4, ...), so that the sixteen rows of a column are one
      // contiguous 64-byte run of atomic adds
      const int ft = tid & 255, fg = tid >> 8;
      const int c = ft >> 4, jrow = ft & 15;
      const float* cf = reinterpret_cast<const float*>(&CJ[0][0][0][0]);
      float sc[NBA];
#pragma unroll
      for (int nb = 0; nb < NBA; ++nb) sc[nb] = cscale[16 * nb + c];
      const int jq = jrow >> 2;
      const int off = (jq * 16 + (c ^ ((jq & 1) * 10 ^ (jq >> 1) * 4))) * 4 + (jrow & 3);
      constexpr int WS = JT * NBA * 256;      // floats of one wave's sums
#pragma unroll
      for (int h = 0; h < JT / (NW / 4); ++h) {
        const int jt = fg + h * (NW / 4);
#pragma unroll
        for (int nb = 0; nb < NBA; ++nb) {
          const int t0 = (jt * NBA + nb) * 256 + off;
          float v = (cf[0 * WS + t0] + cf[1 * WS + t0]) + (cf[2 * WS + t0] + cf[3 * WS + t0]);
          if constexpr (NW == 8) v += (cf[4 * WS + t0] + cf[5 * WS + t0]) + (cf[6 * WS + t0] + cf[7 * WS + t0]);
          colside_add(slab + (int64_t)(16 * nb + c) * npad + ((int64_t)st * JT + jt) * 16 + jrow, v, sc[nb]);
        }
      }
    } else if constexpr (JT % NW == 0) {
#pragma unroll
      for (int h = 0; h < JT / NW; ++h) {
        const int jt = wave + NW * h;      // thread (wave, lane) adds up the waves' sums of tiles wave, wave + NW, ...
#pragma unroll
        for (int nb = 0; nb < NBA; ++nb) {
          f4 v = (CJ[0][jt][nb][cjslot] + CJ[1][jt][nb][cjslot]) + (CJ[2][jt][nb][cjslot] + CJ[3][jt][nb][cjslot]);
          if constexpr (NW == 8)
            v += (CJ[4][jt][nb][cjslot] + CJ[5][jt][nb][cjslot]) + (CJ[6][jt][nb][cjslot] + CJ[7][jt][nb][cjslot]);
          long long* dst = slab + (((int64_t)st * JT + jt) * 16 + 4 * q) * TS + 16 * nb + p;
          const float sc = cscale[16 * nb + p];
          colside_add(dst + 0 * TS, v.x, sc);
          colside_add(dst + 1 * TS, v.y, sc);
          colside_add(dst + 2 * TS, v.z, sc);
          colside_add(dst + 3 * TS, v.w, sc);
        }
      }
    } else {
      // twice as many waves as column tiles: waves jt and jt + JT share tile jt, two of the four rows of a lane each
      const int jt = wave % JT, hf = wave / JT;
#pragma unroll
      for (int nb = 0; nb < NBA; ++nb) {
        f4 v = (CJ[0][jt][nb][cjslot] + CJ[1][jt][nb][cjslot]) + (CJ[2][jt][nb][cjslot] + CJ[3][jt][nb][cjslot]);
        v += (CJ[4][jt][nb][cjslot] + CJ[5][jt][nb][cjslot]) + (CJ[6][jt][nb][cjslot] + CJ[7][jt][nb][cjslot]);
        long long* dst = slab + (((int64_t)st * JT + jt) * 16 + 4 * q + 2 * hf) * TS + 16 * nb + p;
        const float sc = cscale[16 * nb + p];
        colside_add(dst + 0 * TS, hf ? v.z : v.x, sc);
        colside_add(dst + 1 * TS, hf ? v.w : v.y, sc);
      }
    }
    if (EXTRA) {
      // JT = 4: thread (wave, lane) takes tile `wave` (with eight waves the upper four repeat the work and do not add);
      // sum over the waves, then over the 16 lanes of the DPP row (point index p). Every lane then holds the four sums
      // of its row q; lanes p < 4 add component p. (The threads stay uniform up to the add itself: a flush tail
      // limited to some of the lanes cost the kernel ~60 registers.)
      static_assert(!EXTRA || JT == 4, "one tile per wave in the flush of the 17th column");
      const int jw = wave & 3;
      f4 v = (CJE[0][jw][lane] + CJE[1][jw][lane]) + (CJE[2][jw][lane] + CJE[3][jw][lane]);
      if constexpr (NW == 8) v += (CJE[4][jw][lane] + CJE[5][jw][lane]) + (CJE[6][jw][lane] + CJE[7][jw][lane]);
      v.x = row_sum16(v.x);
      v.y = row_sum16(v.y);
      v.z = row_sum16(v.z);
      v.w = row_sum16(v.w);
      const int r = p & 3;
      float add = r == 0 ? v.x : (r == 1 ? v.y : (r == 2 ? v.z : v.w));
      const int64_t j = ((int64_t)st * JT + jw) * 16 + 4 * q + r;
      const bool mine = p < 4 && wave < 4;
      if constexpr (NB > 0) {
        const int col = 16 * NB;
        if (mine) colside_add(cm ? slab + (int64_t)col * npad + j : slab + j * TS + col, add, cscale[16 * NB]);
      } else {
        if (mine) colside_add(slab + j, add, cscale[0]);      // a single column: the slab is [npad] in both layouts
      }
    }
  };

  if (k_begin < k_end) issue(abs_stage(k_begin), 0);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();

  for (int k = k_begin; k < k_end; ++k) {
    const int buf = (k - k_begin) & 1;
    const int st = abs_stage(k);
    if (k + 1 < k_end) issue(abs_stage(k + 1), buf ^ 1);
    const bool dual = is_dual(k);
    const float* xs = reinterpret_cast<const float*>(Xs[buf]);
    if (!dual) {
      // lane (q, p), register r holds entry (column 4q + r, row p): 0 where that is a diagonal entry, else 1
      const int dr = p - 4 * q;
      const f4 dmask = {dr == 0 ? 0.f : 1.f, dr == 1 ? 0.f : 1.f, dr == 2 ? 0.f : 1.f, dr == 3 ? 0.f : 1.f};
#pragma unroll(kLateRhs ? 1 : 2)
      for (int jt = 0; jt < JT; ++jt) {
        float a[KS];
#pragma unroll
        for (int s = 0; s < KS; ++s) a[s] = xs[(jt * KS + s) * 64 + lane];
        f4 v[NBA];
#pragma unroll
        for (int nb = 0; nb < NBA; ++nb) v[nb] = NB ? Vs[buf][(jt * NBA + nb) * 64 + lane] : (f4){0.f, 0.f, 0.f, 0.f};
        f4 e = {0.f, 0.f, 0.f, 0.f};
        if (EXTRA) e = Es[buf][jt * 4 + q];
        // which of the wave's row tiles (if any) is this column tile: the one whose diagonal entries are k(x, x)
        const int dtile = (int)((int64_t)st * JT + jt - row_tile0);
#pragma unroll
        for (int it = 0; it < R; ++it) {
          f4 acc = cq[it];
#pragma unroll
          for (int s = 0; s < KS; ++s) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[s], b[it][s], acc, 0, 0, 0);
          if constexpr (KIND == EGP_MATERN12) {
            // exact k(x, x) = 1 on the diagonal of a diagonal tile (see kmm_kernel.h): the squared distance of a
            // point to itself is set to its exact value 0 before the transform
            if (dtile == it) acc *= dmask;
          }
          f4 kk;
          kk.x = transform<KIND>(acc.x);
          kk.y = transform<KIND>(acc.y);
          kk.z = transform<KIND>(acc.z);
          kk.w = transform<KIND>(acc.w);
          if constexpr (NB > 0) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
              o[it][nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(kk.x, v[nb].x, o[it][nb], 0, 0, 0);
              o[it][nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(kk.y, v[nb].y, o[it][nb], 0, 0, 0);
              o[it][nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(kk.z, v[nb].z, o[it][nb], 0, 0, 0);
              o[it][nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(kk.w, v[nb].w, o[it][nb], 0, 0, 0);
            }
          }
          if (EXTRA) {
            eacc[it] = __builtin_fmaf(kk.x, e.x, eacc[it]);
            eacc[it] = __builtin_fmaf(kk.y, e.y, eacc[it]);
            eacc[it] = __builtin_fmaf(kk.z, e.z, eacc[it]);
            eacc[it] = __builtin_fmaf(kk.w, e.w, eacc[it]);
          }
        }
      }
    } else {
      // Operands of the next column tile are fetched while the current one is worked on; the order of the LDS
      // traffic and the MFMA groups inside a row-tile step is pinned (sched_barrier), because the compiler would
      // otherwise sink the reads of the transposed tile next to their use and expose their latency.
      float a[KS];
#pragma unroll
      for (int s = 0; s < KS; ++s) a[s] = xs[s * 64 + lane];
      f4 v[NBA];
#pragma unroll
      for (int nb = 0; nb < NBA; ++nb) v[nb] = NB ? Vs[buf][nb * 64 + lane] : (f4){0.f, 0.f, 0.f, 0.f};
      f4 e = {0.f, 0.f, 0.f, 0.f};
      if (EXTRA) e = Es[buf][q];
      for (int jt = 0; jt < JT; ++jt) {
        const int jn = jt + 1 < JT ? jt + 1 : JT - 1;
        float an[KS];
        f4 vn[NBA], oj[NBA];
#pragma unroll
        for (int nb = 0; nb < NBA; ++nb) {
          vn[nb] = v[nb];
          oj[nb] = (f4){0.f, 0.f, 0.f, 0.f};
        }
        f4 en = e, ej = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int it = 0; it <= R; ++it) {
          f4 kt = {0.f, 0.f, 0.f, 0.f};
          if (NB && it > 0) {      // transposed tile of the previous step: in flight during this step's distance MFMAs
            const float* rp = patch + ((it - 1) & 1) * kPatch + roff;
            kt.x = rp[0];
            kt.y = rp[8];
            kt.z = rp[16];
            kt.w = rp[24];
          }
          float er = 0.f;
          if (EXTRA && it < R) {
            if constexpr (kErLds) er = Er[wave][it][p];
            else er = erow[it];
          }
          if constexpr (kLateRhs) {
            // The right-hand-side operands of this column tile are first needed after the distance steps and the
            // transform of row tile 0, which cover their LDS latency: they are read here rather than a column tile
            // ahead, which saves the registers of a second copy (this shape has none to spare).
            if (it == 0 && jt > 0) {
              if constexpr (NB > 0) {
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) v[nb] = Vs[buf][(jt * NB + nb) * 64 + lane];
              }
              if (EXTRA) e = Es[buf][jt * 4 + q];
            }
          }
          if (it == R / 2) {
#pragma unroll
            for (int s = 0; s < KS; ++s) an[s] = xs[(jn * KS + s) * 64 + lane];
            if constexpr (!kLateRhs) {
              if constexpr (NB > 0) {
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) vn[nb] = Vs[buf][(jn * NB + nb) * 64 + lane];
              }
              if (EXTRA) en = Es[buf][jn * 4 + q];
            }
          }
          __builtin_amdgcn_sched_barrier(0);
          f4 acc = {0.f, 0.f, 0.f, 0.f};
          if (it < R) {
            acc = cq[it];
#pragma unroll
            for (int s = 0; s < KS; ++s) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[s], b[it][s], acc, 0, 0, 0);
          }
          __builtin_amdgcn_sched_barrier(0);
          if (NB && it > 0) {      // column side of the previous step; also covers the latency of the distance result
#pragma unroll
            for (int nb = 0; nb < NBA; ++nb) {
              oj[nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(kt.x, vrow[it - 1][nb].x, oj[nb], 0, 0, 0);
              oj[nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(kt.y, vrow[it - 1][nb].y, oj[nb], 0, 0, 0);
              oj[nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(kt.z, vrow[it - 1][nb].z, oj[nb], 0, 0, 0);
              oj[nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(kt.w, vrow[it - 1][nb].w, oj[nb], 0, 0, 0);
            }
          }
          __builtin_amdgcn_sched_barrier(0);
          if (it < R) {
            f4 kk;
            kk.x = transform<KIND>(acc.x);
            kk.y = transform<KIND>(acc.y);
            kk.z = transform<KIND>(acc.z);
            kk.w = transform<KIND>(acc.w);
            if constexpr (NB > 0) {
#pragma unroll
              for (int nb = 0; nb < NB; ++nb) {
                o[it][nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(kk.x, v[nb].x, o[it][nb], 0, 0, 0);
                o[it][nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(kk.y, v[nb].y, o[it][nb], 0, 0, 0);
                o[it][nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(kk.z, v[nb].z, o[it][nb], 0, 0, 0);
                o[it][nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(kk.w, v[nb].w, o[it][nb], 0, 0, 0);
              }
              *reinterpret_cast<f4*>(patch + (it & 1) * kPatch + woff) = kk;
            }
            if (EXTRA) {
              // kk.r = k(column point 4q + r, row point p): row side sums over the column points, column side over
              // the row points (lanes p; reduced after the row tiles)
              eacc[it] = __builtin_fmaf(kk.x, e.x, eacc[it]);
              eacc[it] = __builtin_fmaf(kk.y, e.y, eacc[it]);
              eacc[it] = __builtin_fmaf(kk.z, e.z, eacc[it]);
              eacc[it] = __builtin_fmaf(kk.w, e.w, eacc[it]);
              ej.x = __builtin_fmaf(kk.x, er, ej.x);
              ej.y = __builtin_fmaf(kk.y, er, ej.y);
              ej.z = __builtin_fmaf(kk.z, er, ej.z);
              ej.w = __builtin_fmaf(kk.w, er, ej.w);
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (NB > 0) {
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) CJ[wave][jt][nb][cjslot] = oj[nb];
        }
        if (EXTRA) {
          CJE[wave][jt][lane] = ej;
          if constexpr (!kLateRhs) e = en;
        }
#pragma unroll
        for (int s = 0; s < KS; ++s) a[s] = an[s];
        if constexpr (!kLateRhs) {
#pragma unroll
          for (int nb = 0; nb < NBA; ++nb) v[nb] = vn[nb];
        }
      }
    }
    if ((k - k_begin) % kFlushStages == kFlushStages - 1) {
      if constexpr (kFoldMem) fold_to_slab();
      else fold_to_regs();
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (dual) {      // uniform over the workgroup
      flush(st);
      __syncthreads();             // the per-wave sums are free again
    }
  }
  if constexpr (!kFoldMem) {      // the last partial block joins the second level, which then is what gets written
    fold_to_regs();
#pragma unroll
    for (int it = 0; it < R; ++it) {
#pragma unroll
      for (int nb = 0; nb < NBA; ++nb) o[it][nb] = o2[it][nb];
      eacc[it] = eacc2[it];
    }
  }
  fold_to_slab();      // (zeros for a split without stages; with registers as second level the only write)
}

template <int KS, int R, int KIND, int NB, int EXTRA, int NW>
int launch_sym_one(const Prepared& P, const Plan& pl, const f4* Vp, const float* Ep, float* Part, int cm,
                   hipStream_t stream) {
  using L = SymLds<KS, R, NB, EXTRA, NW>;
  auto kern = kmm_kernel_sym<KS, R, KIND, NB, EXTRA, NW>;
  const int nblk = (int)(P.npad / (16 * R * NW));
  if (pl.row_blocks != nblk || P.npad % (16 * R * NW) != 0)
    return fail(EGP_ERR_ARG, "internal: symmetric launch plan (%d blocks) does not match the kernel shape (%d)", pl.row_blocks, nblk);
  static_assert(NW == 8 || L::total <= 80 * 1024, "two workgroups of four waves share a CU");
  static_assert(L::total <= 160 * 1024, "one workgroup of eight waves per CU");
  hipLaunchKernelGGL(kern, dim3(nblk, pl.splits), dim3(64 * NW), 0, stream, P.Xp, P.nrm, Vp, Ep, Part, P.npad, P.d,
                     nblk, pl.stages_per_split, cm);
  EGP_HIP(hipGetLastError());
  return EGP_OK;
}

// Shapes: (row tiles per wave, waves) come from the plan (sym_row_tiles / sym_waves below), which instantiations exist
// is decided here; the two must agree, and launch_sym_one checks that they do.
template <int KS, int KIND>
int launch_sym_shape(const Prepared& P, const Plan& pl, int nb, int extra, const f4* Vp, const float* Ep, float* Part,
                     int cm, hipStream_t stream) {
  if (pl.waves != 4) return fail(EGP_ERR_ARG, "internal: only the four-wave symmetric kernels are instantiated");
  if (nb == 0) return launch_sym_one<KS, 8, KIND, 0, 1, 4>(P, pl, Vp, Ep, Part, cm, stream);
  if (nb == 2) {
    if (!extra) return launch_sym_one<KS, 4, KIND, 2, 0, 4>(P, pl, Vp, Ep, Part, cm, stream);
    if constexpr (KS <= 3) return launch_sym_one<KS, 4, KIND, 2, 1, 4>(P, pl, Vp, Ep, Part, cm, stream);
    else return fail(EGP_ERR_ARG, "internal: no symmetric kernel for 33 columns at this d");
  }
  if (extra) {
    if constexpr (KS <= 4) {
      return launch_sym_one<KS, 8, KIND, 1, 1, 4>(P, pl, Vp, Ep, Part, cm, stream);
    } else {
      return launch_sym_one<KS, 4, KIND, 1, 1, 4>(P, pl, Vp, Ep, Part, cm, stream);
    }
  }
  return launch_sym_one<KS, 8, KIND, 1, 0, 4>(P, pl, Vp, Ep, Part, cm, stream);
}

template <int KS>
int launch_sym_kind(const Prepared& P, const Plan& pl, int nb, int extra, const f4* Vp, const float* Ep, float* Part,
                    int cm, hipStream_t stream) {
  switch (P.kernel_type) {
    case EGP_RBF: return launch_sym_shape<KS, EGP_RBF>(P, pl, nb, extra, Vp, Ep, Part, cm, stream);
    case EGP_MATERN32: return launch_sym_shape<KS, EGP_MATERN32>(P, pl, nb, extra, Vp, Ep, Part, cm, stream);
    case EGP_MATERN12: return launch_sym_shape<KS, EGP_MATERN12>(P, pl, nb, extra, Vp, Ep, Part, cm, stream);
    default: return launch_sym_shape<KS, EGP_MATERN52>(P, pl, nb, extra, Vp, Ep, Part, cm, stream);
  }
}

}  // namespace

// Clears the column-side slab. A fill kernel rather than hipMemsetAsync: memset nodes recorded into a captured
// graph have replayed wrongly on this platform, and a caller may capture the stream.
__global__ __launch_bounds__(256) void zero_slab(f4* __restrict__ p, int64_t count) {
  for (int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x; g < count; g += (int64_t)gridDim.x * 256)
    p[g] = (f4){0.f, 0.f, 0.f, 0.f};
}
void launch_zero_slab(float* slab, size_t floats, hipStream_t stream) {      // floats: a multiple of 4
  const int64_t count = (int64_t)(floats / 4);
  int64_t blocks = (count + 255) / 256;
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(zero_slab, dim3((unsigned)blocks), dim3(256), 0, stream, reinterpret_cast<f4*>(slab), count);
}

// aux[16 nb + p] = sum over the points of |V| in column p of block nb, aux[16 nb_count] the same for the extra column
// (slightly inflated: they only serve as bounds). Two steps with fixed summation orders, so that the value, and with
// it the fixed-point scale of the column, is the same on every run: per-wave partial sums (every thread walks the
// elements of one (block, lane) class), then one wave per column adds the partials up.
__global__ __launch_bounds__(256) void col_abs_partial(const f4* __restrict__ Vp, const float* __restrict__ Ep,
                                                       int64_t npad, int nb_count, int extra, float* __restrict__ part) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t stride = (int64_t)gridDim.x * 256;      // a multiple of 128: block and lane of an element stay fixed
  float* mine = part + ((int64_t)blockIdx.x * 4 + wave) * 17;
  float m = 0.f;
  if (nb_count > 0) {
    const int64_t total = (npad >> 4) * nb_count * 64;
    for (int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x; g < total; g += stride) {
      const f4 v = Vp[g];
      m += (__builtin_fabsf(v.x) + __builtin_fabsf(v.y)) + (__builtin_fabsf(v.z) + __builtin_fabsf(v.w));
    }
    m += __shfl_xor(m, 16);
    m += __shfl_xor(m, 32);
  }
  if (lane < 16) mine[lane] = m;      // column lane of block (blockIdx.x * 4 + wave) % nb_count
  float e = 0.f;
  if (extra) {
    for (int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x; g < npad; g += stride) e += __builtin_fabsf(Ep[g]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) e += __shfl_xor(e, off);
  }
  if (lane == 0) mine[16] = e;
}
__global__ __launch_bounds__(64) void col_abs_final(const float* __restrict__ part, int waves, int nb_count, int extra,
                                                    float* __restrict__ colsum) {
  const int c = blockIdx.x, lane = threadIdx.x;      // one wave per column; lane l takes every 64th partial of it
  float s = 0.f;
  if (c < 16 * nb_count) {
    const int nb = c >> 4, p = c & 15;
    for (int w = nb + lane * nb_count; w < waves; w += 64 * nb_count) s += part[(int64_t)w * 17 + p];
  } else {      // the extra column
    for (int w = lane; w < waves; w += 64) s += part[(int64_t)w * 17 + 16];
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off);
  if (lane == 0) colsum[c] = s * 1.001f;      // covers the rounding of the sums above
}
void launch_col_abs_sums(const f4* Vp, const float* Ep, int64_t npad, int nb, int extra, float* aux,
                         hipStream_t stream) {
  hipLaunchKernelGGL(col_abs_partial, dim3(kColsumBlocks), dim3(256), 0, stream, Vp, Ep, npad, nb, extra, aux + 64);
  hipLaunchKernelGGL(col_abs_final, dim3(16 * nb + extra), dim3(64), 0, stream, aux + 64, kColsumBlocks * 4, nb, extra,
                     aux);
}

// Row tiles per wave of the symmetric kernel for this shape, or 0 where it does not apply. With the second
// accumulation level in device memory, eight row tiles fit the register file (two waves per SIMD) for 1 and 16
// columns at every d <= 31 and for 17 columns up to 4 distance k-steps (d <= 14); 17 columns beyond that and the 32-
// and 33-column shapes keep four.
int sym_row_tiles(int64_t npad_rows, int64_t npad_cols, int ks, int nb, int extra) {
  if (npad_rows != npad_cols || ks > 8 || nb > 2 || npad_rows / (64 * 8) < 64) return 0;
  if (nb == 0) return 8;      // a single column: no contraction block, few registers
  if (nb == 2) return (extra && ks > 3) ? 0 : 4;      // 33 columns beyond d = 11: the stage would not fit 80 KB of LDS
  return (extra && ks > 4) ? 4 : 8;
}

// Waves per workgroup. The kernel is written for four or eight; eight (1024-row blocks, one workgroup per CU) halve
// the atomic adds of the column side, and were measured slower all the same: n = 2^20, d = 11, 16 columns 372.4 ms
// against 368.8, 17 columns 430.6 against 422.1 (whole egp_kmm calls). The adds are off the critical path; what the
// larger workgroup loses is the second, independent workgroup on the CU that keeps the matrix pipe busy while the
// first waits at a stage barrier or converts its column-side sums. So every shape runs four waves, and only those
// instantiations are built.
int sym_waves(int64_t npad, int r, int ks, int nb, int extra) {
  (void)npad;
  (void)r;
  (void)ks;
  (void)nb;
  (void)extra;
  return 4;
}

// stages_total holds the length of one workgroup's sweep; row_blocks the block count
Plan make_plan_sym(int64_t npad, int r, int ks, int nb, int extra) {
  Plan pl;
  pl.big = true;
  pl.sym = true;
  pl.extra_slabs = 2;      // the int64 column-side slab
  pl.waves = sym_waves(npad, r, ks, nb, extra);
  const int rows = 16 * r * pl.waves;
  const int nblk = (int)(npad / rows);
  const int sb = rows / (16 * sym_jt(ks, nb, extra));
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

// Part must hold pl.splits + 2 slabs of npad x (16 nb + extra) floats and kColsideAuxFloats more: the room of the last
// two slabs is the int64 slab of the column-side sums, cleared here, followed by the column sums of |V|, computed here.
int launch_sym(const Prepared& P, const Plan& pl, int nb, int extra, const f4* Vp, const float* Ep, float* Part, int cm,
               hipStream_t stream) {
  ProfScope prof(kProfKmm, stream);
  const size_t slab = (size_t)P.npad * (16 * nb + extra);
  float* cside = Part + (size_t)pl.splits * slab;
  launch_zero_slab(cside, 2 * slab, stream);      // npad is a multiple of 512: a multiple of 4 floats
  launch_col_abs_sums(Vp, Ep, P.npad, nb, extra, cside + 2 * slab, stream);
  switch (P.ks) {
    case 1: return launch_sym_kind<1>(P, pl, nb, extra, Vp, Ep, Part, cm, stream);
    case 2: return launch_sym_kind<2>(P, pl, nb, extra, Vp, Ep, Part, cm, stream);
    case 3: return launch_sym_kind<3>(P, pl, nb, extra, Vp, Ep, Part, cm, stream);
    case 4: return launch_sym_kind<4>(P, pl, nb, extra, Vp, Ep, Part, cm, stream);
    case 5: return launch_sym_kind<5>(P, pl, nb, extra, Vp, Ep, Part, cm, stream);
    case 6: return launch_sym_kind<6>(P, pl, nb, extra, Vp, Ep, Part, cm, stream);
    case 7: return launch_sym_kind<7>(P, pl, nb, extra, Vp, Ep, Part, cm, stream);
    case 8: return launch_sym_kind<8>(P, pl, nb, extra, Vp, Ep, Part, cm, stream);
    default: return fail(EGP_ERR_ARG, "the symmetric kernel supports d <= 31");
  }
}

}  // namespace kmm_detail
}  // namespace egp
