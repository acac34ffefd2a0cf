// Fused kernel-matrix multiply for gfx950: out = K(X,X) V + noise V with K tiles formed in registers.
//
// Paper, Method, "Partitioned kernel MVMs": a row block of the kernel matrix is formed, multiplied by
// the right-hand side and discarded. Here a "partition" is a 16x16 tile that lives in the accumulator
// registers of one wavefront between two MFMA instructions and never reaches LDS or HBM.
//
// Per 16x16 tile (rows i of a wave's resident row tile, columns j streamed through LDS):
//   1. r^2[j][i] = |x~_i|^2 + |x~_j|^2 - 2 x~_j . x~_i       KS steps of v_mfma_f32_16x16x4_f32
//      (the -2 and |x~_j|^2 are folded into the packed column operand / a spare feature slot,
//       |x~_i|^2 enters as the accumulator's initial value: no VALU work for the distance)
//   2. k = g(r^2)                                             1 (RBF) or 2 (Matern) transcendentals
//   3. out[i][:] += k[i][j] V[j][:]                           4 steps of v_mfma_f32_16x16x4_f32
// Step 1 computes the tile transposed so that its accumulator layout (lane = row i, register r and
// lane group q = column j = 4q + r) is exactly the A-operand layout of step 3; the contraction over j
// is reordered accordingly, which a sum permits. V is pre-packed so that the matching B operand of
// step 3 is one 16-byte LDS read per lane.

#include "kmm_kernel.h"

namespace egp {

using namespace kmm_detail;

// Scale applied to x/l so that the MFMA result is the argument the transform wants:
//   RBF:  acc = r^2 log2(e)/2        k = exp2(-acc)
//   M32:  acc = (sqrt3 r log2 e)^2   a = sqrt(acc), k = (1 + a ln2) exp2(-a)
//   M52:  acc = (sqrt5 r log2 e)^2   a = sqrt(acc), k = (1 + a ln2 + (a ln2)^2/3) exp2(-a)
//   M12:  acc = (r log2 e)^2         a = sqrt(acc), k = exp2(-a)
static double point_scale(int kernel_type) {
  switch (kernel_type) {
    case EGP_RBF: return sqrt(0.5 * 1.4426950408889634);
    case EGP_MATERN32: return sqrt(3.0) * 1.4426950408889634;
    case EGP_MATERN12: return 1.4426950408889634;
    default: return sqrt(5.0) * 1.4426950408889634;
  }
}

// ------------------------------------------------------------------------------------------------
// Row preparation (HBM-bound, O(n d)): column means, then scaled + centred + packed points.
// ------------------------------------------------------------------------------------------------
constexpr int kMeanBlocks = 256;

constexpr int kMeanLd = EGP_D_WIDE_MAX + 1;    // leading dimension of the per-block partial sums

__global__ __launch_bounds__(256) void col_sum_partial(const float* __restrict__ X, int64_t n, int d,
                                                       float* __restrict__ partial /*[blocks][kMeanLd]*/) {
  __shared__ float red[256];
  if (d <= 128) {
    // thread = (point slot, feature): 256 / d points per pass
    const int per = 256 / d;
    const int f = threadIdx.x % d, sub = threadIdx.x / d;
    float acc = 0.f;
    if (sub < per)
      for (int64_t p = (int64_t)blockIdx.x * per + sub; p < n; p += (int64_t)gridDim.x * per) acc += X[p * d + f];
    red[threadIdx.x] = (sub < per) ? acc : 0.f;
    __syncthreads();
    if ((int)threadIdx.x < d) {
      float s = 0.f;
      for (int k = 0; k < per; ++k) s += red[k * d + threadIdx.x];
      partial[blockIdx.x * kMeanLd + threadIdx.x] = s;
    }
  } else {
    // one point per pass, threads stride the features
    for (int f = threadIdx.x; f < d; f += 256) {
      float acc = 0.f;
      for (int64_t p = blockIdx.x; p < n; p += gridDim.x) acc += X[p * d + f];
      partial[blockIdx.x * kMeanLd + f] = acc;
    }
  }
}

// mean[f] = (sum of the per-block partial sums) / n: one wave per feature, lanes stride the blocks.
__global__ __launch_bounds__(256) void col_mean_final(const float* __restrict__ partial, int blocks,
                                                      int64_t n, int d, float* __restrict__ mean) {
  const int lane = threadIdx.x & 63;
  for (int f = threadIdx.x >> 6; f < d; f += 4) {
    double s = 0.0;
    for (int b = lane; b < blocks; b += 64) s += (double)partial[b * kMeanLd + f];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off);
    if (lane == 0) mean[f] = (float)(s / (double)n);
  }
}

struct ScaleArg { float inv[EGP_D_WIDE_MAX + 1]; };

// One thread per (padded) point: x~ = (x - mean) * scale / l, norm = sum x~^2, scattered into the
// packed MFMA-operand layout. Column-side factor -2 is NOT applied here; the kernel's row operand
// carries it (see kmm_kernel).
__global__ __launch_bounds__(256) void pack_points(const float* __restrict__ X, int64_t n, int64_t npad,
                                                   int d, int ks, const float* __restrict__ mean,
                                                   ScaleArg sc, float* __restrict__ Xp,
                                                   float* __restrict__ nrm) {
  int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (p >= npad) return;
  const int64_t tile = p >> 4;
  const int pp = (int)(p & 15);
  float* base = Xp + tile * ks * 64;
  float norm = 0.f;
  const bool real = p < n;
  for (int f = 0; f < ks * 4; ++f) {
    float v = 0.f;
    if (f < d && real) {
      v = (X[p * d + f] - mean[f]) * sc.inv[f];
      norm = __builtin_fmaf(v, v, norm);
    }
    if (f != d) base[xp_offset(ks, f, pp)] = v;
  }
  base[xp_offset(ks, d, pp)] = norm;
  nrm[p] = norm;
}

// V (n x t row-major), columns [c0, c0 + 16*NB) -> Vp[tile][nb][lane][r] = V[16 tile + 4q + r][c0+16nb+p]
// (zero beyond n or beyond t), and optionally column c0 + 16*NB -> Ep[point].
__global__ __launch_bounds__(256) void pack_rhs(const float* __restrict__ V, int64_t n, int64_t npad, int t,
                                                int c0, int nb_count, int extra, f4* __restrict__ Vp,
                                                float* __restrict__ Ep) {
  int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;     // (tile, nb, lane)
  const int64_t total = (npad >> 4) * nb_count * 64;
  if (g < total) {
    const int lane = (int)(g & 63);
    const int64_t tn = g >> 6;
    const int nb = (int)(tn % nb_count);
    const int64_t tile = tn / nb_count;
    const int q = lane >> 4, p = lane & 15;
    const int c = c0 + nb * 16 + p;
    f4 v = {0.f, 0.f, 0.f, 0.f};
    if (c < t) {
      const int64_t j = tile * 16 + q * 4;
      if (j + 0 < n) v.x = V[(j + 0) * t + c];
      if (j + 1 < n) v.y = V[(j + 1) * t + c];
      if (j + 2 < n) v.z = V[(j + 2) * t + c];
      if (j + 3 < n) v.w = V[(j + 3) * t + c];
    }
    Vp[g] = v;
  }
  if (extra && g < npad) {
    const int c = c0 + nb_count * 16;
    Ep[g] = (g < n && c < t) ? V[g * t + c] : 0.f;
  }
}

void launch_pack_rhs(const float* V, int64_t n, int64_t npad, int t, int c0, int nb_count, int extra, void* Vp,
                     float* Ep, hipStream_t stream) {
  const int64_t total = (npad >> 4) * nb_count * 64;
  const int64_t threads = total > npad ? total : npad;
  hipLaunchKernelGGL(pack_rhs, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, stream, V, n, npad, t, c0,
                     nb_count, extra, static_cast<f4*>(Vp), Ep);
}

// out[row][c0 + c] = s * sum_split Part[split][row][c] + noise * V[row][c0 + c]. After a symmetric kernel the
// column-side sums (cside: int64 fixed point [row][c], scale from colsum, see colside_exp) are added as well.
__global__ __launch_bounds__(256) void kmm_epilogue(const float* __restrict__ Part, int splits, int64_t npad,
                                                    int ts, const float* __restrict__ V, int64_t n, int t,
                                                    int c0, int tg, float s, float noise,
                                                    float* __restrict__ out, const long long* __restrict__ cside,
                                                    const unsigned* __restrict__ colsum) {
  int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (g >= n * tg) return;
  const int64_t row = g / tg;
  const int c = (int)(g % tg);
  float acc = 0.f;
  for (int sp = 0; sp < splits; ++sp) acc += Part[((int64_t)sp * npad + row) * ts + c];
  if (cside != nullptr) acc += colside_value(cside[row * ts + c], colside_exp(colsum[c]));
  const int64_t o = row * t + c0 + c;
  out[o] = V ? __builtin_fmaf(s, acc, noise * V[o]) : s * acc;
}

// Column-major variants used by the solver (state arrays are [t][ld], column c contiguous, ld = npad,
// entries beyond n are zero).
// Vp[tile][nb][lane=(q,p)] = V[c0 + 16 nb + p][16 tile + 4q .. +3]: one 16-byte load per lane.
// n_valid < 0: columns are zero-padded to npad and 16-byte aligned (solver state); otherwise entries at
// or beyond n_valid are read as zero with scalar loads (arbitrary ld).
__global__ __launch_bounds__(256) void pack_rhs_cm(const float* __restrict__ V, int64_t ld, int64_t npad, int t,
                                                   int nb_count, f4* __restrict__ Vp, int64_t n_valid) {
  int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t total = (npad >> 4) * nb_count * 64;
  if (g >= total) return;
  const int lane = (int)(g & 63);
  const int64_t tn = g >> 6;
  const int nb = (int)(tn % nb_count);
  const int64_t tile = tn / nb_count;
  const int q = lane >> 4, p = lane & 15;
  const int c = nb * 16 + p;
  f4 v = {0.f, 0.f, 0.f, 0.f};
  if (c < t) {
    const int64_t j = tile * 16 + q * 4;
    const float* src = V + (int64_t)c * ld + j;
    if (n_valid < 0) {
      v = *reinterpret_cast<const f4*>(src);
    } else {
      if (j + 0 < n_valid) v.x = src[0];
      if (j + 1 < n_valid) v.y = src[1];
      if (j + 2 < n_valid) v.z = src[2];
      if (j + 3 < n_valid) v.w = src[3];
    }
  }
  Vp[g] = v;
}

// out[c][row] = s * sum_split Part[split][c][row] + noise * V[c][row]; also per-block partial sums of
// V[c][row] * out[c][row] (the d^T Khat d of CG) into dot_part[c][blockIdx.x]. grid = (blocks, t).
__global__ __launch_bounds__(256) void kmm_epilogue_cm(const float* __restrict__ Part, int splits, int64_t npad,
                                                       int ts, const float* __restrict__ V, int64_t ld, int64_t n,
                                                       float s, float noise, float* __restrict__ out,
                                                       float* __restrict__ dot_part, int dot_ld,
                                                       const long long* __restrict__ cside,
                                                       const unsigned* __restrict__ colsum) {
  __shared__ float red[4];
  const int c = blockIdx.y;
  const int ce = cside != nullptr ? colside_exp(colsum[c]) : 0;
  const float4* v4 = reinterpret_cast<const float4*>(V + (int64_t)c * ld);
  float4* o4 = reinterpret_cast<float4*>(out + (int64_t)c * ld);
  float acc = 0.f;
  for (int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x; g < (npad >> 2); g += (int64_t)gridDim.x * 256) {
    float4 sum = {0.f, 0.f, 0.f, 0.f};
    for (int sp = 0; sp < splits; ++sp) {
      const float4 pv = reinterpret_cast<const float4*>(Part + ((int64_t)sp * ts + c) * npad)[g];
      sum.x += pv.x; sum.y += pv.y; sum.z += pv.z; sum.w += pv.w;
    }
    if (cside != nullptr) {      // column-side sums of a symmetric kernel: int64 fixed point, [c][row]
      const long long* cs = cside + (int64_t)c * npad + g * 4;
      sum.x += colside_value(cs[0], ce);
      sum.y += colside_value(cs[1], ce);
      sum.z += colside_value(cs[2], ce);
      sum.w += colside_value(cs[3], ce);
    }
    const float4 v = v4[g];
    float4 r;
    r.x = __builtin_fmaf(s, sum.x, noise * v.x);
    r.y = __builtin_fmaf(s, sum.y, noise * v.y);
    r.z = __builtin_fmaf(s, sum.z, noise * v.z);
    r.w = __builtin_fmaf(s, sum.w, noise * v.w);
    const int64_t row = g * 4;                 // rows beyond n are padding and must stay zero
    if (row + 3 >= n) {
      if (row + 0 >= n) r.x = 0.f;
      if (row + 1 >= n) r.y = 0.f;
      if (row + 2 >= n) r.z = 0.f;
      r.w = 0.f;
    }
    o4[g] = r;
    acc = __builtin_fmaf(v.x, r.x, acc);
    acc = __builtin_fmaf(v.y, r.y, acc);
    acc = __builtin_fmaf(v.z, r.z, acc);
    acc = __builtin_fmaf(v.w, r.w, acc);
  }
  if (dot_part != nullptr) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) dot_part[(int64_t)c * dot_ld + blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
  }
}

// ------------------------------------------------------------------------------------------------
// Host side
// ------------------------------------------------------------------------------------------------
size_t prepared_bytes(int64_t n, int d) {
  const int64_t npad = padded_points(n);
  const int ks = ksteps_for(d);
  size_t b = 0;
  b += round_up((size_t)npad * ks * 4 * sizeof(float), 256);   // Xp
  b += round_up((size_t)npad * sizeof(float), 256);            // nrm
  b += round_up((size_t)kMeanBlocks * kMeanLd * sizeof(float), 256);  // partial sums
  b += round_up((size_t)kMeanLd * sizeof(float), 256);         // mean
  if (d <= EGP_D_MAX) {                                        // bf16-split operands exist for d <= 31 only
    const int ks16 = (d + 1 + 15) / 16;
    b += round_up((size_t)(npad / 16) * ks16 * 3 * 1024, 256);   // XbC
    b += round_up((size_t)(npad / 16) * ks16 * 2 * 1024, 256);   // XbR
  }
  return b;
}

int prepare_points(const float* X, int64_t n, const egp_hyper_t* h, void* ws, Prepared* out,
                   hipStream_t stream, int mode, const float* mean_from) {
  const int d = h->d;
  const int64_t npad = padded_points(n);
  const int ks = ksteps_for(d);
  char* w = static_cast<char*>(ws);
  out->Xp = reinterpret_cast<float*>(w);
  w += round_up((size_t)npad * ks * 4 * sizeof(float), 256);
  out->nrm = reinterpret_cast<float*>(w);
  w += round_up((size_t)npad * sizeof(float), 256);
  float* partial = reinterpret_cast<float*>(w);
  w += round_up((size_t)kMeanBlocks * kMeanLd * sizeof(float), 256);
  float* mean = reinterpret_cast<float*>(w);
  w += round_up((size_t)kMeanLd * sizeof(float), 256);
  const int ks16 = (d + 1 + 15) / 16;
  out->XbC = w;
  w += round_up((size_t)(npad / 16) * ks16 * 3 * 1024, 256);
  out->XbR = w;
  out->mean = mean;
  out->n = n;
  out->npad = npad;
  out->d = d;
  out->ks = ks;
  out->kernel_type = h->kernel_type;
  out->outputscale = h->outputscale;
  out->noise = h->noise;
  out->mode = mode;

  ScaleArg sc;
  const double c = point_scale(h->kernel_type);
  for (int f = 0; f <= EGP_D_WIDE_MAX; ++f) sc.inv[f] = f < d ? (float)(c / (double)h->lengthscales[f]) : 0.f;

  ProfScope prof(kProfPack, stream);
  if (mean_from != nullptr) {
    // a second point set measured against the first one's centre (distances are invariant to the common shift)
    EGP_HIP(hipMemcpyAsync(mean, mean_from, sizeof(float) * d, hipMemcpyDeviceToDevice, stream));
  } else {
    hipLaunchKernelGGL(col_sum_partial, dim3(kMeanBlocks), dim3(256), 0, stream, X, n, d, partial);
    hipLaunchKernelGGL(col_mean_final, dim3(1), dim3(256), 0, stream, partial, kMeanBlocks, n, d, mean);
  }
  hipLaunchKernelGGL(pack_points, dim3((unsigned)((npad + 255) / 256)), dim3(256), 0, stream, X, n, npad, d,
                     ks, mean, sc, out->Xp, out->nrm);
  if (mode == EGP_KMM_SPLIT_BF16_ALL && d <= EGP_D_MAX) launch_pack_points_bf(*out, stream);
  EGP_HIP(hipGetLastError());
  return EGP_OK;
}

namespace {

// `mode` is the call's own copy of the arithmetic mode (Prepared::mode): planning and launching read the same value.
Plan plan_for_mode(int mode, int64_t npad_rows, int64_t npad_cols, int ks, int d, int nb, int extra,
                   bool square = false) {
  if (ks > 8) {      // d > 31: fp32 wide kernels in every mode, symmetric where that applies unless switched off
    if (mode != EGP_KMM_FP32_ONE_SIDED && square && wide_sym_applies(npad_rows, npad_cols, ks, nb, extra))
      return make_plan_wide_sym(npad_rows, ks, extra);
    return make_plan_wide(npad_rows, npad_cols, ks, nb, extra);
  }
  if (mode == EGP_KMM_FP32) {     // shapes the symmetric kernel does not cover run the one-sided one
    const int r = square ? sym_row_tiles(npad_rows, npad_cols, ks, nb, extra) : 0;
    if (r > 0) return make_plan_sym(npad_rows, r, ks, nb, extra);
    return make_plan(npad_rows, npad_cols, ks, nb, extra);
  }
  if (nb == 0 && mode != EGP_KMM_SPLIT_BF16_ALL)
    return make_plan(npad_rows, npad_cols, ks, nb, extra);     // a single column has no contraction to split
  return mode == EGP_KMM_SPLIT_BF16_ALL ? make_plan_bf(npad_rows, npad_cols, d, nb, extra)
                                        : make_plan(npad_rows, npad_cols, ks, nb, extra);
}
// Upper bound of the column-split count over every launch shape of every mode. Each plan takes
// splits <= min(64, max(1, 1024 / row_blocks), stages_total); a workgroup covers at most 64 * 8 rows and a stage at
// least 16 column points, so row_blocks >= npad_rows / 512 and stages_total <= npad_cols / 16. The partial-sum
// buffer is sized from this bound, not from a list of shapes.
int max_splits(int64_t npad_rows, int64_t npad_cols) {
  const int64_t rb_min = npad_rows / (64 * 8) > 0 ? npad_rows / (64 * 8) : 1;
  int64_t w = 1024 / rb_min;
  if (w < 1) w = 1;
  if (w > 64) w = 64;
  const int64_t s = npad_cols / 16;
  return (int)(w < s ? w : s);
}

// A launch whose plan asks for more splits than the partial-sum buffer holds is refused on the host.
int check_splits(const Plan& pl, int splits_max) {
  if (pl.splits > splits_max)
    return fail(EGP_ERR_WS, "internal: launch plan wants %d column splits, workspace holds %d", pl.splits, splits_max);
  return EGP_OK;
}

int launch_ks(const Prepared& P, const Prepared& Q, const Plan& pl, int nb, int extra, f4* Vp, const float* Ep,
              float* Part, int cm, hipStream_t stream, void* Vb) {
  if (P.ks > 8) {
    if (pl.sym) return launch_wide_sym(P, pl, extra, Vp, Ep, Part, cm, stream);
    return launch_wide(P, Q, pl, nb, extra, Vp, Ep, Part, cm, stream);
  }
  if (pl.sym) return launch_sym(P, pl, nb, extra, Vp, Ep, Part, cm, stream);
  const int mode = P.mode;
  if (nb == 0 && mode != EGP_KMM_SPLIT_BF16_ALL) {
    // a single column has no MFMA contraction to move to bf16: the fp32 kernel serves the contraction-only split mode
    ProfScope prof(kProfKmm, stream);
    return launch_all_ks<0>(P, Q, pl, nb, extra, Vp, Ep, Part, cm, stream);
  }
  if (mode == EGP_KMM_SPLIT_BF16_ALL) return launch_all_bf(P, Q, pl, nb, extra, Vp, Vb, Ep, Part, cm, stream);
  if (mode == EGP_KMM_SPLIT_BF16) {
    {
      ProfScope prof(kProfPack, stream);
      launch_split_vp(Vp, (P.npad >> 4) * nb * 64, stream);
    }
    ProfScope prof(kProfKmm, stream);
    return launch_all_ks_split(P, Q, pl, nb, extra, Vp, Ep, Part, cm, stream);
  }
  ProfScope prof(kProfKmm, stream);
  return launch_all_ks<0>(P, Q, pl, nb, extra, Vp, Ep, Part, cm, stream);
}

}  // namespace

// The next group of right-hand-side columns: nb blocks of 16 through the MFMA contraction, extra = 1 for a 17th /
// 33rd (or, up to d = 31, a lone) column on the VALU.
static void next_group(int rem, int ks, int* nb, int* extra, int* tg) {
  if (rem == 1 && ks <= 8) { *nb = 0; *extra = 1; *tg = 1; }      // a single column: VALU contraction, no MFMA block
  else if (rem <= 16) { *nb = 1; *extra = 0; *tg = rem; }
  else if (rem == 17) { *nb = 1; *extra = 1; *tg = 17; }
  else if (rem <= 32) { *nb = 2; *extra = 0; *tg = rem; }
  else if (rem == 33) { *nb = 2; *extra = 1; *tg = 33; }
  else { *nb = 2; *extra = 0; *tg = 32; }
}

// Host-only check of the launch planning (no GPU work): the largest column-split count that a product of these
// sizes launches with in mode `mode`, row-major and (t <= 33, square) column-major entry alike, and the count
// its workspace holds.
void kmm_plan_splits(int64_t n_rows, int64_t n_cols, int d, int t, int mode, int* used, int* sized) {
  const int64_t prow = padded_points(n_rows), pcol = padded_points(n_cols);
  const int ks = ksteps_for(d);
  int worst = 0;
  for (int c0 = 0; c0 < t;) {
    int nb, extra, tg;
    next_group(t - c0, ks, &nb, &extra, &tg);
    const int s = plan_for_mode(mode, prow, pcol, ks, d, nb, extra, prow == pcol).splits;
    if (s > worst) worst = s;
    c0 += tg;
  }
  if (t <= 33 && prow == pcol) {
    const bool single = t == 1 && ks <= 8;
    const int nb = single ? 0 : (t > 17 ? 2 : 1), extra = (single || t == 17 || t == 33) ? 1 : 0;
    const int s = plan_for_mode(mode, prow, pcol, ks, d, nb, extra, true).splits;
    if (s > worst) worst = s;
  }
  *used = worst;
  *sized = max_splits(prow, pcol);
}

static int widest_ts(int t) { return t <= 16 ? 16 : (t == 17 ? 17 : (t <= 32 ? 32 : 33)); }

size_t kmm_cross_ws_bytes(int64_t n_rows, int64_t n_cols, int t) {
  const int64_t prow = padded_points(n_rows), pcol = padded_points(n_cols);
  // the split count depends on the shape class only; take the larger of the fp32 and the all-bf16 plans
  const int splits = max_splits(prow, pcol);
  const int nb = t > 17 ? 2 : 1;
  size_t b = 0;
  b += round_up((size_t)pcol * nb * 16 * sizeof(float), 256);                    // Vp
  b += round_up((size_t)pcol * sizeof(float), 256);                              // Ep
  // Part (+2 slabs and the column maxima: column-side region of the symmetric kernels)
  b += round_up(((size_t)(splits + 2) * prow * widest_ts(t) + kmm_detail::kColsideAuxFloats) * sizeof(float), 256);
  b += round_up((size_t)pcol * nb * 32 * sizeof(float), 256);                    // split V of the all-bf16 mode
  return b;
}

size_t kmm_core_ws_bytes(int64_t n, int t) { return kmm_cross_ws_bytes(n, n, t); }

int kmm_core(const Prepared& P, const float* V, int t, float* out, void* ws2, hipStream_t stream) {
  return kmm_cross(P, P, V, t, out, ws2, stream, 0);
}

// out (Q.n x t, row-major) = K(Q points, P points) V; the noise term is added only when Q and P are the same
// set. V is P.n x t row-major, or, when v_ld > 0, stored by columns: column c at V + c * v_ld (P.n entries).
int kmm_cross(const Prepared& P, const Prepared& Q, const float* V, int t, float* out, void* ws2,
              hipStream_t stream, int64_t v_ld) {
  const int64_t npad = P.npad;
  const bool square = Q.Xp == P.Xp;
  const int splits_max = max_splits(Q.npad, npad);
  char* w = static_cast<char*>(ws2);
  const int tg_max = t > 33 ? 33 : t;
  const int nb_max = tg_max > 17 ? 2 : 1;
  f4* Vp = reinterpret_cast<f4*>(w);
  w += round_up((size_t)npad * nb_max * 16 * sizeof(float), 256);
  float* Ep = reinterpret_cast<float*>(w);
  w += round_up((size_t)npad * sizeof(float), 256);
  float* Part = reinterpret_cast<float*>(w);
  w += round_up(((size_t)(splits_max + 2) * Q.npad * widest_ts(t) + kColsideAuxFloats) * sizeof(float), 256);
  void* Vb = w;

  int c0 = 0;
  while (c0 < t) {
    const int rem = t - c0;
    int nb, extra, tg;
    next_group(rem, P.ks, &nb, &extra, &tg);
    const int ts = 16 * nb + extra;
    const Plan pl = plan_for_mode(P.mode, Q.npad, npad, P.ks, P.d, nb, extra, square);
    if (int rc = check_splits(pl, splits_max)) return rc;
    if (v_ld > 0) {
      // columns stored one after the other (e.g. Lanczos vectors): 16 columns per block, the odd one as Ep
      ProfScope prof(kProfPack, stream);
      const int64_t total = (npad >> 4) * nb * 64;
      if (nb > 0)
        hipLaunchKernelGGL(pack_rhs_cm, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, V + c0 * v_ld, v_ld,
                           npad, tg - extra, nb, Vp, P.n);
      if (extra) {
        launch_zero_slab(Ep, (size_t)npad, stream);      // a fill kernel, not a memset node (the stream may be captured)
        EGP_HIP(hipMemcpyAsync(Ep, V + (int64_t)(c0 + tg - 1) * v_ld, P.n * sizeof(float), hipMemcpyDeviceToDevice,
                               stream));
      }
    } else {
      ProfScope prof(kProfPack, stream);
      launch_pack_rhs(V, P.n, npad, t, c0, nb, extra, Vp, Ep, stream);
    }
    const int rc = launch_ks(P, Q, pl, nb, extra, Vp, Ep, Part, 0, stream, Vb);
    if (rc != EGP_OK) return rc;
    const int64_t outs = Q.n * tg;
    ProfScope eprof(kProfPack, stream);
    const float* cside = Part + (size_t)pl.splits * Q.npad * ts;      // behind the row-side slabs (symmetric kernels)
    hipLaunchKernelGGL(kmm_epilogue, dim3((unsigned)((outs + 255) / 256)), dim3(256), 0, stream, Part, pl.splits,
                       Q.npad, ts, square ? V : nullptr, Q.n, t, c0, tg, P.outputscale, square ? P.noise : 0.f, out,
                       pl.sym ? reinterpret_cast<const long long*>(cside) : nullptr,
                       reinterpret_cast<const unsigned*>(cside + 2 * (size_t)Q.npad * ts));
    EGP_HIP(hipGetLastError());
    c0 += tg;
  }
  return EGP_OK;
}

// Column-major variant for the solver: V and out are [t][ld] with ld = P.npad (zero beyond n), t <= 33.
// dot_part (optional) receives kmm_cm_dot_blocks() partial sums of V[c].out[c] per column, leading
// dimension dot_ld.
int kmm_cm_dot_blocks(int64_t npad) {
  int64_t b = (npad / 4 + 255) / 256;
  return (int)(b > 64 ? 64 : b);
}

int kmm_core_cm(const Prepared& P, const float* V, int t, float* out, void* ws2, float* dot_part, int dot_ld,
                hipStream_t stream) {
  const int64_t npad = P.npad;
  const int splits_max = max_splits(npad, npad);
  char* w = static_cast<char*>(ws2);
  const bool single = t == 1 && P.ks <= 8;      // one column: consumed straight from the state array on the VALU
  const int nb = single ? 0 : (t > 17 ? 2 : 1);
  const int extra = (single || t == 17 || t == 33) ? 1 : 0;
  const Plan pl = plan_for_mode(P.mode, npad, npad, P.ks, P.d, nb, extra, true);
  if (int rc = check_splits(pl, splits_max)) return rc;
  const int ts = 16 * nb + extra;
  f4* Vp = reinterpret_cast<f4*>(w);
  w += round_up((size_t)npad * (nb > 0 ? nb : 1) * 16 * sizeof(float), 256);
  w += round_up((size_t)npad * sizeof(float), 256);      // the row-major path's extra-column buffer (unused here)
  float* Part = reinterpret_cast<float*>(w);
  w += round_up(((size_t)(splits_max + 2) * npad * widest_ts(t) + kColsideAuxFloats) * sizeof(float), 256);
  void* Vb = w;
  if (nb > 0) {
    ProfScope prof(kProfPack, stream);
    const int64_t total = (npad >> 4) * nb * 64;
    hipLaunchKernelGGL(pack_rhs_cm, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, V, npad, npad,
                       extra ? t - 1 : t, nb, Vp, (int64_t)-1);
  }
  // the 17th / 33rd column is consumed straight from the state array
  const float* Ep = extra ? V + (int64_t)(t - 1) * npad : nullptr;
  const int rc = launch_ks(P, P, pl, nb, extra, Vp, Ep, Part, 1, stream, Vb);
  if (rc != EGP_OK) return rc;
  ProfScope eprof(kProfPack, stream);
  const float* cside = Part + (size_t)pl.splits * npad * ts;      // behind the row-side slabs (symmetric kernels)
  hipLaunchKernelGGL(kmm_epilogue_cm, dim3(kmm_cm_dot_blocks(npad), t), dim3(256), 0, stream, Part, pl.splits, npad,
                     ts, V, npad, P.n, P.outputscale, P.noise, out, dot_part, dot_ld,
                     pl.sym ? reinterpret_cast<const long long*>(cside) : nullptr,
                     reinterpret_cast<const unsigned*>(cside + 2 * (size_t)npad * ts));
  EGP_HIP(hipGetLastError());
  return EGP_OK;
}

}  // namespace egp
