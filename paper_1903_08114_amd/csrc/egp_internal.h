// Internal declarations shared by the translation units of libegp (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "egp.h"

namespace egp {

// ---- error plumbing -------------------------------------------------------------------------
int fail(int code, const char* fmt, ...);
#define EGP_HIP(call)                                                                       \
  do {                                                                                      \
    hipError_t e_ = (call);                                                                 \
    if (e_ != hipSuccess)                                                                   \
      return ::egp::fail(EGP_ERR_DEVICE, "%s failed: %s", #call, hipGetErrorString(e_));    \
  } while (0)

inline size_t round_up(size_t x, size_t m) { return (x + m - 1) / m * m; }

// ---- packed operand geometry ----------------------------------------------------------------
// Points are grouped in tiles of 16. A tile of the packed point array holds KS "k-steps" of 64 floats:
// element (s, lane) with lane = 16*q + p is scaled feature 4*s + q of point p of the tile; feature
// index d holds the squared norm of the scaled point, larger indices are zero. This is exactly the
// per-lane operand of one 16x16x4 fp32 MFMA step, for the row side and the column side alike.
constexpr int kTile = 16;
constexpr int kPadPoints = 512;  // packed arrays are padded to a multiple of this many points
inline int ksteps_for(int d) { return (d + 1 + 3) / 4; }
inline int64_t padded_points(int64_t n) { return (int64_t)round_up((size_t)n, kPadPoints); }

// Float offset, inside one 16-point tile of the packed point array, of feature slot f of point pp (0..15).
// Up to 8 k-steps (d <= 31) a tile is [ks][64]: step f/4, lane (f%4)*16 + pp. Beyond that the steps are grouped
// by four, [ks/4][64][4], so that one 128-bit LDS read serves four MFMA steps; the ks%4 left-over steps keep the
// [step][64] form behind the groups.
__host__ __device__ inline int xp_offset(int ks, int f, int pp) {
  const int s = f >> 2, lane = (f & 3) * 16 + pp;
  if (ks <= 8 || s >= (ks & ~3)) return s * 64 + lane;
  return (s >> 2) * 256 + lane * 4 + (s & 3);
}

struct Prepared {   // device arrays carved from a workspace by prepare_points()
  float* Xp;        // [npad/16] tiles of KS*64 floats, element order given by xp_offset()
  float* nrm;       // [npad] squared norms of the scaled points (0 for padding)
  float* mean;      // [d] centre subtracted before scaling
  void* XbC;        // bf16-split column operands (filled in mode EGP_KMM_SPLIT_BF16_ALL only)
  void* XbR;        // bf16-split row operands
  int64_t n, npad;
  int d, ks, kernel_type;
  float outputscale, noise;
  int mode;         // egp_kmm_mode_t of the call that prepared the points; every plan and launch below reads this copy
};

// Options of one library call, fixed at its extern "C" entry point and passed down by value: the arithmetic of the
// fused multiply and whether converged trailing columns leave the solver's iteration. Nothing below the entry points
// reads the process-wide defaults, so a call sees one mode from its workspace layout to its last launch.
struct CallOpts {
  int mode;       // egp_kmm_mode_t
  bool shrink;    // column shrinking in the batched solver
};

size_t prepared_bytes(int64_t n, int d);
// Scale, centre and pack X for kernel `h` into ws (>= prepared_bytes). Asynchronous on stream.
// mean_from: device pointer to the centre of another prepared set (for a second point set), or NULL.
// mode: the call's egp_kmm_mode_t (recorded in *out; the bf16-split operands are packed only in EGP_KMM_SPLIT_BF16_ALL).
int prepare_points(const float* X, int64_t n, const egp_hyper_t* h, void* ws, Prepared* out,
                   hipStream_t stream, int mode, const float* mean_from = nullptr);

// out = Khat V using prepared points. ws2 >= kmm_core_ws_bytes. V/out are row-major n x t.
size_t kmm_core_ws_bytes(int64_t n, int t);
void kmm_plan_splits(int64_t n_rows, int64_t n_cols, int d, int t, int mode, int* used, int* sized);   // host-only planning check
int kmm_core(const Prepared& P, const float* V, int t, float* out, void* ws2, hipStream_t stream);
size_t kmm_cross_ws_bytes(int64_t n_rows, int64_t n_cols, int t);
int kmm_cross(const Prepared& P, const Prepared& Q, const float* V, int t, float* out, void* ws2,
              hipStream_t stream, int64_t v_ld = 0);

void launch_pack_rhs(const float* V, int64_t n, int64_t npad, int t, int c0, int nb_count, int extra, void* Vp,
                     float* Ep, hipStream_t stream);
size_t kmm_grad_core_ws_bytes(int64_t n, int d, int t);
int kmm_grad_core(const Prepared& P, const egp_hyper_t* h, const float* V, int t, float* dout, void* ws2,
                  hipStream_t stream);
size_t bilinear_core_ws_bytes(int64_t n, int d, int t);
int bilinear_core(const Prepared& P, const egp_hyper_t* h, const float* A, const float* B, int t, const float* wcol,
                  double* out, void* ws2, hipStream_t stream);
size_t lanczos_ws_bytes_core(int64_t n, int d, int r);
int lanczos_core(const float* X, int64_t n, const egp_hyper_t* h, const float* b, int r, float* Q, double* alpha,
                 double* beta, int32_t* steps, void* ws, hipStream_t stream, int mode);
size_t cross_ws_bytes_core(int64_t nq, int64_t n, int d, int t);
int cross_core(const float* Xq, int64_t nq, const float* X, int64_t n, const float* V, int t, const egp_hyper_t* h,
               float* out, void* ws, hipStream_t stream, int64_t v_ld, int mode);
size_t predict_ws_bytes_core(int64_t nq, int64_t n, int d, int r);
int predict_core(const float* Xq, int64_t nq, const float* X, int64_t n, const egp_hyper_t* h, const float* a,
                 const float* Q, int r, const double* alpha, const double* beta, float* mean, float* var, void* ws,
                 hipStream_t stream, int mode,
                 const double* Tdense = nullptr, int ldt = 0);
size_t block_lanczos_ws_bytes_core(int64_t n, int d, int b, int blocks);
int block_lanczos_core(const float* X, int64_t n, const egp_hyper_t* h, const float* B0, int b, int blocks, float* Q,
                       double* T, int32_t* rows_out, void* ws, hipStream_t stream, int mode);
size_t pivchol_ws_bytes(int64_t n, int d, int rank);
int pivchol_core(const float* X, int64_t n, const egp_hyper_t* h, float tol_abs, egp_precond_t* P, void* ws,
                 hipStream_t stream);
size_t precond_apply_ws(int64_t n, int t, int rank);
int precond_apply_core(const float* L, int rank, const double* Minv_dev, int64_t n, float noise, const float* R,
                       int t, float* Z, float* rz_partial, void* ws, hipStream_t stream);
int precond_apply_blocks(int64_t n);
// coef_dev / coef_ld (optional): where the k x t coefficients Y of the call live in the workspace afterwards
int precond_apply_cm(const float* L, int rank, const double* Minv_dev, int64_t n, float noise, const float* R,
                     int64_t ld, int t, float* Z, float* rz_part, int part_ld, void* ws, hipStream_t stream,
                     const double** coef_dev = nullptr, int* coef_ld = nullptr);
// G (device, ra x rb doubles) = A B^T over n points; A, B have one row per vector (leading dimensions lda, ldb)
size_t gram_cm_ws_bytes(int64_t n, int ra, int rb);
int gram_cm(const float* A, int ra, int64_t lda, const float* B, int rb, int64_t ldb, int64_t n, double* G_dev,
            void* ws, hipStream_t stream);
// Out[c][i] = sum_m In[m][i] Cf[m][c] for i < n (fp64 sums), zero for n <= i < ld_out; k rows in, t <= 32 rows out
int combine_cm(const float* In, int k, int64_t ld_in, const double* Cf_dev, int t, int64_t n, float* Out,
               int64_t ld_out, hipStream_t stream);
void launch_to_colmajor(const float* src, int64_t n, int t, int64_t ld, float* dst, hipStream_t stream);
int kmm_cm_dot_blocks(int64_t npad);
int kmm_core_cm(const Prepared& P, const float* V, int t, float* out, void* ws2, float* dot_part, int dot_ld,
                hipStream_t stream);
size_t mbcg_ws_bytes_core(int64_t n, int d, int t, int rank, int max_iter);
// co.shrink: trailing columns that have met the tolerance leave the iteration (see egp_mbcg)
int mbcg_core(const float* X, int64_t n, const float* B, int t, const egp_hyper_t* h, const egp_precond_t* P,
              int max_iter, float tol, float* U, double* cg_coef, double* gamma0, int32_t* iters_done,
              float* rel_resid, float* resid_hist, void* ws, hipStream_t stream, const CallOpts& co);

size_t mll_ws_bytes_core(int64_t n, int d, int tp, int rank, int max_iter);
int mll_core(const float* X, int64_t n, const float* y, const float* W1, const float* W2, int tp,
             const egp_hyper_t* h, int rank_req, int max_iter, float tol, egp_mll_result_t* res, void* ws,
             hipStream_t stream, const CallOpts& co);
int train_adam_core(const float* X, int64_t n, const float* y, const float* W1, const float* W2, int tp,
                    egp_hyper_t* h, float* lengthscales_io, int rank, int max_iter, float tol,
                    const egp_adam_t* opt, egp_mll_result_t* last, double* mll_history, void* ws,
                    hipStream_t stream, const CallOpts& co);
}  // namespace egp
#include <vector>
namespace egp {
bool tridiag_log_quadrature(std::vector<double> a, std::vector<double> b, double* result);

// ---- optional in-stream timing of kernel groups with HIP events (egp_profile_*) ----
enum ProfTag { kProfKmm = 0, kProfPack = 1, kProfCgVec = 2, kProfPrecond = 3, kProfPivChol = 4, kProfGrad = 5,
               kProfTags = 6 };
struct ProfScope {   // records an event pair around the launches made during its lifetime
  ProfScope(int tag, hipStream_t stream);
  ~ProfScope();
  int tag_;
  hipStream_t stream_;
  void* slot_;
};

int validate_hyper(const egp_hyper_t* h, int d_max = EGP_D_WIDE_MAX);
int validate_ptr(const void* p, const char* name);

}  // namespace egp
