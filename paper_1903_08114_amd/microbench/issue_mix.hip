// Instruction-mix microbenchmark for gfx950: which instruction classes co-execute on one SIMD?
//
// Each wave runs `iters` iterations of a fixed mix of independent instructions: bf16 MFMA (16x16x16),
// fp32 MFMA (16x16x4), plain VALU (v_fma_f32) and transcendental (v_exp_f32). With 1 or 2 waves per
// SIMD on all 256 CUs, the time per iteration shows whether the classes overlap or add. The fused
// kernel-matrix multiply is priced against these figures (fp32 MFMA time and VALU time add).
//
// Build: python -m paper_1903_08114_amd.build   (produces paper_1903_08114_amd/microbench/issue_mix)
// Run:   ./paper_1903_08114_amd/microbench/issue_mix
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>
typedef float f4 __attribute__((ext_vector_type(4)));
typedef short s4 __attribute__((ext_vector_type(4)));
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s line %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)
#define MF32(a, b, c) __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0)
#define MBF(a, b, c) __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, b, c, 0, 0, 0)

// per iteration: NB bf16 MFMAs, NF fp32 MFMAs, NV v_fma, NE v_exp, all on independent registers
template <int NB, int NF, int NV, int NE>
__global__ __launch_bounds__(256) void mix(float* out, int iters, float seed) {
  const int lane = threadIdx.x & 63;
  f4 ab[8], af[8];
  float ev[32], ex[16];
  s4 a = {(short)(lane + 1), (short)(lane + 2), (short)(lane + 3), (short)(lane + 4)};
  s4 b = {(short)(lane + 5), (short)(lane + 6), (short)(lane + 7), (short)(lane + 8)};
  float fa = seed + lane, fb = 0.5f + lane;
#pragma unroll
  for (int i = 0; i < 8; ++i) { ab[i] = (f4){0.f, 0.f, 0.f, 0.f}; af[i] = (f4){0.f, 0.f, 0.f, 0.f}; }
#pragma unroll
  for (int i = 0; i < 32; ++i) ev[i] = seed * i;
#pragma unroll
  for (int i = 0; i < 16; ++i) ex[i] = seed * i;
  for (int it = 0; it < iters; ++it) {
    fa += 1e-7f;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
#pragma unroll
      for (int i = 0; i < NB / 8; ++i) ab[(r + i) & 7] = MBF(a, b, ab[(r + i) & 7]);
#pragma unroll
      for (int i = 0; i < NF / 8; ++i) af[(r + i) & 7] = MF32(fa, fb, af[(r + i) & 7]);
#pragma unroll
      for (int i = 0; i < NV / 8; ++i) ev[(r * (NV / 8) + i) & 31] = __builtin_fmaf(ev[(r * (NV / 8) + i) & 31], 0.999f, fb);
#pragma unroll
      for (int i = 0; i < NE / 8; ++i) ex[(r * (NE / 8) + i) & 15] = __builtin_amdgcn_exp2f(-ex[(r * (NE / 8) + i) & 15]);
    }
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) s += ab[i].x + ab[i].w + af[i].x + af[i].y;
#pragma unroll
  for (int i = 0; i < 32; ++i) s += ev[i];
#pragma unroll
  for (int i = 0; i < 16; ++i) s += ex[i];
  out[blockIdx.x * 256 + threadIdx.x] = s;
}

template <int NB, int NF, int NV, int NE>
void run(int wps, float* out) {
  const int iters = 20000;
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  hipLaunchKernelGGL((mix<NB, NF, NV, NE>), dim3(256 * wps), dim3(256), 0, 0, out, 100, 1e-9f);
  CK(hipDeviceSynchronize());
  CK(hipEventRecord(e0));
  hipLaunchKernelGGL((mix<NB, NF, NV, NE>), dim3(256 * wps), dim3(256), 0, 0, out, iters, 1e-9f);
  CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
  float ms; CK(hipEventElapsedTime(&ms, e0, e1));
  const double cyc = ms * 1e-3 * 2.4e9 / ((double)iters * wps);
  printf("waves/SIMD %d  bf16-mfma %3d  f32-mfma %3d  v_fma %3d  v_exp %3d : %8.1f cycles/iter\n", wps, NB, NF, NV, NE, cyc);
  fflush(stdout);
}

int main() {
  float* out; CK(hipMalloc(&out, 256 * 8 * 256 * 4));
  for (int w = 1; w <= 2; ++w) {
    run<32, 0, 0, 0>(w, out);     // bf16 MFMA alone
    run<0, 32, 0, 0>(w, out);     // fp32 MFMA alone
    run<0, 56, 0, 0>(w, out);     // the fused kernel's MFMA count for 8 tiles
    run<32, 32, 0, 0>(w, out);    // both MFMA kinds
    run<0, 0, 64, 0>(w, out);     // VALU alone
    run<0, 0, 0, 32>(w, out);     // transcendental alone
    run<32, 0, 64, 0>(w, out);    // bf16 MFMA + VALU
    run<32, 0, 0, 32>(w, out);    // bf16 MFMA + transcendental
    run<0, 32, 64, 0>(w, out);    // fp32 MFMA + VALU
    run<0, 32, 0, 32>(w, out);    // fp32 MFMA + transcendental
    run<0, 56, 0, 32>(w, out);    // the fused kernel's mix for 8 tiles (RBF)
  }
  return 0;
}
