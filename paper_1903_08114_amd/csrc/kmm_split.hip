// The bf16-split instantiations of the fused kernel (see kmm_kernel.h) and the in-place split of a packed V.
#include "kmm_kernel.h"

namespace egp {
namespace kmm_detail {

// Each packed quad of four fp32 values becomes {hi01, hi23, lo01, lo23}: high parts by truncation to bf16,
// low parts = the exact remainders rounded to bf16.
__global__ __launch_bounds__(256) void split_vp(f4* __restrict__ Vp, int64_t count) {
  const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (g >= count) return;
  const f4 v = Vp[g];
  const unsigned u0 = __float_as_uint(v.x), u1 = __float_as_uint(v.y);
  const unsigned u2 = __float_as_uint(v.z), u3 = __float_as_uint(v.w);
  const f2 l01 = {v.x - __uint_as_float(u0 & 0xffff0000u), v.y - __uint_as_float(u1 & 0xffff0000u)};
  const f2 l23 = {v.z - __uint_as_float(u2 & 0xffff0000u), v.w - __uint_as_float(u3 & 0xffff0000u)};
  f4 o;
  o.x = __uint_as_float(__builtin_amdgcn_perm(u1, u0, 0x07060302u));
  o.y = __uint_as_float(__builtin_amdgcn_perm(u3, u2, 0x07060302u));
  o.z = __uint_as_float(__builtin_bit_cast(unsigned, __builtin_convertvector(l01, bf2)));
  o.w = __uint_as_float(__builtin_bit_cast(unsigned, __builtin_convertvector(l23, bf2)));
  Vp[g] = o;
}

void launch_split_vp(f4* Vp, int64_t count, hipStream_t stream) {
  hipLaunchKernelGGL(split_vp, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, stream, Vp, count);
}

int launch_all_ks_split(const Prepared& P, const Prepared& Q, const Plan& pl, int nb, int extra, const f4* Vp,
                        const float* Ep, float* Part, int cm, hipStream_t stream) {
  return launch_all_ks<1>(P, Q, pl, nb, extra, Vp, Ep, Part, cm, stream);
}

}  // namespace kmm_detail
}  // namespace egp
