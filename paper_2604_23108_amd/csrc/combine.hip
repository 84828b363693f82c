// Gated un-permute and combine for gfx950 (appendix, background: y = sum_i G_i(x) E_i(x)).
// Bandwidth-bound: every thread owns 16 bytes of one output row, reads the K_e expert
// rows of its token through inv_perm with 16-byte loads and accumulates in fp32 in slot
// order, so the result does not depend on scheduling.
#include "common.h"

namespace mohge {

template <bool BF16>
__global__ void __launch_bounds__(256) combine_kernel(const uint4* __restrict__ y_perm,
                                                      const int32_t* __restrict__ inv_perm,
                                                      const float* __restrict__ gates,
                                                      uint4* __restrict__ y, int T, int Ke,
                                                      int vec_per_row) {
  const long long total = (long long)T * vec_per_row;
  for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (long long)gridDim.x * blockDim.x) {
    const int t = (int)(idx / vec_per_row), v = (int)(idx % vec_per_row);
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int slot = 0; slot < Ke; ++slot) {
      const float g = gates[(size_t)t * Ke + slot];
      const int r = inv_perm[(size_t)t * Ke + slot];
      const uint4 u = y_perm[(size_t)r * vec_per_row + v];
      if constexpr (BF16) {
        acc[0] = fmaf(g, __uint_as_float(u.x << 16), acc[0]);
        acc[1] = fmaf(g, __uint_as_float(u.x & 0xffff0000u), acc[1]);
        acc[2] = fmaf(g, __uint_as_float(u.y << 16), acc[2]);
        acc[3] = fmaf(g, __uint_as_float(u.y & 0xffff0000u), acc[3]);
        acc[4] = fmaf(g, __uint_as_float(u.z << 16), acc[4]);
        acc[5] = fmaf(g, __uint_as_float(u.z & 0xffff0000u), acc[5]);
        acc[6] = fmaf(g, __uint_as_float(u.w << 16), acc[6]);
        acc[7] = fmaf(g, __uint_as_float(u.w & 0xffff0000u), acc[7]);
      } else {
        acc[0] = fmaf(g, __uint_as_float(u.x), acc[0]);
        acc[1] = fmaf(g, __uint_as_float(u.y), acc[1]);
        acc[2] = fmaf(g, __uint_as_float(u.z), acc[2]);
        acc[3] = fmaf(g, __uint_as_float(u.w), acc[3]);
      }
    }
    uint4 o;
    if constexpr (BF16) {
      o.x = pack_bf16x2(acc[0], acc[1]);
      o.y = pack_bf16x2(acc[2], acc[3]);
      o.z = pack_bf16x2(acc[4], acc[5]);
      o.w = pack_bf16x2(acc[6], acc[7]);
    } else {
      o.x = __float_as_uint(acc[0]);
      o.y = __float_as_uint(acc[1]);
      o.z = __float_as_uint(acc[2]);
      o.w = __float_as_uint(acc[3]);
    }
    y[idx] = o;
  }
}

hipError_t launch_combine(const LayerDesc& L, int dtype, const void* y_perm,
                          const int32_t* inv_perm, const float* gates, void* y, hipStream_t s) {
  const bool bf = dtype == MOHGE_BF16;
  const int vec_per_row = L.d * (bf ? 2 : 4) / 16;
  const long long total = (long long)L.T * vec_per_row;
  long long blocks = (total + 255) / 256;
  if (blocks > 256 * 64) blocks = 256 * 64;
  if (bf)
    hipLaunchKernelGGL((combine_kernel<true>), dim3((unsigned)blocks), dim3(256), 0, s,
                       static_cast<const uint4*>(y_perm), inv_perm, gates, static_cast<uint4*>(y),
                       L.T, L.Ke, vec_per_row);
  else
    hipLaunchKernelGGL((combine_kernel<false>), dim3((unsigned)blocks), dim3(256), 0, s,
                       static_cast<const uint4*>(y_perm), inv_perm, gates, static_cast<uint4*>(y),
                       L.T, L.Ke, vec_per_row);
  return hipGetLastError();
}

}  // namespace mohge
