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
                                                      const uint4* y_add, uint4* y, int T, int Ke,
                                                      int vec_per_row) {
  const long long total = (long long)T * vec_per_row;
  for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (long long)gridDim.x * blockDim.x) {
    const int t = (int)(idx / vec_per_row), v = (int)(idx % vec_per_row);
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (y_add) {          // the term added to the gated sum (may be y itself: read before written)
      const uint4 u = y_add[idx];
      if constexpr (BF16) {
        acc[0] = __uint_as_float(u.x << 16); acc[1] = __uint_as_float(u.x & 0xffff0000u);
        acc[2] = __uint_as_float(u.y << 16); acc[3] = __uint_as_float(u.y & 0xffff0000u);
        acc[4] = __uint_as_float(u.z << 16); acc[5] = __uint_as_float(u.z & 0xffff0000u);
        acc[6] = __uint_as_float(u.w << 16); acc[7] = __uint_as_float(u.w & 0xffff0000u);
      } else {
        acc[0] = __uint_as_float(u.x); acc[1] = __uint_as_float(u.y);
        acc[2] = __uint_as_float(u.z); acc[3] = __uint_as_float(u.w);
      }
    }
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
                          const int32_t* inv_perm, const float* gates, const void* y_add, void* y,
                          hipStream_t s) {
  const bool bf = dtype == MOHGE_BF16;
  const int vec_per_row = L.d * (bf ? 2 : 4) / 16;
  const long long total = (long long)L.T * vec_per_row;
  long long blocks = (total + 255) / 256;
  if (blocks > 256 * 64) blocks = 256 * 64;
  if (bf)
    hipLaunchKernelGGL((combine_kernel<true>), dim3((unsigned)blocks), dim3(256), 0, s,
                       static_cast<const uint4*>(y_perm), inv_perm, gates,
                       static_cast<const uint4*>(y_add), static_cast<uint4*>(y), L.T, L.Ke, vec_per_row);
  else
    hipLaunchKernelGGL((combine_kernel<false>), dim3((unsigned)blocks), dim3(256), 0, s,
                       static_cast<const uint4*>(y_perm), inv_perm, gates,
                       static_cast<const uint4*>(y_add), static_cast<uint4*>(y), L.T, L.Ke, vec_per_row);
  return hipGetLastError();
}

// Routing of always-on ("shared") experts: every token goes to every one of the N experts of
// the single group with gate 1.  Sorted position r = s*T + t <-> pair p = t*N + s.
__global__ void __launch_bounds__(256) shared_routing_kernel(int T, int N, int32_t* expert_idx,
                                                             float* gates, int32_t* counts,
                                                             int32_t* offsets, int32_t* perm,
                                                             int32_t* inv_perm) {
  const long long P = (long long)T * N;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < P; i += (long long)gridDim.x * 256) {
    const int t_of_p = (int)(i / N), s_of_p = (int)(i % N);     // i as pair id
    expert_idx[i] = s_of_p;
    gates[i] = 1.f;
    inv_perm[i] = s_of_p * T + t_of_p;
    const int s_of_r = (int)(i / T), t_of_r = (int)(i % T);     // i as sorted position
    perm[i] = t_of_r * N + s_of_r;
  }
  if (blockIdx.x == 0)
    for (int i = threadIdx.x; i <= N; i += 256) {      // N can equal the block size
      offsets[i] = i * T;
      if (i < N) counts[i] = T;
    }
}

hipError_t launch_shared_routing(const LayerDesc& L, int32_t* expert_idx, float* gates,
                                 int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv_perm,
                                 hipStream_t s) {
  long long blocks = ((long long)L.P + 255) / 256;
  if (blocks < 1) blocks = 1;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(shared_routing_kernel, dim3((unsigned)blocks), dim3(256), 0, s, L.T, L.N, expert_idx,
                     gates, counts, offsets, perm, inv_perm);
  return hipGetLastError();
}

}  // namespace mohge

// ---------------------------------------------------------------------------------------
// backward of the gated combine (bf16):  y_t = sum_slot gate[t,slot] * y_perm[r(t,slot)]
//   dgates[t,slot] = <dy_t, y_perm[r]>,   dy_perm[r] = gate[t,slot] * dy_t
// One wave per token; lanes stride the row in 16-byte chunks; the dot product is folded with a
// butterfly, so the result does not depend on scheduling.
// ---------------------------------------------------------------------------------------
namespace mohge {

__global__ void __launch_bounds__(256) combine_bwd_kernel(const uint4* __restrict__ dy,
                                                          const uint4* __restrict__ y_perm,
                                                          const int32_t* __restrict__ inv_perm,
                                                          const float* __restrict__ gates,
                                                          float* __restrict__ dgates,
                                                          uint4* __restrict__ dy_perm, int T, int Ke,
                                                          int vec_per_row) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  for (int slot = 0; slot < Ke; ++slot) {
    const float g = gates[(size_t)t * Ke + slot];
    const int r = inv_perm[(size_t)t * Ke + slot];
    float dot = 0.f;
    for (int v = lane; v < vec_per_row; v += 64) {
      const uint4 a = dy[(size_t)t * vec_per_row + v];
      const uint4 b = y_perm[(size_t)r * vec_per_row + v];
      const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
      uint32_t ow[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float a0 = __uint_as_float(aw[i] << 16), a1 = __uint_as_float(aw[i] & 0xffff0000u);
        const float b0 = __uint_as_float(bw[i] << 16), b1 = __uint_as_float(bw[i] & 0xffff0000u);
        dot = fmaf(a0, b0, dot);
        dot = fmaf(a1, b1, dot);
        ow[i] = pack_bf16x2(g * a0, g * a1);
      }
      dy_perm[(size_t)r * vec_per_row + v] = make_uint4(ow[0], ow[1], ow[2], ow[3]);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) dot += __shfl_xor(dot, off, 64);
    if (lane == 0) dgates[(size_t)t * Ke + slot] = dot;
  }
}

hipError_t launch_combine_bwd(const LayerDesc& L, const void* dy, const void* y_perm,
                              const int32_t* inv_perm, const float* gates, float* dgates,
                              void* dy_perm, hipStream_t s) {
  const int vec_per_row = L.d * 2 / 16;
  hipLaunchKernelGGL(combine_bwd_kernel, dim3((unsigned)((L.T + 3) / 4)), dim3(256), 0, s,
                     static_cast<const uint4*>(dy), static_cast<const uint4*>(y_perm), inv_perm, gates,
                     dgates, static_cast<uint4*>(dy_perm), L.T, L.Ke, vec_per_row);
  return hipGetLastError();
}

}  // namespace mohge
