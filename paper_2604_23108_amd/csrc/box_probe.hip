// Measurement aids, not part of the layer: kernels that show what the box delivers, so that the
// fractions the layer's kernels reach can be read against measured ceilings and not only against
// data-sheet peaks.
//   read probe   every byte of a buffer is read exactly once and nothing else happens:
//                - contiguous: a workgroup streams one contiguous stretch;
//                - rows: the access pattern of the decode kernels (a wave owns 32 rows of
//                  `row_bytes`; one wave instruction reads 16 rows x 64 bytes), the waves walking
//                  along their rows in step, or each starting at a different step (staggered);
//   MFMA probe   every wave issues independent chains of v_mfma_f32_32x32x16_bf16 and nothing
//                else: the matrix-core rate the chip sustains under that load.
#include "common.h"

namespace mohge {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kProbeU = 8;                          // 16-byte loads in flight per lane and row set
constexpr int kProbeChunk = 256 * kProbeU;          // uint4 per workgroup iteration (32 KB)

__global__ void __launch_bounds__(256) probe_read_contig(const uint4* __restrict__ p, long long per_block,
                                                         unsigned* out) {
  const uint4* q = p + (long long)blockIdx.x * per_block;        // per_block: a multiple of kProbeChunk
  unsigned acc = 0;
  for (long long i = threadIdx.x; i < per_block; i += kProbeChunk) {
    uint4 v[kProbeU];
#pragma unroll
    for (int u = 0; u < kProbeU; ++u) v[u] = q[i + 256 * u];
#pragma unroll
    for (int u = 0; u < kProbeU; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  if (acc == 0x12345678u) out[0] = acc;              // keeps the loads alive
}

// grid = rows / 128; row_bytes a multiple of 64 * kProbeU
__global__ void __launch_bounds__(256) probe_read_rows(const unsigned char* __restrict__ p, int row_bytes,
                                                       int staggered, unsigned* out) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, r = lane & 15, q = lane >> 4;
  const long long wave = (long long)blockIdx.x * 4 + w;
  const unsigned char* a = p + (wave * 32 + r) * row_bytes + 16 * q;
  const unsigned char* b = p + (wave * 32 + 16 + r) * row_bytes + 16 * q;
  const int nsteps = row_bytes / (64 * kProbeU);
  int st = staggered ? (int)((wave * 5) % nsteps) : 0;
  unsigned acc = 0;
  for (int s = 0; s < nsteps; ++s) {
    const int k = st * 64 * kProbeU;
    uint4 va[kProbeU], vb[kProbeU];
#pragma unroll
    for (int u = 0; u < kProbeU; ++u) {
      va[u] = *reinterpret_cast<const uint4*>(a + k + 64 * u);
      vb[u] = *reinterpret_cast<const uint4*>(b + k + 64 * u);
    }
#pragma unroll
    for (int u = 0; u < kProbeU; ++u)
      acc ^= va[u].x ^ va[u].y ^ va[u].z ^ va[u].w ^ vb[u].x ^ vb[u].y ^ vb[u].z ^ vb[u].w;
    if (++st == nsteps) st = 0;
  }
  if (acc == 0x12345678u) out[0] = acc;
}

constexpr int kMfmaChains = 4;
__global__ void __launch_bounds__(256) probe_mfma(float* out, int iters) {
  bf16x8 a, b;
  // operands with full mantissas, different in every lane (constant small integers would toggle
  // few bits and draw less power than real data)
  for (int i = 0; i < 8; ++i) {
    const unsigned h = (threadIdx.x * 8u + i + blockIdx.x * 2048u) * 2654435761u;
    a[i] = (__bf16)((float)((h >> 9) & 1023u) / 512.f - 1.f);
    b[i] = (__bf16)((float)((h >> 19) & 1023u) / 512.f - 1.f);
  }
  f32x16 acc[kMfmaChains];
  for (int j = 0; j < kMfmaChains; ++j)
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < kMfmaChains; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
  }
  float s = 0.f;
  for (int j = 0; j < kMfmaChains; ++j) s += acc[j][0];
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

// bytes actually read are returned through *bytes_read (0 when the buffer is too small for one unit)
hipError_t launch_probe_read(const void* buf, size_t bytes, int row_bytes, int staggered, void* out,
                             size_t* bytes_read, hipStream_t s) {
  *bytes_read = 0;
  if (row_bytes == 0) {
    const long long chunks = (long long)(bytes / (kProbeChunk * 16));
    if (chunks < 1) return hipSuccess;
    const long long blocks = chunks < 4096 ? chunks : 4096;
    const long long per_block = chunks / blocks * kProbeChunk;             // uint4 per workgroup
    hipLaunchKernelGGL(probe_read_contig, dim3((unsigned)blocks), dim3(256), 0, s,
                       static_cast<const uint4*>(buf), per_block, static_cast<unsigned*>(out));
    *bytes_read = (size_t)(blocks * per_block) * 16;
  } else {
    const long long blocks = (long long)(bytes / row_bytes) / 128;
    if (blocks < 1) return hipSuccess;
    hipLaunchKernelGGL(probe_read_rows, dim3((unsigned)blocks), dim3(256), 0, s,
                       static_cast<const unsigned char*>(buf), row_bytes, staggered, static_cast<unsigned*>(out));
    *bytes_read = (size_t)blocks * 128 * row_bytes;
  }
  return hipGetLastError();
}

hipError_t launch_probe_mfma(void* out, int blocks, int iters, double* flops, hipStream_t s) {
  hipLaunchKernelGGL(probe_mfma, dim3(blocks), dim3(256), 0, s, static_cast<float*>(out), iters);
  *flops = (double)blocks * 4 * kMfmaChains * (double)iters * 2.0 * 32 * 32 * 16;
  return hipGetLastError();
}

}  // namespace mohge
