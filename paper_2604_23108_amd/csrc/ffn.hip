// Expert feed-forward networks: choice of kernel family, workspace size, and the plain
// fp32 kernels used when the layer is stored in fp32.
#include "common.h"
#include "tiled.h"

namespace mohge {

hipError_t launch_ffn_tiled(const LayerDesc& L, const void* x, const int32_t* perm,
                            const int32_t* offsets, const GroupPtrs& W, void* y_perm, void* ws,
                            hipStream_t s, int stages, void* pre, int parts, const FfnOptions& o);
hipError_t launch_ffn_skinny(const LayerDesc& L, const void* x, const int32_t* perm,
                             const int32_t* offsets, const GroupPtrs& W, void* y_perm, void* ws,
                             hipStream_t s, int stages, const float* const* s13, const float* const* s2,
                             const void* const* b13 = nullptr, const void* const* b2 = nullptr);

// ---- fp32: one wave per (sorted row, output element block) ----------------------------
// A wave computes 4 outputs of one row at a time: lanes stride the reduction dimension
// with float4 loads, partial sums are folded with a butterfly, fp32 throughout.
struct F32Args {
  const float* A;
  const int32_t* perm;
  const int32_t* offsets;
  const float* W[kMaxGroups];
  float* C;
  int lda, ldc, Ke, Ng, N, Ne, d, P;
  int F[kMaxGroups];
};

__device__ __forceinline__ float wave_sum_f32(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

__device__ __forceinline__ float dot_wave(const float* a, const float* b, int K, int lane) {
  float s = 0.f;
  for (int k = lane * 4; k < K; k += 256) {
    const float4 u = *reinterpret_cast<const float4*>(a + k);
    const float4 v = *reinterpret_cast<const float4*>(b + k);
    s = fmaf(u.x, v.x, s); s = fmaf(u.y, v.y, s); s = fmaf(u.z, v.z, s); s = fmaf(u.w, v.w, s);
  }
  return wave_sum_f32(s);
}

template <bool UP>
__global__ void __launch_bounds__(256) ffn_f32_kernel(const F32Args a) {
  const int r = blockIdx.x;                       // sorted position
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  // expert of this row: offsets is non-decreasing, Ne <= 256
  int e = 0;
  while (e + 1 < a.Ne && a.offsets[e + 1] <= r) ++e;
  const int g = e / a.N, i = e % a.N, F = a.F[g];
  const int K = UP ? a.d : F, ncols = UP ? F : a.d;
  long long src = r;
  if (UP && a.perm) src = a.perm[r] / a.Ke;
  const float* arow = a.A + src * a.lda;
  float* crow = a.C + (long long)r * a.ldc;
  for (int c = blockIdx.y * 4 + w; c < ncols; c += gridDim.y * 4) {
    if constexpr (UP) {
      const float* Wb = a.W[g] + (long long)i * 2 * F * K;
      const float gt = dot_wave(arow, Wb + (long long)c * K, K, lane);
      const float up = dot_wave(arow, Wb + (long long)(F + c) * K, K, lane);
      if (lane == 0) crow[c] = gt / (1.f + expf(-gt)) * up;
    } else {
      const float* Wb = a.W[g] + (long long)i * a.d * K;
      const float v = dot_wave(arow, Wb + (long long)c * K, K, lane);
      if (lane == 0) crow[c] = v;
    }
  }
}

static hipError_t launch_ffn_f32(const LayerDesc& L, const void* x, const int32_t* perm,
                                 const int32_t* offsets, const GroupPtrs& W, void* y_perm, void* ws,
                                 hipStream_t s, int stages) {
  F32Args up;
  up.A = static_cast<const float*>(x);
  up.perm = perm; up.offsets = offsets;
  up.C = static_cast<float*>(ws);
  up.lda = L.d; up.ldc = L.Fmax; up.Ke = L.Ke; up.Ng = L.Ng; up.N = L.N; up.Ne = L.Ne; up.d = L.d;
  up.P = L.P;
  F32Args dn = up;
  dn.A = static_cast<const float*>(ws);
  dn.perm = nullptr;
  dn.C = static_cast<float*>(y_perm);
  dn.lda = L.Fmax; dn.ldc = L.d;
  for (int g = 0; g < kMaxGroups; ++g) {
    up.F[g] = dn.F[g] = g < L.Ng ? L.F[g] : 0;
    up.W[g] = static_cast<const float*>(W.w13[g]);
    dn.W[g] = static_cast<const float*>(W.w2[g]);
  }
  if (L.P == 0) return hipSuccess;
  if (stages & 1) hipLaunchKernelGGL((ffn_f32_kernel<true>), dim3(L.P, 8), dim3(256), 0, s, up);
  if (stages & 2) hipLaunchKernelGGL((ffn_f32_kernel<false>), dim3(L.P, 8), dim3(256), 0, s, dn);
  return hipGetLastError();
}

static bool use_skinny(const LayerDesc& L) { return L.T <= 32; }

// workspace: the hidden activations h, one row of max F_g per sorted position; the tiled
// matrix-core path keeps its tile schedules in front of them
size_t ffn_workspace_bytes(const LayerDesc& L, int dtype) {
  const size_t elt = dtype == MOHGE_BF16 ? 2 : 4;
  size_t b = (size_t)(L.P > 0 ? L.P : 1) * L.Fmax * elt;
  if (dtype == MOHGE_BF16 && !use_skinny(L)) b += tiled_sched_bytes(L);
  return (b + 255) / 256 * 256;
}

hipError_t launch_expert_ffn(const LayerDesc& L, int dtype, const void* x, const int32_t* perm,
                             const int32_t* offsets, const GroupPtrs& W, void* y_perm, void* ws,
                             hipStream_t s, int stages, int parts, const FfnOptions& o) {
  if (dtype == MOHGE_F32) return launch_ffn_f32(L, x, perm, offsets, W, y_perm, ws, s, stages);
  // With at most 32 tokens no expert can receive more than 32 rows: one pass of the
  // weight-streaming kernel covers it.  Otherwise the tiled matrix-core kernel.
  if (use_skinny(L)) return launch_ffn_skinny(L, x, perm, offsets, W, y_perm, ws, s, stages, nullptr, nullptr);
  return launch_ffn_tiled(L, x, perm, offsets, W, y_perm, ws, s, stages, nullptr, parts, o);
}

size_t ffn_bwd_waiting_header_offset(const LayerDesc& L);

long long fused_flag_offset(const LayerDesc& L, int dtype, int which_call) {
  if (dtype != MOHGE_BF16) return -1;
  switch (which_call) {
    case MOHGE_CALL_EXPERT_FFN: return use_skinny(L) ? -1 : (long long)tiled_waiting_header_offset(L);
    case MOHGE_CALL_FFN_SAVED: return (long long)tiled_waiting_header_offset(L);   // training forward: tile path for every T
    case MOHGE_CALL_EXPERT_FFN_BWD: return (long long)ffn_bwd_waiting_header_offset(L);
    default: return -1;
  }
}

// the schedule and the product launch of the forward can be issued separately only where they
// are two launches: the fused form of the matrix-core path
bool ffn_parts_supported(const LayerDesc& L, int dtype) {
  return dtype == MOHGE_BF16 && !use_skinny(L);
}

// Decode with FP8 E4M3 weights (one fp32 scale per weight row): the weight-streaming kernel only
bool ffn_w8_supported(const LayerDesc& L) { return use_skinny(L); }

hipError_t launch_expert_ffn_w8(const LayerDesc& L, const void* x, const int32_t* perm,
                                const int32_t* offsets, const GroupPtrs& Wq, const float* const* s13,
                                const float* const* s2, void* y_perm, void* ws, hipStream_t s) {
  return launch_ffn_skinny(L, x, perm, offsets, Wq, y_perm, ws, s, 3, s13, s2);
}

// Decode with MXFP4 weights (E2M1 codes, an E8M0 scale per 32 elements of a weight row)
hipError_t launch_expert_ffn_w4(const LayerDesc& L, const void* x, const int32_t* perm,
                                const int32_t* offsets, const GroupPtrs& Wq, const void* const* b13,
                                const void* const* b2, void* y_perm, void* ws, hipStream_t s) {
  return launch_ffn_skinny(L, x, perm, offsets, Wq, y_perm, ws, s, 3, nullptr, nullptr, b13, b2);
}

// Training forward (bf16): what the backward pass needs is kept in `saved`:
//   [tile schedules][h: P x Fmax][backward factors b SiLU'(a) | SiLU(a): P x 2*Fmax]
static size_t saved_pre_offset(const LayerDesc& L) {
  const size_t b = tiled_sched_bytes(L) + (size_t)(L.P > 0 ? L.P : 1) * L.Fmax * 2;
  return (b + 255) / 256 * 256;
}

size_t ffn_saved_bytes(const LayerDesc& L) {
  return saved_pre_offset(L) + ((size_t)(L.P > 0 ? L.P : 1) * 2 * L.Fmax * 2 + 255) / 256 * 256;
}

const void* saved_h(const LayerDesc& L, const void* saved) {
  return static_cast<const unsigned char*>(saved) + tiled_sched_bytes(L);
}

const void* saved_pre(const LayerDesc& L, const void* saved) {
  return static_cast<const unsigned char*>(saved) + saved_pre_offset(L);
}

hipError_t launch_expert_ffn_train(const LayerDesc& L, const void* x, const int32_t* perm,
                                   const int32_t* offsets, const GroupPtrs& W, void* y_perm,
                                   void* saved, hipStream_t s, const FfnOptions& o) {
  void* pre = static_cast<unsigned char*>(saved) + saved_pre_offset(L);
  return launch_ffn_tiled(L, x, perm, offsets, W, y_perm, saved, s, 3, pre, 3, o);
}

}  // namespace mohge
