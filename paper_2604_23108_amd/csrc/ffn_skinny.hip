// Expert feed-forward networks for decode-sized token counts on gfx950 (a handful of
// tokens per expert): bandwidth-bound, every touched expert's weights are streamed once.
//
// A wave owns 2 x 16 weight rows (up: 16 W_gate rows and the matching 16 W_up rows;
// down: 32 consecutive W_down rows) and runs over the whole reduction dimension with
// v_mfma_f32_16x16x32_bf16, the weight rows as the first operand and up to 32 of the
// expert's tokens as the second.  Lanes load 16 contiguous bytes of "their" weight row,
// which is the operand layout, so weights go global -> registers -> matrix core with no
// LDS traffic; token rows come through L1/L2 (lanes past the token count load nothing).
// Experts without tokens are skipped on the device: their workgroups exit at once.
#include <type_traits>

#include "common.h"

namespace mohge {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

struct SkinnyArgs {
  const uint16_t* A;              // up: x; down: H
  const int32_t* perm;            // up only, may be NULL
  const int32_t* offsets;
  const uint16_t* W[kMaxGroups];
  uint16_t* C;
  int lda, ldc, Ke, Ng, N, d;
  int F[kMaxGroups];
  int blk_prefix[kMaxGroups + 1]; // first workgroup of each group
};

union Frag {
  uint4 u;
  bf16x8 v;
};

template <bool UP>
__global__ void __launch_bounds__(256) ffn_skinny_kernel(const SkinnyArgs a) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int r = lane & 15, q = lane >> 4;
  int g = 0;
  while (g + 1 < a.Ng && (int)blockIdx.x >= a.blk_prefix[g + 1]) ++g;
  const int F = a.F[g];
  const int K = UP ? a.d : F;
  const int ncols = UP ? F : a.d;
  // workgroup = 4 waves; up: 64 hidden units; down: 128 output features
  constexpr int COLS_PER_BLOCK = UP ? 64 : 128;
  const int blocks_per_expert = (ncols + COLS_PER_BLOCK - 1) / COLS_PER_BLOCK;
  const int local = blockIdx.x - a.blk_prefix[g];
  const int i = local / blocks_per_expert, cb = local % blocks_per_expert;
  const int e = g * a.N + i;
  const int row0 = a.offsets[e], cnt = a.offsets[e + 1] - row0;
  if (cnt <= 0) return;
  const int c0 = cb * COLS_PER_BLOCK + w * (UP ? 16 : 32);
  if (c0 >= ncols) return;

  // the two weight-row sets of this wave
  const uint16_t* wp[2];
  if constexpr (UP) {
    const uint16_t* base = a.W[g] + (long long)i * 2 * F * K;
    wp[0] = base + (long long)(c0 + r) * K + 8 * q;
    wp[1] = base + (long long)(F + c0 + r) * K + 8 * q;
  } else {
    const uint16_t* base = a.W[g] + (long long)i * a.d * K;
    int n1 = c0 + 16 + r;
    if (n1 > a.d - 1) n1 = a.d - 1;
    wp[0] = base + (long long)(c0 + r) * K + 8 * q;
    wp[1] = base + (long long)n1 * K + 8 * q;
  }

  for (int tb0 = 0; tb0 < cnt; tb0 += 32) {
    const uint16_t* xp[2];
    bool xv[2];
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
      const int tt = tb0 + 16 * tb + r;
      xv[tb] = tt < cnt;
      const int pos = row0 + (xv[tb] ? tt : 0);
      long long src;
      if constexpr (UP) src = a.perm ? (long long)(a.perm[pos] / a.Ke) : (long long)pos;
      else src = pos;
      xp[tb] = a.A + src * a.lda + 8 * q;
    }
    f32x4 acc[2][2];
#pragma unroll
    for (int f = 0; f < 2; ++f)
#pragma unroll
      for (int tb = 0; tb < 2; ++tb) acc[f][tb] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto step = [&](int k0, auto UC) {
      constexpr int U = decltype(UC)::value;
      Frag wf[2][U], xf[2][U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
#pragma unroll
        for (int f = 0; f < 2; ++f) wf[f][u].u = *reinterpret_cast<const uint4*>(wp[f] + k0 + 32 * u);
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) {
          xf[tb][u].u = make_uint4(0u, 0u, 0u, 0u);
          if (xv[tb]) xf[tb][u].u = *reinterpret_cast<const uint4*>(xp[tb] + k0 + 32 * u);
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int f = 0; f < 2; ++f)
#pragma unroll
          for (int tb = 0; tb < 2; ++tb)
            acc[f][tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[f][u].v, xf[tb][u].v, acc[f][tb], 0, 0, 0);
    };
    int k0 = 0;
    for (; k0 + 256 <= K; k0 += 256) step(k0, std::integral_constant<int, 8>{});
    for (; k0 + 128 <= K; k0 += 128) step(k0, std::integral_constant<int, 4>{});
    for (; k0 < K; k0 += 64) step(k0, std::integral_constant<int, 2>{});

    // lane holds token r of each token block, weight rows 4q..4q+3 of each row set
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
      const int tt = tb0 + 16 * tb + r;
      if (tt >= cnt) continue;
      uint16_t* crow = a.C + (long long)(row0 + tt) * a.ldc;
      if constexpr (UP) {
        float v[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          const float gt = acc[0][tb][b], up = acc[1][tb][b];
          v[b] = gt / (1.f + __expf(-gt)) * up;
        }
        uint2 o;
        o.x = pack_bf16x2(v[0], v[1]);
        o.y = pack_bf16x2(v[2], v[3]);
        *reinterpret_cast<uint2*>(crow + c0 + 4 * q) = o;
      } else {
#pragma unroll
        for (int f = 0; f < 2; ++f) {
          const int col = c0 + 16 * f + 4 * q;
          if (col < ncols) {
            uint2 o;
            o.x = pack_bf16x2(acc[f][tb][0], acc[f][tb][1]);
            o.y = pack_bf16x2(acc[f][tb][2], acc[f][tb][3]);
            *reinterpret_cast<uint2*>(crow + col) = o;
          }
        }
      }
    }
  }
}

hipError_t launch_ffn_skinny(const LayerDesc& L, const void* x, const int32_t* perm,
                             const int32_t* offsets, const GroupPtrs& W, void* y_perm, void* ws,
                             hipStream_t s, int stages) {
  SkinnyArgs up;
  up.A = static_cast<const uint16_t*>(x);
  up.perm = perm;
  up.offsets = offsets;
  up.C = static_cast<uint16_t*>(ws);
  up.lda = L.d; up.ldc = L.Fmax; up.Ke = L.Ke; up.Ng = L.Ng; up.N = L.N; up.d = L.d;
  SkinnyArgs dn = up;
  dn.A = static_cast<const uint16_t*>(ws);
  dn.perm = nullptr;
  dn.C = static_cast<uint16_t*>(y_perm);
  dn.lda = L.Fmax; dn.ldc = L.d;
  int nu = 0, nd = 0;
  for (int g = 0; g < kMaxGroups; ++g) {
    up.F[g] = dn.F[g] = g < L.Ng ? L.F[g] : 0;
    up.W[g] = static_cast<const uint16_t*>(W.w13[g]);
    dn.W[g] = static_cast<const uint16_t*>(W.w2[g]);
    up.blk_prefix[g] = nu;
    dn.blk_prefix[g] = nd;
    if (g < L.Ng) {
      nu += L.N * (L.F[g] / 64);
      nd += L.N * ((L.d + 127) / 128);
    }
  }
  up.blk_prefix[kMaxGroups] = nu;
  dn.blk_prefix[kMaxGroups] = nd;
  if (stages & 1) hipLaunchKernelGGL((ffn_skinny_kernel<true>), dim3(nu), dim3(256), 0, s, up);
  if (stages & 2) hipLaunchKernelGGL((ffn_skinny_kernel<false>), dim3(nd), dim3(256), 0, s, dn);
  return hipGetLastError();
}

}  // namespace mohge
