// Arguments and the per-workgroup unit of the bf16 decode kernels of the expert networks (a
// handful of tokens per expert: every touched expert's weights are streamed once), shared by the
// two-launch form and the single-launch decode layer.
#pragma once
#include <type_traits>

#include "common.h"

namespace mohge {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

struct SkinnyArgs {
  const uint16_t* A;              // up: x; down: H
  const int32_t* perm;            // up only, may be NULL
  const int32_t* offsets;
  const uint16_t* W[kMaxGroups];  // bf16 weights, or E4M3 codes (W8)
  const float* S[kMaxGroups];     // W8: scale per weight row, same row order as W
  const uint8_t* S4[kMaxGroups];  // W4: E8M0 scale per 32 elements of a weight row, [rows][K/32]
  uint16_t* C;
  int lda, ldc, Ke, Ng, N, d;
  int F[kMaxGroups];
  int blk_prefix[kMaxGroups + 1]; // first workgroup of each group
};

// host: argument blocks of the up and the down launch, nu / nd workgroups (one per unit); s13/s2:
// FP8 row scales or NULL, b13/b2: MXFP4 block scales or NULL
void skinny_args(const LayerDesc& L, const void* x, const int32_t* perm, const int32_t* offsets,
                 const GroupPtrs& W, void* y_perm, void* h, const float* const* s13, const float* const* s2,
                 const void* const* b13, const void* const* b2, SkinnyArgs& up, SkinnyArgs& dn, int& nu, int& nd);

union Frag {
  uint4 u;
  bf16x8 v;
};

// 8-byte store performed at device scope (written through the XCD's L2): once the store has
// completed (vmcnt), a workgroup on any XCD that has not cached the line before reads the new data.
__device__ __forceinline__ void store8_device_scope(void* p, const uint2 v) {
  typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
  const u32x2 q = {v.x, v.y};
  asm volatile("global_store_dwordx2 %0, %1, off sc1" ::"v"(p), "v"(q) : "memory");
}

// One unit of the bf16 decode kernels: workgroup `blk` of the launch that has one workgroup of 4
// waves per (expert, 64 hidden units) [UP] or (expert, 128 output features) [down].  COHERENT:
// the output rows are stored at device scope (for a consumer in the same launch).
template <bool UP, bool COHERENT>
__device__ __forceinline__ void skinny_unit(const SkinnyArgs& a, const int blk) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int r = lane & 15, q = lane >> 4;
  int g = 0;
  while (g + 1 < a.Ng && blk >= a.blk_prefix[g + 1]) ++g;
  const int F = a.F[g];
  const int K = UP ? a.d : F;
  const int ncols = UP ? F : a.d;
  // workgroup = 4 waves; up: 64 hidden units; down: 128 output features
  constexpr int COLS_PER_BLOCK = UP ? 64 : 128;
  const int blocks_per_expert = (ncols + COLS_PER_BLOCK - 1) / COLS_PER_BLOCK;
  const int local = blk - a.blk_prefix[g];
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
    // NTB = token blocks of 16 in flight: decode mostly has a handful of tokens per expert, and
    // the second block would cost its operand loads and matrix-core steps for nothing
    auto pass = [&](auto NTBC) {
      constexpr int NTB = decltype(NTBC)::value;
      const uint16_t* xp[2];
      bool xv[2];
  #pragma unroll
      for (int tb = 0; tb < NTB; ++tb) {
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
        for (int tb = 0; tb < NTB; ++tb) acc[f][tb] = f32x4{0.f, 0.f, 0.f, 0.f};

      auto step = [&](int k0, auto UC) {
        constexpr int U = decltype(UC)::value;
        Frag wf[2][U], xf[2][U];
  #pragma unroll
        for (int u = 0; u < U; ++u) {
  #pragma unroll
          for (int f = 0; f < 2; ++f) wf[f][u].u = *reinterpret_cast<const uint4*>(wp[f] + k0 + 32 * u);
  #pragma unroll
          for (int tb = 0; tb < NTB; ++tb) {
            xf[tb][u].u = make_uint4(0u, 0u, 0u, 0u);
            if (xv[tb]) xf[tb][u].u = *reinterpret_cast<const uint4*>(xp[tb] + k0 + 32 * u);
          }
        }
  #pragma unroll
        for (int u = 0; u < U; ++u)
  #pragma unroll
          for (int f = 0; f < 2; ++f)
  #pragma unroll
            for (int tb = 0; tb < NTB; ++tb)
              acc[f][tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[f][u].v, xf[tb][u].v, acc[f][tb], 0, 0, 0);
      };
      // The deepest unrolling only with one token block: the registers of the rarer two-block pass
      // would otherwise set the kernel's occupancy.
      // Every wave starts its walk along the rows at a different main step and wraps around.  All
      // weight rows begin at multiples of the row size, a power of two at the usual hidden sizes,
      // so waves that walk in step ask the same few memory channels at any one time; staggered
      // they spread over all of them (a pure-read kernel with this access pattern: 5.2-5.6 TB/s in
      // step, 6.2 TB/s staggered, at a row of 8 KB; this kernel, which also loads tokens and feeds
      // the matrix cores, gains 1.5 %).  The order of the fp32 additions then depends on the wave,
      // which is fixed by the launch: results stay bit-identical from run to run.
      constexpr int MAIN = NTB == 1 ? 256 : 128;
      const int nmain = K / MAIN;
      int st = nmain > 0 ? (int)(((long long)blk * 4 + w) * 5 % nmain) : 0;
      for (int sidx = 0; sidx < nmain; ++sidx) {
        step(st * MAIN, std::integral_constant<int, MAIN / 32>{});
        if (++st == nmain) st = 0;
      }
      int k0 = nmain * MAIN;
      for (; k0 + 128 <= K; k0 += 128) step(k0, std::integral_constant<int, 4>{});
      for (; k0 < K; k0 += 64) step(k0, std::integral_constant<int, 2>{});

      // lane holds token r of each token block, weight rows 4q..4q+3 of each row set
  #pragma unroll
      for (int tb = 0; tb < NTB; ++tb) {
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
          if constexpr (COHERENT) store8_device_scope(crow + c0 + 4 * q, o);
          else *reinterpret_cast<uint2*>(crow + c0 + 4 * q) = o;
        } else {
  #pragma unroll
          for (int f = 0; f < 2; ++f) {
            const int col = c0 + 16 * f + 4 * q;
            if (col < ncols) {
              uint2 o;
              o.x = pack_bf16x2(acc[f][tb][0], acc[f][tb][1]);
              o.y = pack_bf16x2(acc[f][tb][2], acc[f][tb][3]);
              if constexpr (COHERENT) store8_device_scope(crow + col, o);
              else *reinterpret_cast<uint2*>(crow + col) = o;
            }
          }
        }
      }
    };
    if (cnt - tb0 > 16) pass(std::integral_constant<int, 2>{});
    else pass(std::integral_constant<int, 1>{});
  }
}

}  // namespace mohge
