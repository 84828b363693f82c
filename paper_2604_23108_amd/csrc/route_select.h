// Router arguments and the selection phase of the two-level router (section 3.2 of the paper),
// shared by the router kernels and the single-launch decode layer.
#pragma once
#include "common.h"

namespace mohge {

typedef float f32x4 __attribute__((ext_vector_type(4)));

struct RouteArgs {
  const void* x;
  const float* wg;
  const float* we;
  const float* bias;
  int32_t* gidx;
  int32_t* eidx;
  float* gates;
  float* gs;
  float* es1;
  int T, d, Ng, N, Ne, Kg, Ke, mode;
  int NO;        // Ng + Ne
  int NOpad;     // NO rounded up to a multiple of 16, plus 4 (row stride of lg)
  int Nepad;     // Ne rounded up to 64
  int kslice;    // hidden elements per wave
  int region0;   // bytes of the first LDS region (partial totals / per-wave rows)
  int dsplit;    // > 1: the hidden dimension is also split over grid.y workgroups, which leave
                 //   their fp64 logit sums in gpart; route_finish_kernel adds them and selects
  double* gpart; // [dsplit][T][NO]
};

template <bool BF16>
__device__ __forceinline__ void load8(const void* base, size_t elem_off, float (&v)[8]) {
  if constexpr (BF16) {
    const uint4 u = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(base) + elem_off);
    v[0] = __uint_as_float(u.x << 16); v[1] = __uint_as_float(u.x & 0xffff0000u);
    v[2] = __uint_as_float(u.y << 16); v[3] = __uint_as_float(u.y & 0xffff0000u);
    v[4] = __uint_as_float(u.z << 16); v[5] = __uint_as_float(u.z & 0xffff0000u);
    v[6] = __uint_as_float(u.w << 16); v[7] = __uint_as_float(u.w & 0xffff0000u);
  } else {
    const float4* p = reinterpret_cast<const float4*>(static_cast<const float*>(base) + elem_off);
    const float4 a = p[0], b = p[1];
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
    v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// Phase 2 when the group size is a power of two (at most 64), so that a group is an aligned run
// of N lanes: lane l holds experts l, l + 64, ... (NJ of them; NJ = 1 when every expert has a lane
// of its own) and everything stays in registers.  Group maximum and sum are butterflies over the N
// lanes (every lane of the group ends with the same bits), the group gate's top-K_g and the expert
// top-k are rank counts against values fetched from other lanes (readlane for a position all lanes
// agree on, a lane permutation for the partners inside the group), the ascending output slots
// come from ballots and population counts, the normalisation from a wave-wide butterfly.  No LDS
// beyond the logits row, no barriers.
__device__ __forceinline__ float lane_value(float v, int uniform_lane) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), uniform_lane));
}

template <int NJ>
__device__ __forceinline__ void route_select_small(const RouteArgs& a, const float* lg, int t0, int BT, int NW,
                                                   int w, int lane) {
  const int klimit = (a.mode == MOHGE_SELECT_GLOBAL) ? a.Ke : a.Ke / a.Kg;
  const int iters = (BT + NW - 1) / NW;
  const float NEG_INF = -__builtin_inff();
  const int N = a.N;
  const int li = lane & (N - 1);             // position inside the group (groups are aligned lane runs)
  const int lb = lane - li;                  // first lane of the group
  int e[NJ], g[NJ];
  bool valid[NJ];
  float bias[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    e[j] = lane + 64 * j;
    valid[j] = e[j] < a.Ne;
    g[j] = valid[j] ? e[j] / N : 0;
    bias[j] = (a.bias && valid[j]) ? a.bias[e[j]] : 0.f;
  }
  for (int it = 0; it < iters; ++it) {
    const int tl = it * NW + w;
    const int t = t0 + tl;
    const bool live = (tl < BT) && (t < a.T);
    const float* lrow = lg + (size_t)(live ? tl : 0) * a.NOpad;
    // group gate: rank of each group's logit (ties to the lower id)
    const float zg = (lane < a.Ng) ? lrow[lane] : NEG_INF;
    int grank = 0;
    for (int g2 = 0; g2 < a.Ng; ++g2) {
      const float z2 = lane_value(zg, g2);
      grank += (z2 > zg) || (z2 == zg && g2 < lane);
    }
    const bool gsel = (lane < a.Ng) && (grank < a.Kg);
    const unsigned long long gmask = __ballot(gsel);
    const float gs_mine = 1.f / (1.f + expf(-zg));            // lanes < N_g: GS of group `lane`
    if (live && lane < a.Ng) {
      if (a.gs) a.gs[(size_t)t * a.Ng + lane] = gs_mine;
      if (gsel) {
        // (a NaN logit could make more than K_g lanes qualify: never write past the row)
        const int slot = __popcll(gmask & ((1ull << lane) - 1ull));
        if (slot < a.Kg) a.gidx[(size_t)t * a.Kg + slot] = lane;
      }
    }
    float z[NJ], e1[NJ], e2[NJ], key[NJ];
    bool in[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      z[j] = valid[j] ? lrow[a.Ng + e[j]] + bias[j] : NEG_INF;
      in[j] = valid[j] && ((gmask >> g[j]) & 1ull);
      // softmax inside the group: maximum and sum over its N lanes
      float mx = in[j] ? z[j] : NEG_INF;
      for (int off = 1; off < N; off <<= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
      const float ex = in[j] ? expf(z[j] - mx) : 0.f;
      float sum = ex;
      for (int off = 1; off < N; off <<= 1) sum += __shfl_xor(sum, off, 64);
      e1[j] = in[j] ? ex / sum : 0.f;
      const float gs_g = __shfl(gs_mine, g[j], 64);           // GS of this expert's group
      e2[j] = in[j] ? e1[j] * gs_g : 0.f;
      key[j] = in[j] ? ((a.mode == MOHGE_SELECT_GLOBAL) ? e2[j] : z[j]) : NEG_INF;
    }
    // expert top-k: rank among the candidates (ties to the lower id)
    int rank[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) rank[j] = 0;
    if (a.mode == MOHGE_SELECT_GLOBAL) {
      // the candidates are the members of the kept groups only (the mask is the same in every lane)
      for (unsigned long long m = gmask; m != 0ull; m &= m - 1ull) {
        const int e0 = (int)__builtin_ctzll(m) * N;            // first expert of a kept group
        if (e0 >= a.Ne) break;
        const int jj = e0 >> 6, l0 = e0 & 63;
        float kj = key[0];
#pragma unroll
        for (int j = 1; j < NJ; ++j) kj = jj == j ? key[j] : kj;
        for (int i = 0; i < N; ++i) {
          const float k2 = lane_value(kj, l0 + i);
          const int e2i = e0 + i;
#pragma unroll
          for (int j = 0; j < NJ; ++j) rank[j] += (k2 > key[j]) || (k2 == key[j] && e2i < e[j]);
        }
      }
    } else {
#pragma unroll
      for (int j = 0; j < NJ; ++j)
        for (int i = 1; i < N; ++i) {
          const int other = lb + ((li + i) & (N - 1));        // lane of another member of the group
          const float k2 = __shfl(key[j], other, 64);
          rank[j] += (k2 > key[j]) || (k2 == key[j] && other < lane);
        }
    }
    bool sel[NJ];
    unsigned long long smask[NJ];
    float dsum = 0.f;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      sel[j] = in[j] && rank[j] < klimit;
      smask[j] = __ballot(sel[j]);
      if (sel[j]) dsum += e2[j];
    }
    const float D = wave_sum(dsum);
    int base = 0;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      if (live && valid[j]) {
        if (a.es1) a.es1[(size_t)t * a.Ne + e[j]] = e1[j];
        if (sel[j]) {
          const int slot = base + __popcll(smask[j] & ((1ull << lane) - 1ull));
          if (slot < a.Ke) {
            a.eidx[(size_t)t * a.Ke + slot] = e[j];
            a.gates[(size_t)t * a.Ke + slot] = e2[j] / D;
          }
        }
      }
      base += __popcll(smask[j]);
    }
  }
}

// Phase 2 for the BT tokens from t0 whose logits are in lg ([BT][NOpad], LDS); uses the first
// LDS region for the per-wave rows.
__device__ __forceinline__ void route_select(const RouteArgs& a, unsigned char* smem, const float* lg,
                                             int t0, int BT, int NW, int w, int lane) {
  if ((a.N & (a.N - 1)) == 0 && a.N <= 64) {
    if (a.Ne <= 64) route_select_small<1>(a, lg, t0, BT, NW, w, lane);
    else if (a.Ne <= 128) route_select_small<2>(a, lg, t0, BT, NW, w, lane);
    else route_select_small<4>(a, lg, t0, BT, NW, w, lane);
    return;
  }
  // ---- phase 2: one wavefront per token, lane <-> expert ---------------------
  float* zrow = reinterpret_cast<float*>(smem) + (size_t)w * 5 * a.Nepad;  // biased expert logits
  float* e1row = zrow + a.Nepad;                                            // ES'
  float* e2row = e1row + a.Nepad;                                           // ES''
  float* krow = e2row + a.Nepad;                                            // selection key
  float* xrow = krow + a.Nepad;                                             // exp(z - max of the group)
  const int klimit = (a.mode == MOHGE_SELECT_GLOBAL) ? a.Ke : a.Ke / a.Kg;
  const bool vec4 = (a.N & 3) == 0;      // group rows can be read four members at a time
  const int iters = (BT + NW - 1) / NW;
  const float NEG_INF = -__builtin_inff();
  // the logit bias does not depend on the token: fetched once (a load inside the token loop would
  // also wait for the previous token's result stores)
  float bias_r[4] = {0.f, 0.f, 0.f, 0.f};
  if (a.bias)
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (lane + 64 * j < a.Ne) bias_r[j] = a.bias[lane + 64 * j];
  for (int it = 0; it < iters; ++it) {
    const int tl = it * NW + w;
    const int t = t0 + tl;
    const bool live = (tl < BT) && (t < a.T);
    const float* lrow = lg + (size_t)(live ? tl : 0) * a.NOpad;

    // group gating: rank of each group's logit (ties to the lower id)
    const float zg = (lane < a.Ng) ? lrow[lane] : NEG_INF;
    int grank = 0;
    for (int g2 = 0; g2 < a.Ng; ++g2) {
      const float z2 = lrow[g2];
      grank += (z2 > zg) || (z2 == zg && g2 < lane);
    }
    const bool gsel = (lane < a.Ng) && (grank < a.Kg);
    const unsigned long long gmask = __ballot(gsel);
    if (live && lane < a.Ng) {
      if (a.gs) a.gs[(size_t)t * a.Ng + lane] = 1.f / (1.f + expf(-zg));
      if (gsel) {
        // (a NaN logit could make more than K_g lanes qualify: never write past the row)
        const int slot = __popcll(gmask & ((1ull << lane) - 1ull));
        if (slot < a.Kg) a.gidx[(size_t)t * a.Kg + slot] = lane;
      }
    }

    // zrow / e1row / e2row / krow are private to this wave: LDS operations of one wave
    // complete in order, so only the compiler has to be kept from reordering them
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (lane + 64 * j < a.Ne) zrow[lane + 64 * j] = lrow[a.Ng + lane + 64 * j] + bias_r[j];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();

    // every expert's exp(z - max of its group) once (one expf per lane and expert instead of
    // one per lane and group member); the sums below add these in member order
    for (int e = lane; e < a.Ne; e += 64) {
      const int g = e / a.N;
      float ex = 0.f;
      if ((gmask >> g) & 1ull) {
        const float* zg_row = zrow + g * a.N;
        float mx = NEG_INF;
        if (vec4) {
          // (rows of a group start on a 16-byte boundary when N is a multiple of 4)
#pragma unroll 4
          for (int i = 0; i < a.N; i += 4) {
            const float4 v = *reinterpret_cast<const float4*>(zg_row + i);
            mx = fmaxf(fmaxf(mx, fmaxf(v.x, v.y)), fmaxf(v.z, v.w));
          }
        } else {
#pragma unroll 8
          for (int i = 0; i < a.N; ++i) mx = fmaxf(mx, zg_row[i]);
        }
        ex = expf(zrow[e] - mx);
      }
      xrow[e] = ex;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();

    for (int e = lane; e < a.Nepad; e += 64) {
      const int g = e < a.Ne ? e / a.N : 0;
      const bool in = e < a.Ne && ((gmask >> g) & 1ull);
      float e1 = 0.f, e2 = 0.f;
      if (in) {
        const float* xg_row = xrow + g * a.N;
        float sum = 0.f;
        if (vec4) {
#pragma unroll 4
          for (int i = 0; i < a.N; i += 4) {         // same member order as the scalar loop
            const float4 v = *reinterpret_cast<const float4*>(xg_row + i);
            sum += v.x; sum += v.y; sum += v.z; sum += v.w;
          }
        } else {
#pragma unroll 8
          for (int i = 0; i < a.N; ++i) sum += xg_row[i];
        }
        e1 = xrow[e] / sum;
        e2 = e1 * (1.f / (1.f + expf(-lrow[g])));
      }
      if (e < a.Ne) {
        e1row[e] = e1;
        e2row[e] = e2;
      }
      // (entries past N_e exist so that the rank loop can read the keys four at a time)
      krow[e] = in ? ((a.mode == MOHGE_SELECT_GLOBAL) ? e2 : zrow[e]) : NEG_INF;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();

    unsigned long long smask[4] = {0ull, 0ull, 0ull, 0ull};
    float dsum = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (64 * j < a.Ne) {
        const int e = lane + 64 * j;
        const bool valid = e < a.Ne;
        const int g = valid ? e / a.N : 0;
        const bool in = valid && ((gmask >> g) & 1ull);
        bool sel = false;
        if (in) {
          const float key = krow[e];
          int rank = 0;
          if (a.mode == MOHGE_SELECT_GLOBAL) {
#pragma unroll 8
            for (int e2i = 0; e2i < a.Nepad; e2i += 4) {
              const float4 k4 = *reinterpret_cast<const float4*>(krow + e2i);
              rank += (k4.x > key) || (k4.x == key && e2i < e);
              rank += (k4.y > key) || (k4.y == key && e2i + 1 < e);
              rank += (k4.z > key) || (k4.z == key && e2i + 2 < e);
              rank += (k4.w > key) || (k4.w == key && e2i + 3 < e);
            }
          } else if (vec4) {
#pragma unroll 4
            for (int i = 0; i < a.N; i += 4) {
              const int e2i = g * a.N + i;
              const float4 k4 = *reinterpret_cast<const float4*>(krow + e2i);
              rank += (k4.x > key) || (k4.x == key && e2i < e);
              rank += (k4.y > key) || (k4.y == key && e2i + 1 < e);
              rank += (k4.z > key) || (k4.z == key && e2i + 2 < e);
              rank += (k4.w > key) || (k4.w == key && e2i + 3 < e);
            }
          } else {
#pragma unroll 8
            for (int i = 0; i < a.N; ++i) {
              const int e2i = g * a.N + i;
              const float k2 = krow[e2i];
              rank += (k2 > key) || (k2 == key && e2i < e);
            }
          }
          sel = rank < klimit;
        }
        smask[j] = __ballot(sel);
        if (sel) dsum += e2row[e];
      }
    }
    const float D = wave_sum(dsum);
    int base = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (64 * j < a.Ne) {
        const int e = lane + 64 * j;
        if (live && e < a.Ne) {
          if (a.es1) a.es1[(size_t)t * a.Ne + e] = e1row[e];
          if ((smask[j] >> lane) & 1ull) {
            const int slot = base + __popcll(smask[j] & ((1ull << lane) - 1ull));
            if (slot < a.Ke) {
              a.eidx[(size_t)t * a.Ke + slot] = e;
              a.gates[(size_t)t * a.Ke + slot] = e2row[e] / D;
            }
          }
        }
        base += __popcll(smask[j]);
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
}

}  // namespace mohge
