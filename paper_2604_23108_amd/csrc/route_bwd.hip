// Backward pass of the two-level router (section 3.2) including the gradients of the
// Group-Wise Auxiliary Loss (3.3) and the Intra-Group Experts Auxiliary Loss (3.4.2), and the
// assembly of the layer's input gradient, for gfx950 (x in bf16, everything else fp32).
//
// The routing decisions and the routing frequencies f are constants.  Per token, with the
// forward's GS, ES' (zero outside kept groups), gates, and the incoming dgate:
//   D      = sum_kept ES'_e GS_g(e),      gd = sum_kept dgate_e gate_e
//   dES''_e = (dgate_e - gd) / D                     (kept experts, else 0)
//   dES'_e  = dES''_e GS_g + v_e/(sigma_g+eps) - (sum_i v_i ES'_i)/(sigma_g+eps)^2   (kept groups)
//   dGS_g   = sum_i dES''_i ES'_i + (u_g - sum_j u_j GS_j/S)/S,   S = sum_j GS_j     (all groups)
//   dzE_e   = ES'_e (dES'_e - sum_i dES'_i ES'_i),   dzG_g = dGS_g GS_g (1 - GS_g)
// with u_g = alpha_G (F_g/F_max) f^G_g / T and v_e = alpha_E f^E_e / T.  Then
//   dW_G = dzG^T x,  dW_E = dzE^T x,  dx_t = sum_slot dx_perm[r(t,slot)] + dzG_t W_G + dzE_t W_E.
//
// Kernels: (1) one wave per token for the scalar chain above; (2) the two weight gradients as a
// reduction over tokens, split over the grid with partial sums added in a fixed order (no
// atomics: bit-identical from run to run); (3) the input gradient, 8 tokens per workgroup so
// that every router weight is fetched once per 8 tokens.
#include "common.h"

namespace mohge {

struct RouteBwdArgs {
  const uint16_t* x;
  const float* w_group;
  const float* w_expert;
  const float* gs;
  const float* es1;
  const int32_t* gidx;
  const int32_t* eidx;
  const float* gates;
  const float* dgates;
  const float* stats;        // f^G[Ng], p^G[Ng], f^E[Ne], p^E[Ne] or NULL (no auxiliary terms)
  const uint16_t* dx_perm;
  const int32_t* inv_perm;
  uint16_t* dx;
  float* dw_group;
  float* dw_expert;
  float* dz;                 // [T, Z], Z = Ng + Ne: group logits first
  float* part;               // [S, Z, d]
  int T, d, Ng, N, Ne, Kg, Ke, Z, S, tok_per_split;
  float alpha_g, alpha_e, eps;
  float ratio[kMaxGroups];
};

__global__ void __launch_bounds__(256) route_bwd_token_kernel(const RouteBwdArgs a) {
  __shared__ float sh_v[kMaxExperts], sh_u[kMaxGroups];
  __shared__ float ex[4][3][kMaxExperts];   // per wave: ES', dES'', dES'
  __shared__ float gq[4][4][kMaxGroups];    // per wave: sigma, sum v ES', sum dES'' ES', sum dES' ES'
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const float invT = 1.f / (float)a.T;
  for (int e = threadIdx.x; e < a.Ne; e += 256)
    sh_v[e] = a.stats ? a.alpha_e * a.stats[2 * a.Ng + e] * invT : 0.f;
  if (threadIdx.x < a.Ng)
    sh_u[threadIdx.x] = a.stats ? a.alpha_g * a.ratio[threadIdx.x] * a.stats[threadIdx.x] * invT : 0.f;
  const int t = blockIdx.x * 4 + w;
  const bool live = t < a.T;
  const int tt = live ? t : a.T - 1;         // idle waves redo the last token and store nothing
  const float* gs = a.gs + (size_t)tt * a.Ng;
  const float* es1 = a.es1 + (size_t)tt * a.Ne;
  const int32_t* eidx = a.eidx + (size_t)tt * a.Ke;
  const int32_t* gidx = a.gidx + (size_t)tt * a.Kg;
  const float* dgate = a.dgates + (size_t)tt * a.Ke;
  const float* gate = a.gates + (size_t)tt * a.Ke;

  // gates -> ES''
  float D = 0.f, gd = 0.f;
  for (int s = 0; s < a.Ke; ++s) {
    const int e = eidx[s];
    D += es1[e] * gs[e / a.N];
    gd = fmaf(dgate[s], gate[s], gd);
  }
  const float invD = 1.f / D;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int e = lane + 64 * j;
    if (e < a.Ne) {
      float d2 = 0.f;
      for (int s = 0; s < a.Ke; ++s)
        if (eidx[s] == e) d2 = (dgate[s] - gd) * invD;
      ex[w][0][e] = es1[e];
      ex[w][1][e] = d2;
    }
  }
  __syncthreads();
  if (lane < a.Ng) {
    float sigma = 0.f, vs = 0.f, dg = 0.f;
    for (int i = 0; i < a.N; ++i) {
      const int e = lane * a.N + i;
      sigma += ex[w][0][e];
      vs = fmaf(sh_v[e], ex[w][0][e], vs);
      dg = fmaf(ex[w][1][e], ex[w][0][e], dg);
    }
    gq[w][0][lane] = sigma; gq[w][1][lane] = vs; gq[w][2][lane] = dg;
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int e = lane + 64 * j;
    if (e < a.Ne) {
      const int g = e / a.N;
      bool kept = false;
      for (int s = 0; s < a.Kg; ++s) kept |= gidx[s] == g;
      float d1 = 0.f;
      if (kept) {
        const float den = gq[w][0][g] + a.eps;
        d1 = ex[w][1][e] * gs[g] + sh_v[e] / den - gq[w][1][g] / (den * den);
      }
      ex[w][2][e] = d1;
    }
  }
  __syncthreads();
  if (lane < a.Ng) {
    const int g = lane;
    float wsum = 0.f;
    for (int i = 0; i < a.N; ++i) wsum = fmaf(ex[w][2][g * a.N + i], ex[w][0][g * a.N + i], wsum);
    gq[w][3][g] = wsum;
    float S = 0.f, us = 0.f;
    for (int j = 0; j < a.Ng; ++j) S += gs[j];
    for (int j = 0; j < a.Ng; ++j) us = fmaf(sh_u[j], gs[j] / S, us);
    bool kept = false;
    for (int s = 0; s < a.Kg; ++s) kept |= gidx[s] == g;
    const float dGS = (kept ? gq[w][2][g] : 0.f) + (sh_u[g] - us) / S;
    if (live) a.dz[(size_t)t * a.Z + g] = dGS * gs[g] * (1.f - gs[g]);
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int e = lane + 64 * j;
    if (e < a.Ne && live) {
      const int g = e / a.N;
      // ES' is zero outside kept groups, and so is dES'
      a.dz[(size_t)t * a.Z + a.Ng + e] = ex[w][0][e] * (ex[w][2][e] - gq[w][3][g]);
    }
  }
}

// partial sums of dW[z, c] = sum_t dz[t, z] x[t, c] on the fp32 matrix cores
// (v_mfma_f32_32x32x2_f32: C[32x32] += A[32x2] B[2x32]): grid (ceil(d/1024), S), a wave owns 256
// columns and a pass of 32 rows z, and takes the tokens of its split two at a time.  Lane
// (j = lane%32, k = lane/32) loads dz[t+k, z0+j] (the A operand as it is) and the 8 columns
// c0 + 8j .. +7 of x[t+k] (one 16-byte load); MFMA m takes element m of every lane's eight, so
// its 32 B-columns are the tile columns {8j + m}.  A lane ends up with 8 consecutive columns of
// 16 rows.  Loads run one group of 4 steps ahead of the arithmetic; nothing crosses waves.
typedef float f32x16_t __attribute__((ext_vector_type(16)));
constexpr int kZC = 32, kTU = 4;

__global__ void __launch_bounds__(256) route_bwd_wgrad_kernel(const RouteBwdArgs a) {
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int j = lane & 31, k = lane >> 5;
  const int c0 = (blockIdx.x * 4 + w) * 256;
  if (c0 >= a.d) return;                       // wave-uniform; the kernel has no barriers
  const int c = c0 + 8 * j;
  const bool col_ok = c < a.d;
  const int cc = col_ok ? c : 0;
  const int t0 = blockIdx.y * a.tok_per_split;
  const int t1 = min(a.T, t0 + a.tok_per_split);
  for (int z0 = 0; z0 < a.Z; z0 += kZC) {
    const int zl = z0 + j;
    // step at token t: this lane's token is t + k (dz = 0 past the split or past Z)
    auto load = [&](int t, uint4& xv, float& dzv) {
      const int tok = t + k, tt = min(tok, a.T - 1);
      xv = *reinterpret_cast<const uint4*>(a.x + (size_t)tt * a.d + cc);
      const float v = a.dz[(size_t)tt * a.Z + min(zl, a.Z - 1)];
      dzv = (tok < t1 && zl < a.Z) ? v : 0.f;
    };
    f32x16_t acc[8];
#pragma unroll
    for (int m = 0; m < 8; ++m)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[m][r] = 0.f;
    uint4 xc[kTU];
    float dc[kTU];
#pragma unroll
    for (int i = 0; i < kTU; ++i) load(t0 + 2 * i, xc[i], dc[i]);
    for (int t = t0; t < t1; t += 2 * kTU) {
      uint4 xn[kTU];
      float dn[kTU];
#pragma unroll
      for (int i = 0; i < kTU; ++i) load(t + 2 * kTU + 2 * i, xn[i], dn[i]);
#pragma unroll
      for (int i = 0; i < kTU; ++i) {
        const uint32_t u[4] = {xc[i].x, xc[i].y, xc[i].z, xc[i].w};
#pragma unroll
        for (int m = 0; m < 8; ++m) {
          const float xf = __uint_as_float((m & 1) ? (u[m >> 1] & 0xffff0000u) : (u[m >> 1] << 16));
          acc[m] = __builtin_amdgcn_mfma_f32_32x32x2f32(dc[i], xf, acc[m], 0, 0, 0);
        }
      }
#pragma unroll
      for (int i = 0; i < kTU; ++i) { xc[i] = xn[i]; dc[i] = dn[i]; }
    }
    // accumulator r of a lane: row 8*(r/4) + 4*k + r%4 of the pass, B-column j
    if (col_ok) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int z = z0 + 8 * (r / 4) + 4 * k + (r % 4);
        if (z < a.Z) {
          float4* dst = reinterpret_cast<float4*>(a.part + ((size_t)blockIdx.y * a.Z + z) * a.d + c);
          dst[0] = make_float4(acc[0][r], acc[1][r], acc[2][r], acc[3][r]);
          dst[1] = make_float4(acc[4][r], acc[5][r], acc[6][r], acc[7][r]);
        }
      }
    }
  }
}

// dW = sum of the S partial slices, in a fixed order: thread (q, j) of a workgroup adds slices
// j, j + 8, ... of four neighbouring elements, then the 8 sums are added in index order.
__global__ void __launch_bounds__(256) route_bwd_wsum_kernel(const RouteBwdArgs a) {
  __shared__ float4 red[8][32];
  const size_t n4 = (size_t)a.Z * a.d / 4;                 // d is a multiple of 4
  const int q = threadIdx.x & 31, j = threadIdx.x >> 5;
  const size_t i4 = (size_t)blockIdx.x * 32 + q;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  if (i4 < n4) {
    const float4* p = reinterpret_cast<const float4*>(a.part) + i4;
    for (int k = j; k < a.S; k += 8) {
      const float4 v = p[(size_t)k * n4];
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
  }
  red[j][q] = s;
  __syncthreads();
  if (j == 0 && i4 < n4) {
    float4 t = red[0][q];
#pragma unroll
    for (int k = 1; k < 8; ++k) { t.x += red[k][q].x; t.y += red[k][q].y; t.z += red[k][q].z; t.w += red[k][q].w; }
    const size_t i = i4 * 4, z = i / a.d, c = i % a.d;
    float* dst = z < (size_t)a.Ng ? a.dw_group + z * a.d + c : a.dw_expert + (z - a.Ng) * a.d + c;
    *reinterpret_cast<float4*>(dst) = t;
  }
}

// dx: grid (ceil(T/8), ceil(d/2048)); a thread owns 8 columns of 8 tokens
__global__ void __launch_bounds__(256) route_bwd_dx_kernel(const RouteBwdArgs a) {
  constexpr int TB = 8;
  const int c = (blockIdx.y * 256 + threadIdx.x) * 8;      // c >= d: helps staging dz only
  const int t0 = blockIdx.x * TB;
  float acc[TB][8];
#pragma unroll
  for (int k = 0; k < TB; ++k) {
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[k][i] = 0.f;
    const int t = t0 + k;
    if (t < a.T && a.dx_perm && c < a.d) {
      // four slots at a time: the row loads are issued together, then added in slot order
      for (int s0 = 0; s0 < a.Ke; s0 += 4) {
        uint4 u[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int r = a.inv_perm[(size_t)t * a.Ke + min(s0 + i, a.Ke - 1)];
          u[i] = *reinterpret_cast<const uint4*>(a.dx_perm + (size_t)r * a.d + c);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          if (s0 + i < a.Ke) {
            acc[k][0] += __uint_as_float(u[i].x << 16); acc[k][1] += __uint_as_float(u[i].x & 0xffff0000u);
            acc[k][2] += __uint_as_float(u[i].y << 16); acc[k][3] += __uint_as_float(u[i].y & 0xffff0000u);
            acc[k][4] += __uint_as_float(u[i].z << 16); acc[k][5] += __uint_as_float(u[i].z & 0xffff0000u);
            acc[k][6] += __uint_as_float(u[i].w << 16); acc[k][7] += __uint_as_float(u[i].w & 0xffff0000u);
          }
        }
      }
    }
  }
  // dz of the workgroup's 8 tokens: one contiguous block of dz[T, Z], staged in LDS and read
  // back as broadcasts
  __shared__ float dzs[TB * (kMaxGroups + kMaxExperts)];
  {
    const int n = TB * a.Z;
    const size_t base = (size_t)t0 * a.Z, lim = (size_t)a.T * a.Z;
    for (int i = threadIdx.x; i < n; i += 256) dzs[i] = base + i < lim ? a.dz[base + i] : 0.f;
  }
  __syncthreads();
  if (c < a.d) {
    for (int z = 0; z < a.Z; ++z) {
      const float* wr = z < a.Ng ? a.w_group + (size_t)z * a.d + c : a.w_expert + (size_t)(z - a.Ng) * a.d + c;
      const float4 w0 = *reinterpret_cast<const float4*>(wr), w1 = *reinterpret_cast<const float4*>(wr + 4);
#pragma unroll
      for (int k = 0; k < TB; ++k) {
        const float dzv = dzs[k * a.Z + z];
        acc[k][0] = fmaf(dzv, w0.x, acc[k][0]); acc[k][1] = fmaf(dzv, w0.y, acc[k][1]);
        acc[k][2] = fmaf(dzv, w0.z, acc[k][2]); acc[k][3] = fmaf(dzv, w0.w, acc[k][3]);
        acc[k][4] = fmaf(dzv, w1.x, acc[k][4]); acc[k][5] = fmaf(dzv, w1.y, acc[k][5]);
        acc[k][6] = fmaf(dzv, w1.z, acc[k][6]); acc[k][7] = fmaf(dzv, w1.w, acc[k][7]);
      }
    }
  }
  if (c >= a.d) return;
#pragma unroll
  for (int k = 0; k < TB; ++k) {
    const int t = t0 + k;
    if (t < a.T) {
      uint4 o;
      o.x = pack_bf16x2(acc[k][0], acc[k][1]); o.y = pack_bf16x2(acc[k][2], acc[k][3]);
      o.z = pack_bf16x2(acc[k][4], acc[k][5]); o.w = pack_bf16x2(acc[k][6], acc[k][7]);
      *reinterpret_cast<uint4*>(a.dx + (size_t)t * a.d + c) = o;
    }
  }
}

// token splits of the weight-gradient reduction: about 64 tokens each, at most 256 splits and at
// most 64 MB of partial sums
static int wgrad_splits(const LayerDesc& L) {
  long long s = (L.T + 63) / 64;
  const long long cap = (64ll << 20) / ((long long)(L.Ng + L.Ne) * L.d * 4);
  if (s > cap) s = cap;
  if (s > 256) s = 256;
  return s < 1 ? 1 : (int)s;
}

static size_t up256(size_t b) { return (b + 255) / 256 * 256; }

// workspace: dz [T, Z] fp32, then the partial sums [S, Z, d] fp32
size_t route_bwd_workspace_bytes(const LayerDesc& L) {
  const size_t Z = L.Ng + L.Ne, T = L.T > 0 ? L.T : 1;
  return up256(T * Z * 4) + up256((size_t)wgrad_splits(L) * Z * L.d * 4);
}

hipError_t launch_route_bwd(const LayerDesc& L, const mohge_config& cfg, const void* x,
                            const float* w_group, const float* w_expert, const float* gs,
                            const float* es1, const int32_t* group_idx, const int32_t* expert_idx,
                            const float* gates, const float* dgates, const float* stats,
                            const void* dx_perm, const int32_t* inv_perm, void* dx, float* dw_group,
                            float* dw_expert, float* dz_out, void* ws, hipStream_t s) {
  RouteBwdArgs a{};
  a.x = static_cast<const uint16_t*>(x);
  a.w_group = w_group; a.w_expert = w_expert; a.gs = gs; a.es1 = es1;
  a.gidx = group_idx; a.eidx = expert_idx; a.gates = gates; a.dgates = dgates; a.stats = stats;
  a.dx_perm = static_cast<const uint16_t*>(dx_perm); a.inv_perm = inv_perm;
  a.dx = static_cast<uint16_t*>(dx); a.dw_group = dw_group; a.dw_expert = dw_expert;
  a.T = L.T; a.d = L.d; a.Ng = L.Ng; a.N = L.N; a.Ne = L.Ne; a.Kg = L.Kg; a.Ke = L.Ke;
  a.Z = L.Ng + L.Ne;
  a.S = wgrad_splits(L);
  a.tok_per_split = (L.T + a.S - 1) / a.S;
  a.alpha_g = cfg.alpha_g; a.alpha_e = cfg.alpha_e; a.eps = cfg.eps;
  for (int g = 0; g < kMaxGroups; ++g) a.ratio[g] = g < L.Ng ? (float)L.F[g] / (float)L.Fmax : 0.f;
  unsigned char* base = static_cast<unsigned char*>(ws);
  const size_t dz_bytes = up256((size_t)L.T * a.Z * 4);
  a.dz = dz_out ? dz_out : reinterpret_cast<float*>(base);
  a.part = reinterpret_cast<float*>(base + dz_bytes);
  hipLaunchKernelGGL(route_bwd_token_kernel, dim3((unsigned)((L.T + 3) / 4)), dim3(256), 0, s, a);
  hipLaunchKernelGGL(route_bwd_wgrad_kernel, dim3((unsigned)((L.d + 1023) / 1024), (unsigned)a.S), dim3(256), 0, s, a);
  hipLaunchKernelGGL(route_bwd_wsum_kernel, dim3((unsigned)(((size_t)a.Z * L.d / 4 + 31) / 32)), dim3(256), 0, s, a);
  hipLaunchKernelGGL(route_bwd_dx_kernel, dim3((unsigned)((L.T + 7) / 8), (unsigned)((L.d + 2047) / 2048)),
                     dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace mohge
