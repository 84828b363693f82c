// Group-Wise Auxiliary Loss L_G (section 3.3) and Intra-Group Experts Auxiliary Loss
// L_E (section 3.4.2) for gfx950.
//
// Both are sums over tokens of per-token quantities, followed by a few operations per
// group / expert.  Stage 1: every workgroup owns a contiguous range of tokens, a wave
// takes one token at a time with lane <-> group / expert and keeps fp64 running sums in
// registers; waves are added in a fixed order.  Stage 2: one workgroup adds the
// per-workgroup partial sums (rows of partial sums read side by side, fixed order) and
// evaluates the losses.  No atomics, so the result is bit-identical from run to run.
#include "common.h"

namespace mohge {

struct AuxArgs {
  const float* gs;
  const float* es1;
  const int32_t* gidx;
  const int32_t* eidx;
  float* losses;
  float* stats;
  double* part;          // [nblk][2*(Ng+Ne)]: score sums, then counts
  int T, Ng, N, Ne, Kg, Ke, nblk, tok_per_blk;
  float alpha_g, alpha_e, eps;
  int freq_norm;
  float ratio[kMaxGroups];   // F_g / max F
};

__global__ void __launch_bounds__(256) aux_partial_kernel(const AuxArgs a) {
  __shared__ double red[4][2 * (kMaxGroups + kMaxExperts)];
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int ncol = a.Ng + a.Ne;
  const int tbeg = blockIdx.x * a.tok_per_blk;
  const int tend = min(a.T, tbeg + a.tok_per_blk);
  double pG = 0.0, cG = 0.0, pE[4] = {0.0, 0.0, 0.0, 0.0}, cE[4] = {0.0, 0.0, 0.0, 0.0};
  for (int t = tbeg + w; t < tend; t += 4) {
    if (lane < a.Ng) {
      // s'_{g,t} = GS_{g,t} / sum_j GS_{j,t}
      const float* row = a.gs + (size_t)t * a.Ng;
      float sum = 0.f;
      for (int j = 0; j < a.Ng; ++j) sum += row[j];
      pG += (double)(row[lane] / sum);
      for (int s = 0; s < a.Kg; ++s) cG += (a.gidx[(size_t)t * a.Kg + s] == lane) ? 1.0 : 0.0;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int e = lane + 64 * j;
      if (e < a.Ne) {
        // S^E_{g,i,t} = ES'_{g,i,t} / (sum_j ES'_{g,j,t} + eps)
        const float* row = a.es1 + (size_t)t * a.Ne;
        const int g0 = (e / a.N) * a.N;
        float sum = 0.f;
        for (int i = 0; i < a.N; ++i) sum += row[g0 + i];
        pE[j] += (double)(row[e] / (sum + a.eps));
        for (int s = 0; s < a.Ke; ++s) cE[j] += (a.eidx[(size_t)t * a.Ke + s] == e) ? 1.0 : 0.0;
      }
    }
  }
  if (lane < a.Ng) { red[w][lane] = pG; red[w][ncol + lane] = cG; }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int e = lane + 64 * j;
    if (e < a.Ne) { red[w][a.Ng + e] = pE[j]; red[w][ncol + a.Ng + e] = cE[j]; }
  }
  __syncthreads();
  for (int c = threadIdx.x; c < 2 * ncol; c += blockDim.x)
    a.part[(size_t)blockIdx.x * 2 * ncol + c] = ((red[0][c] + red[1][c]) + red[2][c]) + red[3][c];
}

__global__ void __launch_bounds__(1024) aux_final_kernel(const AuxArgs a) {
  __shared__ double tot[2 * (kMaxGroups + kMaxExperts)];
  __shared__ double red[1024];
  const int ncol = a.Ng + a.Ne, C = 2 * ncol;
  // thread t adds column t % C over the partial-sum rows r, r + R, r + 2R, ... (r = t / C, R =
  // row groups that fit the workgroup): neighbouring threads read neighbouring columns of one
  // row.  Then the R sums of a column are added in index order: a fixed order throughout.
  const int R = 1024 / C > 0 ? 1024 / C : 1;
  const int col = threadIdx.x % C, r = threadIdx.x / C;
  if (r < R) {
    double s0 = 0.0, s1 = 0.0;
    int b = r;
    for (; b + R < a.nblk; b += 2 * R) {
      s0 += a.part[(size_t)b * C + col];
      s1 += a.part[(size_t)(b + R) * C + col];
    }
    if (b < a.nblk) s0 += a.part[(size_t)b * C + col];
    red[r * C + col] = s0 + s1;
  }
  __syncthreads();
  for (int c = threadIdx.x; c < C; c += blockDim.x) {
    double s = 0.0;
    for (int i = 0; i < R; ++i) s += red[i * C + c];
    tot[c] = s;
  }
  __syncthreads();
  const double invT = 1.0 / (double)a.T;
  const double fscale = a.freq_norm ? invT : 1.0;
  // f and p per group / expert
  for (int c = threadIdx.x; c < ncol; c += blockDim.x) {
    const double p = tot[c] * invT;
    const double f = tot[ncol + c] * fscale *
                     (c < a.Ng ? (double)a.Ng / (double)a.Kg : (double)a.N / (double)a.Ke);
    tot[c] = p;
    tot[ncol + c] = f;
    if (a.stats) {
      if (c < a.Ng) { a.stats[c] = (float)f; a.stats[a.Ng + c] = (float)p; }
      else { a.stats[2 * a.Ng + (c - a.Ng)] = (float)f; a.stats[2 * a.Ng + a.Ne + (c - a.Ng)] = (float)p; }
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double LG = 0.0, LE = 0.0;
    for (int g = 0; g < a.Ng; ++g) LG += (double)a.ratio[g] * tot[ncol + g] * tot[g];
    for (int e = 0; e < a.Ne; ++e) LE += tot[ncol + a.Ng + e] * tot[a.Ng + e];
    a.losses[0] = (float)((double)a.alpha_g * LG);
    a.losses[1] = (float)((double)a.alpha_e * LE);
  }
}

// 16 tokens per workgroup (4 per wave, each a chain of dependent loads), at most 1024 workgroups
static int aux_blocks(const LayerDesc& L) {
  int b = (L.T + 15) / 16;
  return b < 1 ? 1 : (b > 1024 ? 1024 : b);
}

size_t aux_workspace_bytes(const LayerDesc& L) {
  return ((size_t)aux_blocks(L) * 2 * (L.Ng + L.Ne) * sizeof(double) + 255) / 256 * 256;
}

hipError_t launch_aux_loss(const LayerDesc& L, const mohge_config& cfg, const float* gs,
                           const float* es1, const int32_t* group_idx, const int32_t* expert_idx,
                           float* losses, float* stats, void* ws, hipStream_t s) {
  AuxArgs a;
  a.gs = gs; a.es1 = es1; a.gidx = group_idx; a.eidx = expert_idx; a.losses = losses; a.stats = stats;
  a.part = static_cast<double*>(ws);
  a.T = L.T; a.Ng = L.Ng; a.N = L.N; a.Ne = L.Ne; a.Kg = L.Kg; a.Ke = L.Ke;
  a.nblk = aux_blocks(L);
  a.tok_per_blk = (L.T + a.nblk - 1) / a.nblk;
  a.alpha_g = cfg.alpha_g; a.alpha_e = cfg.alpha_e; a.eps = cfg.eps; a.freq_norm = cfg.aux_freq_norm;
  for (int g = 0; g < kMaxGroups; ++g) a.ratio[g] = g < L.Ng ? (float)L.F[g] / (float)L.Fmax : 0.f;
  hipLaunchKernelGGL(aux_partial_kernel, dim3(a.nblk), dim3(256), 0, s, a);
  hipLaunchKernelGGL(aux_final_kernel, dim3(1), dim3(1024), 0, s, a);
  return hipGetLastError();
}

}  // namespace mohge
