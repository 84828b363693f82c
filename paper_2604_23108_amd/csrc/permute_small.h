// Stable counting sort of the (token, slot) pairs by expert: the pieces shared by the permutation
// kernels and the single-launch decode layer (wave-level histogram and scatter, and the whole sort
// of up to kBlockPairs pairs by one workgroup).
#pragma once
#include "common.h"

namespace mohge {

constexpr int kSegPairs = 512;                 // pairs per wave segment
constexpr int kWavesPerBlock = 4;
constexpr int kBlockPairs = kSegPairs * kWavesPerBlock;
constexpr int kFusedMaxCells = 8192;            // segments x experts that the fused scatter stages in LDS

struct PermArgs {
  const int32_t* eidx;
  int32_t* counts;
  int32_t* offsets;
  int32_t* perm;
  int32_t* inv_perm;
  int32_t* seg_hist;   // [nseg][Ne], overwritten with segment bases by the scan
  int P, Ne, nseg, nbits;
};

// lanes of the wave that are active and hold the same `key` as this lane
__device__ __forceinline__ unsigned long long match_mask(int key, int nbits, bool active) {
  unsigned long long m = __ballot(active);
  for (int b = 0; b < nbits; ++b) {
    const unsigned long long bal = __ballot((key >> b) & 1);
    m &= ((key >> b) & 1) ? bal : ~bal;
  }
  return m;
}

// expert id of pair p, forced into [0, Ne) so that a corrupt input cannot index outside
// the LDS tables (the result is then meaningless but every access stays in bounds)
__device__ __forceinline__ int load_expert(const PermArgs& a, int p) {
  const int e = a.eidx[p];
  return e < 0 ? 0 : (e >= a.Ne ? a.Ne - 1 : e);
}

__device__ __forceinline__ void wave_histogram(const PermArgs& a, int seg, int lane, int* hist) {
  const int p0 = seg * kSegPairs;
  for (int i = 0; i < kSegPairs; i += 64) {
    const int p = p0 + i + lane;
    if (p < a.P) atomicAdd(&hist[load_expert(a, p)], 1);
  }
}

// base[e] = first free output position for expert e in this segment (LDS, wave private)
__device__ __forceinline__ void wave_scatter(const PermArgs& a, int seg, int lane, int* base) {
  const int p0 = seg * kSegPairs;
  for (int i = 0; i < kSegPairs; i += 64) {
    const int p = p0 + i + lane;
    const bool active = p < a.P;
    const int e = active ? load_expert(a, p) : 0;
    const unsigned long long m = match_mask(e, a.nbits, active);
    const unsigned long long lt = (1ull << lane) - 1ull;
    int r = 0;
    if (active) {
      r = base[e] + __popcll(m & lt);
      // (a position outside [0, P) can only come from corrupted bases: never write there)
      if (r >= 0 && r < a.P) {
        a.perm[r] = p;
        a.inv_perm[p] = r;
      }
    }
    // `base` belongs to this wave and LDS operations of one wave complete in order: only the
    // compiler has to be kept from moving the cursor update across the reads
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    // the highest lane of each set of equal experts advances the bucket cursor
    if (active && (m >> lane) == 1ull) base[e] = r + 1;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
}

// P <= kBlockPairs: histogram, scan and scatter in one workgroup.
// hist: LDS, [kWavesPerBlock][kMaxExperts]; wtot: LDS, [kWavesPerBlock].  Called by all 256 threads.
__device__ __forceinline__ void permute_small_body(const PermArgs& a, int (*hist)[kMaxExperts], int* wtot) {
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  for (int e = threadIdx.x; e < kWavesPerBlock * kMaxExperts; e += blockDim.x) (&hist[0][0])[e] = 0;
  __syncthreads();
  wave_histogram(a, w, lane, hist[w]);
  __syncthreads();
  // one expert per thread (Ne <= 256): its count over the four segments, then an exclusive scan
  // over the experts (inside the waves by shuffles, across them through LDS)
  const int e = threadIdx.x;
  int h[kWavesPerBlock], c = 0;
#pragma unroll
  for (int ww = 0; ww < kWavesPerBlock; ++ww) {
    h[ww] = e < a.Ne ? hist[ww][e] : 0;
    c += h[ww];
  }
  int incl = c;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int up = __shfl_up(incl, off, 64);
    if (lane >= off) incl += up;
  }
  if (lane == 63) wtot[w] = incl;
  __syncthreads();
  int off_e = incl - c;
  for (int ww = 0; ww < w; ++ww) off_e += wtot[ww];
  if (e < a.Ne) {
    int run = off_e;
#pragma unroll
    for (int ww = 0; ww < kWavesPerBlock; ++ww) {
      hist[ww][e] = run;            // becomes the base of (segment ww, expert e)
      run += h[ww];
    }
    a.counts[e] = c;
    a.offsets[e] = off_e;
    if (e == a.Ne - 1) a.offsets[a.Ne] = off_e + c;
  }
  __syncthreads();
  wave_scatter(a, w, lane, hist[w]);
}

}  // namespace mohge
