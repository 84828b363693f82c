// Token permutation for gfx950: a deterministic, stable counting sort of the
// P = T*K_e (token, slot) pairs by expert id.
//
// The pair list is cut into wave segments of 512 consecutive pairs.  Every wave
// (1) histograms its segment in LDS, (2) a scan turns the [segment][expert] counts
// into the first output position of every (segment, expert), (3) every wave walks its
// segment again 64 pairs at a time and ranks equal experts inside the 64 with ballots
// (one ballot per bit of the expert id), so the order inside a bucket is the pair order.
// Integer LDS atomics only feed counts, so nothing depends on execution order.
// Up to 2048 pairs the three steps run in one single-workgroup kernel;
// while segments x experts <= 8192 the scan is folded into the scatter kernel (two launches
// instead of three).  (One workgroup of sixteen waves for up to 32768 pairs, a single launch, was
// slower than the two launches: 15 against 11 us at 16384 pairs, 28 against 12 us at 32768.)
#include <mutex>

#include "common.h"
#include "permute_small.h"

namespace mohge {

// Segment histograms of mohge_permute_static: the one scratch buffer of the permutation, held in
// the library's own device memory so that the call needs no workspace from the caller.  Every GPU
// the library runs on holds its own copy at its own address; host code never uses the array's
// name as an address, only the pointer hipGetSymbolAddress returned for the current device.
static __device__ __align__(256) unsigned char scratch[MOHGE_PERMUTE_STATIC_BYTES];
constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mutex;

// device address of `scratch` on the current device (looked up once per device)
static hipError_t static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

__global__ void __launch_bounds__(256) permute_hist_kernel(const PermArgs a) {
  __shared__ int hist[kWavesPerBlock][kMaxExperts];
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  for (int e = threadIdx.x; e < kWavesPerBlock * kMaxExperts; e += blockDim.x) (&hist[0][0])[e] = 0;
  __syncthreads();
  const int seg = blockIdx.x * kWavesPerBlock + w;
  if (seg < a.nseg) wave_histogram(a, seg, lane, hist[w]);
  __syncthreads();
  if (seg < a.nseg)
    for (int e = lane; e < a.Ne; e += 64) a.seg_hist[(size_t)seg * a.Ne + e] = hist[w][e];
}

// One workgroup of 16 waves.  Wave v handles experts v, v+16, ...: an exclusive scan of
// that expert's counts over the segments; then an exclusive scan over experts.
__global__ void __launch_bounds__(1024) permute_scan_kernel(const PermArgs a) {
  __shared__ int cnt[kMaxExperts + 1];
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  for (int e = w; e < a.Ne; e += 16) {
    int carry = 0;
    for (int s0 = 0; s0 < a.nseg; s0 += 64) {
      const int s = s0 + lane;
      const int v = (s < a.nseg) ? a.seg_hist[(size_t)s * a.Ne + e] : 0;
      int incl = v;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const int up = __shfl_up(incl, off, 64);
        if (lane >= off) incl += up;
      }
      if (s < a.nseg) a.seg_hist[(size_t)s * a.Ne + e] = carry + incl - v;
      carry += __shfl(incl, 63, 64);
    }
    if (lane == 0) cnt[e] = carry;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0;
    for (int e = 0; e < a.Ne; ++e) {
      const int c = cnt[e];
      a.counts[e] = c;
      a.offsets[e] = run;
      run += c;
    }
    a.offsets[a.Ne] = run;
  }
}

// FUSED: the segment histograms are still raw counts; every workgroup sums them itself
// (column totals -> offsets, counts of earlier segments -> its own bases) instead of reading
// the output of a separate scan kernel.  Used while the number of segments is small.
template <bool FUSED>
__global__ void __launch_bounds__(256) permute_scatter_kernel(const PermArgs a) {
  __shared__ int base[kWavesPerBlock][kMaxExperts];
  __shared__ int wtot[4];
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int seg = blockIdx.x * kWavesPerBlock + w;
  if constexpr (FUSED) {
    // stage the whole [segment][expert] count matrix in LDS with independent, coalesced
    // loads (one memory round trip), then walk it per expert
    __shared__ int hist[kFusedMaxCells];
    const int cells = a.nseg * a.Ne;
    for (int i = threadIdx.x; i < cells; i += blockDim.x) hist[i] = a.seg_hist[i];
    __syncthreads();
    const int e = threadIdx.x;                      // one expert per thread (Ne <= 256)
    const int seg0 = blockIdx.x * kWavesPerBlock;
    int run = 0, pre[kWavesPerBlock] = {0, 0, 0, 0};
    if (e < a.Ne) {
      for (int s = 0; s < a.nseg; ++s) {
#pragma unroll
        for (int k = 0; k < kWavesPerBlock; ++k)
          if (s == seg0 + k) pre[k] = run;
        run += hist[s * a.Ne + e];
      }
    }
    // exclusive scan of the totals over the experts
    int incl = run;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int up = __shfl_up(incl, off, 64);
      if (lane >= off) incl += up;
    }
    if (lane == 63) wtot[w] = incl;
    __syncthreads();
    int off_e = incl - run;
    for (int ww = 0; ww < w; ++ww) off_e += wtot[ww];
    if (e < a.Ne) {
#pragma unroll
      for (int k = 0; k < kWavesPerBlock; ++k) base[k][e] = off_e + pre[k];
      if (blockIdx.x == 0) {
        a.counts[e] = run;
        a.offsets[e] = off_e;
        if (e == a.Ne - 1) a.offsets[a.Ne] = off_e + run;
      }
    }
  } else {
    const int segc = seg < a.nseg ? seg : a.nseg - 1;
    for (int e = lane; e < a.Ne; e += 64) base[w][e] = a.seg_hist[(size_t)segc * a.Ne + e] + a.offsets[e];
  }
  __syncthreads();
  // every wave runs the same number of rounds (pairs past P are inactive)
  PermArgs b = a;
  if (seg >= a.nseg) b.P = 0;
  wave_scatter(b, seg, lane, base[w]);
}

__global__ void __launch_bounds__(256) permute_small_kernel(const PermArgs a) {
  __shared__ int hist[kWavesPerBlock][kMaxExperts];
  __shared__ int wtot[kWavesPerBlock];
  permute_small_body(a, hist, wtot);
}

template <typename V>
__global__ void __launch_bounds__(256) gather_rows_kernel(const V* __restrict__ x, V* __restrict__ xp,
                                                          const int32_t* __restrict__ perm, int P,
                                                          int Ke, int vec_per_row) {
  // one wave per output row, 16 bytes per lane per step
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= P) return;
  const int lane = threadIdx.x & 63;
  const V* src = x + (size_t)(perm[r] / Ke) * vec_per_row;
  V* dst = xp + (size_t)r * vec_per_row;
  for (int i = lane; i < vec_per_row; i += 64) dst[i] = src[i];
}

size_t permute_workspace_bytes(const LayerDesc& L) {
  const size_t nseg = ((size_t)L.P + kSegPairs - 1) / kSegPairs;
  const size_t b = (nseg > 0 ? nseg : 1) * (size_t)L.Ne * sizeof(int32_t);
  return (b + 255) / 256 * 256;
}

hipError_t launch_permute(const LayerDesc& L, int dtype, const int32_t* expert_idx,
                          int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv_perm,
                          const void* x, void* x_perm, void* ws, hipStream_t s) {
  PermArgs a;
  a.eidx = expert_idx; a.counts = counts; a.offsets = offsets; a.perm = perm; a.inv_perm = inv_perm;
  a.seg_hist = static_cast<int32_t*>(ws);
  a.P = L.P; a.Ne = L.Ne;
  a.nseg = (L.P + kSegPairs - 1) / kSegPairs;
  a.nbits = 0;
  while ((1 << a.nbits) < L.Ne) ++a.nbits;
  if (L.P <= kBlockPairs) {
    hipLaunchKernelGGL(permute_small_kernel, dim3(1), dim3(256), 0, s, a);
  } else {
    const int nblk = (a.nseg + kWavesPerBlock - 1) / kWavesPerBlock;
    hipLaunchKernelGGL(permute_hist_kernel, dim3(nblk), dim3(256), 0, s, a);
    if (a.nseg * a.Ne <= kFusedMaxCells) {
      hipLaunchKernelGGL(permute_scatter_kernel<true>, dim3(nblk), dim3(256), 0, s, a);
    } else {
      hipLaunchKernelGGL(permute_scan_kernel, dim3(1), dim3(1024), 0, s, a);
      hipLaunchKernelGGL(permute_scatter_kernel<false>, dim3(nblk), dim3(256), 0, s, a);
    }
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (x_perm && L.P > 0) {
    const int row_bytes = L.d * (dtype == MOHGE_BF16 ? 2 : 4);
    hipLaunchKernelGGL((gather_rows_kernel<uint4>), dim3((L.P + 3) / 4), dim3(256), 0, s,
                       static_cast<const uint4*>(x), static_cast<uint4*>(x_perm), perm, L.P, L.Ke,
                       row_bytes / 16);
    e = hipGetLastError();
  }
  return e;
}

// The same launches with the segment histograms in the library's static device array.  The
// histogram kernel overwrites every cell the later kernels read, so nothing has to be cleared
// between calls.
hipError_t launch_permute_static(const LayerDesc& L, int dtype, const int32_t* expert_idx,
                                 int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv_perm,
                                 const void* x, void* x_perm, hipStream_t s) {
  if (permute_workspace_bytes(L) > (size_t)MOHGE_PERMUTE_STATIC_BYTES) return hipErrorInvalidValue;
  void* ws = nullptr;
  hipError_t e = static_scratch(&ws);
  if (e != hipSuccess) return e;
  return launch_permute(L, dtype, expert_idx, counts, offsets, perm, inv_perm, x, x_perm, ws, s);
}

}  // namespace mohge
