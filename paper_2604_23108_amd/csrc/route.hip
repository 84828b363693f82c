// Two-level router (section 3.2 of the paper) for gfx950.
//
// One workgroup owns 16*TM tokens.  Phase 1 computes the N_g + N_e logits of its
// tokens with the fp32 matrix cores (v_mfma_f32_16x16x4_f32): tokens are the M
// rows, router rows (group embeddings first, then expert embeddings) the N columns.
// Each lane loads 8 consecutive hidden elements of "its" token / router row straight
// from global memory -- this is already the operand layout the instruction wants, so
// no LDS staging is needed.  The hidden dimension is split over the waves of the
// workgroup; every wave folds its fp32 accumulators into fp64 totals after each 64
// hidden elements, and the per-wave totals are added in fp64 in a fixed order.  This
// keeps the logit error near 1e-7, which bit-exact top-k agreement with an fp64
// reference needs.
// With few tokens (decode) one workgroup per 16 tokens leaves most of the chip idle while two
// compute units grind through the whole reduction: then the hidden dimension is split over
// grid.y workgroups as well, each leaves its fp64 sums in a workspace, and a second small kernel
// adds them in a fixed order and runs phase 2.
// Phase 2 runs one wavefront per token with lane <-> expert: group top-K_g by rank
// counting, softmax inside kept groups, scaling by the group score, expert top-k by
// rank counting, a ballot + popcount to assign ascending output slots, and a
// cross-lane sum for the gate normalisation.
#include <type_traits>

#include "common.h"
#include "route_select.h"

namespace mohge {

template <bool BF16, int TM, int TN>
__global__ void __launch_bounds__(512) route_kernel(const RouteArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  constexpr int BT = 16 * TM, NC = 16 * TN;
  const int NW = blockDim.x >> 6;
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r = lane & 15, q = lane >> 4;
  const int t0 = blockIdx.x * BT;
  double* part = reinterpret_cast<double*>(smem);                 // [NW][BT][NC]
  float* lg = reinterpret_cast<float*>(smem + a.region0);         // [BT][NOpad]

  // ---- phase 1: logits ----------------------------------------------------
  size_t xrow[TM];
#pragma unroll
  for (int tm = 0; tm < TM; ++tm) {
    int t = t0 + 16 * tm + r;
    xrow[tm] = (size_t)(t < a.T ? t : a.T - 1) * a.d;
  }
  for (int nc = 0; nc < a.NO; nc += NC) {
    const float* wrow[TN];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
      int o = nc + 16 * tn + r;
      if (o > a.NO - 1) o = a.NO - 1;
      wrow[tn] = (o < a.Ng) ? a.wg + (size_t)o * a.d : a.we + (size_t)(o - a.Ng) * a.d;
    }
    f32x4 acc[TM][TN];
    double tot[TM][TN][4];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
      for (int tn = 0; tn < TN; ++tn) {
        acc[tm][tn] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < 4; ++i) tot[tm][tn][i] = 0.0;
      }
    const int kbeg = ((int)blockIdx.y * NW + w) * a.kslice, kend = kbeg + a.kslice;
    // The token rows are read exactly once from HBM in small pieces (16 rows x 64 bytes per
    // wave-wide load), so the loop is bound by memory latency unless many loads are in
    // flight: all token loads of a chunk of up to XS 32-element steps are requested up
    // front and kept packed in registers; the router rows (L2 resident) are requested one
    // step ahead.  The fp32 accumulators are folded into the fp64 totals after every pair of
    // steps (64 elements).
    constexpr int XS = BF16 ? 16 : 4;
    typedef typename std::conditional<BF16, uint4, float4>::type xraw_t;
    constexpr int XR = BF16 ? 1 : 2;                 // raw registers-of-16-bytes per step
    for (int kc = kbeg; kc < kend; kc += 32 * XS) {
      xraw_t xraw[TM][XS][XR];
#pragma unroll
      for (int st = 0; st < XS; ++st)
        if (kc + 32 * st < kend) {
#pragma unroll
          for (int tm = 0; tm < TM; ++tm) {
            const xraw_t* p = reinterpret_cast<const xraw_t*>(
                static_cast<const char*>(a.x) + (xrow[tm] + kc + 32 * st + 8 * q) * (BF16 ? 2 : 4));
#pragma unroll
            for (int u = 0; u < XR; ++u) xraw[tm][st][u] = p[u];
          }
        }
      float wb[2][TN][8];
#pragma unroll
      for (int tn = 0; tn < TN; ++tn) load8<false>(wrow[tn], (size_t)(kc + 8 * q), wb[0][tn]);
#pragma unroll
      for (int st = 0; st < XS; ++st) {
        const int k = kc + 32 * st;
        if (k < kend) {
          if (st + 1 < XS && k + 32 < kend) {
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) load8<false>(wrow[tn], (size_t)(k + 32 + 8 * q), wb[(st + 1) & 1][tn]);
          }
          float xa[TM][8];
#pragma unroll
          for (int tm = 0; tm < TM; ++tm) {
            if constexpr (BF16) {
              const uint4 u = xraw[tm][st][0];
              xa[tm][0] = __uint_as_float(u.x << 16); xa[tm][1] = __uint_as_float(u.x & 0xffff0000u);
              xa[tm][2] = __uint_as_float(u.y << 16); xa[tm][3] = __uint_as_float(u.y & 0xffff0000u);
              xa[tm][4] = __uint_as_float(u.z << 16); xa[tm][5] = __uint_as_float(u.z & 0xffff0000u);
              xa[tm][6] = __uint_as_float(u.w << 16); xa[tm][7] = __uint_as_float(u.w & 0xffff0000u);
            } else {
              const float4 lo = xraw[tm][st][0], hi = xraw[tm][st][XR - 1];
              xa[tm][0] = lo.x; xa[tm][1] = lo.y; xa[tm][2] = lo.z; xa[tm][3] = lo.w;
              xa[tm][4] = hi.x; xa[tm][5] = hi.y; xa[tm][6] = hi.z; xa[tm][7] = hi.w;
            }
          }
#pragma unroll
          for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
              for (int tn = 0; tn < TN; ++tn)
                acc[tm][tn] = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[tm][j], wb[st & 1][tn][j], acc[tm][tn], 0, 0, 0);
          if ((st & 1) || k + 32 >= kend) {
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
              for (int tn = 0; tn < TN; ++tn) {
#pragma unroll
                for (int i = 0; i < 4; ++i) tot[tm][tn][i] += (double)acc[tm][tn][i];
                acc[tm][tn] = f32x4{0.f, 0.f, 0.f, 0.f};
              }
          }
        }
      }
    }
    // Accumulator element i of lane (r, q) is token 4q+i, router row r of the 16x16 tile.
    // Every wave stores its fp64 totals in its own slice; then they are added in wave order.
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
      for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          part[((size_t)w * BT + 16 * tm + 4 * q + i) * NC + 16 * tn + r] = tot[tm][tn][i];
    __syncthreads();
    for (int idx = threadIdx.x; idx < BT * NC; idx += blockDim.x) {
      const int tl = idx / NC, ol = idx % NC;
      double sum = 0.0;
      for (int ww = 0; ww < NW; ++ww) sum += part[(size_t)ww * BT * NC + idx];
      if (nc + ol < a.NO) {
        if (a.dsplit > 1) {
          if (t0 + tl < a.T) a.gpart[((size_t)blockIdx.y * a.T + t0 + tl) * a.NO + nc + ol] = sum;
        } else {
          lg[tl * a.NOpad + nc + ol] = (float)sum;
        }
      }
    }
    __syncthreads();
  }

  if (a.dsplit > 1) return;          // route_finish_kernel takes over
  route_select(a, smem, lg, t0, BT, NW, w, lane);
}

// ---------------------------------------------------------------------------------------
// Prefill form (bf16 tokens, many tokens): the logits on the bf16 matrix cores, exactly.
// A router weight (fp32, 24 significant bits) is the exact sum of three bf16 numbers (its
// leading 8 bits, the next 8, the rest: each taken by truncation, the remainders are exact
// in fp32), a token element is one bf16 number, and a product of two bf16 numbers is exact in
// fp32.  So  x . w = x . w_hi + x . w_mid + x . w_lo  with v_mfma_f32_16x16x32_bf16, whose only
// rounding is the fp32 accumulation; the large part (w_hi) is accumulated over 64 hidden
// elements at a time and then added to an fp64 total, as in the fp32 form above, which keeps
// the logit error below 1e-7.  Sixteen times the fp32 matrix rate at three times the work.
//
// A small kernel first splits the router rows into the three bf16 planes (workspace:
// [3][rows padded to whole passes][d], padding rows zero).  In the main kernel a workgroup of 8
// waves owns 16*TG tokens: waves = TG token groups of 16 x (8/TG) parts of every 128-deep chunk
// of the hidden dimension.  A wave loads its token fragments straight from global memory in
// operand layout (several chunks ahead); the three planes of a chunk go global -> LDS without
// passing registers (global_load_lds, double buffered, 16-byte pieces XOR-swizzled by the row so
// that the 128-bit fragment reads are conflict free).  The waves of a token group add their fp64
// totals through LDS in fixed order.  Router rows are processed 16*TN at a time (TN <= 5 column
// tiles: more would not fit the registers); wider routers make several passes over the token rows.
// ---------------------------------------------------------------------------------------
typedef __bf16 rbf16x8 __attribute__((ext_vector_type(8)));

constexpr int kPfChunk = 128;            // hidden elements per chunk

// planes[p][row][k], p = 0 (leading bits), 1, 2; rows >= NO are zero
__global__ void __launch_bounds__(256) route_split_kernel(const float* __restrict__ wg, const float* __restrict__ we,
                                                          uint16_t* __restrict__ planes, int Ng, int NO,
                                                          int rows, int d) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;      // one thread per 4 hidden elements
  const int per_row = d / 4;
  if (idx >= (long long)rows * per_row) return;
  const int o = (int)(idx / per_row), k = (int)(idx % per_row) * 4;
  float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
  if (o < NO) v = *reinterpret_cast<const float4*>(((o < Ng) ? wg + (size_t)o * d : we + (size_t)(o - Ng) * d) + k);
  const float f[4] = {v.x, v.y, v.z, v.w};
  uint32_t hi[4], mid[4], lo[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    hi[i] = __float_as_uint(f[i]) & 0xffff0000u;
    const float r1 = f[i] - __uint_as_float(hi[i]);          // exact
    mid[i] = __float_as_uint(r1) & 0xffff0000u;
    const float r2 = r1 - __uint_as_float(mid[i]);           // exact, at most 8 significant bits
    lo[i] = __float_as_uint(r2) & 0xffff0000u;
  }
  const size_t plane = (size_t)rows * d, at = (size_t)o * d + k;
  *reinterpret_cast<uint2*>(planes + at) = make_uint2((hi[0] >> 16) | hi[1], (hi[2] >> 16) | hi[3]);
  *reinterpret_cast<uint2*>(planes + plane + at) = make_uint2((mid[0] >> 16) | mid[1], (mid[2] >> 16) | mid[3]);
  *reinterpret_cast<uint2*>(planes + 2 * plane + at) = make_uint2((lo[0] >> 16) | lo[1], (lo[2] >> 16) | lo[3]);
}

template <int TG, int TN>
__global__ void __launch_bounds__(512) route_prefill_kernel(const RouteArgs a, const uint16_t* __restrict__ planes,
                                                            int plane_rows) {
  extern __shared__ __align__(1024) unsigned char smem[];
  constexpr int KQ = 8 / TG;                 // waves along the hidden dimension
  constexpr int KS = 4 / KQ;                 // 32-deep MFMA steps of a wave per chunk
  constexpr int BT = 16 * TG, NC = 16 * TN;
  constexpr int PLANE = NC * 256, BUF = 3 * PLANE;
  constexpr int NCOPY = 3 * NC / 4;          // wave-wide copies (4 rows x 256 bytes) per chunk
  constexpr int XP = 4;                      // token chunks in flight
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int tg = w / KQ, kq = w % KQ;
  const int r = lane & 15, q = lane >> 4;
  const int t0 = blockIdx.x * BT;
  float* lg = reinterpret_cast<float*>(smem + a.region0);         // [BT][NOpad]
  double* red = reinterpret_cast<double*>(smem);                  // [BT][NC], after the chunk loop
  const int nchunks = a.d / kPfChunk;

  const int tok = t0 + tg * 16 + r;
  const uint16_t* xrow = static_cast<const uint16_t*>(a.x) + (size_t)(tok < a.T ? tok : a.T - 1) * a.d +
                         kq * 32 * KS + 8 * q;
  const size_t plane_elems = (size_t)plane_rows * a.d;

  for (int nc = 0; nc < a.NO; nc += NC) {
    f32x4 acc_h[TN], acc_l[TN];
    double tot[TN][4];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
      acc_h[tn] = f32x4{0.f, 0.f, 0.f, 0.f};
      acc_l[tn] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int i = 0; i < 4; ++i) tot[tn][i] = 0.0;
    }
    // copy idx (wave-uniform) of a chunk: plane idx / (NC/4), rows 4*(idx % (NC/4)) .. +3 of the
    // pass; lane l fills row l/16, physical piece l%16, which holds logical piece (l%16) ^ (row & 15)
    auto copy_w = [&](int c, int b) {
      for (int idx = w; idx < NCOPY; idx += 8) {
        const int p = idx / (NC / 4), row = 4 * (idx % (NC / 4)) + (lane >> 4);
        const int piece = (lane & 15) ^ (row & 15);
        const uint16_t* src = planes + p * plane_elems + (size_t)(nc + row) * a.d + (size_t)c * kPfChunk + piece * 8;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                         (__attribute__((address_space(3))) void*)(smem + b * BUF + idx * 1024),
                                         16, 0, 0);
      }
    };
    uint4 xr[XP][KS];
    auto load_x = [&](int c, int slot) {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        xr[slot][ks] = *reinterpret_cast<const uint4*>(xrow + (size_t)c * kPfChunk + 32 * ks);
    };

    __syncthreads();                     // the previous pass has left the buffers
    copy_w(0, 0);
#pragma unroll
    for (int u = 0; u < XP; ++u)
      if (u < nchunks) load_x(u, u);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    for (int c0 = 0; c0 < nchunks; c0 += XP) {
#pragma unroll
      for (int u = 0; u < XP; ++u) {
        const int c = c0 + u;
        if (c < nchunks) {
          rbf16x8 xa[KS];
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) xa[ks] = __builtin_bit_cast(rbf16x8, xr[u][ks]);
          // the next chunk's planes into the other buffer (nobody reads it any more: barrier at
          // the end of the previous chunk), then the token fragments of a later chunk
          if (c + 1 < nchunks) copy_w(c + 1, (u + 1) & 1);
          __builtin_amdgcn_sched_barrier(0);
          if (c + XP < nchunks) load_x(c + XP, u);
          __builtin_amdgcn_sched_barrier(0);
          const unsigned char* fb = smem + (u & 1) * BUF + r * 256;
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) {
            const int piece = ((kq * KS + ks) * 4 + q) ^ r;
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
              const unsigned char* f = fb + 16 * tn * 256 + piece * 16;
              const rbf16x8 bh = *reinterpret_cast<const rbf16x8*>(f);
              const rbf16x8 bm = *reinterpret_cast<const rbf16x8*>(f + PLANE);
              const rbf16x8 bl = *reinterpret_cast<const rbf16x8*>(f + 2 * PLANE);
              acc_h[tn] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa[ks], bh, acc_h[tn], 0, 0, 0);
              acc_l[tn] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa[ks], bm, acc_l[tn], 0, 0, 0);
              acc_l[tn] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa[ks], bl, acc_l[tn], 0, 0, 0);
            }
            // the large part goes into the fp64 totals after every 64 hidden elements of this wave
            if (KS == 2 ? ks == 1 : ((u & 1) || c + 1 == nchunks)) {
#pragma unroll
              for (int tn = 0; tn < TN; ++tn) {
#pragma unroll
                for (int i = 0; i < 4; ++i) tot[tn][i] += (double)acc_h[tn][i];
                acc_h[tn] = f32x4{0.f, 0.f, 0.f, 0.f};
              }
            }
          }
          // my pieces of the next chunk's planes have landed when at most the token loads issued
          // after them are outstanding (loads complete in order)
          if (c + XP < nchunks) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(KS) : "memory");
          else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
          __syncthreads();
        }
      }
    }
    // the small parts, then the waves of a token group in fixed order
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
      for (int i = 0; i < 4; ++i) tot[tn][i] += (double)acc_l[tn][i];
    for (int step = 0; step < KQ; ++step) {
      if (kq == step) {
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            // accumulator element i of lane (r, q): token 4q+i, router row r of the tile
            const int tl = tg * 16 + 4 * q + i, ol = 16 * tn + r;
            double v = tot[tn][i];
            if (step > 0) v += red[tl * NC + ol];
            if (step < KQ - 1) red[tl * NC + ol] = v;
            else if (nc + ol < a.NO) lg[tl * a.NOpad + nc + ol] = (float)v;
          }
      }
      __syncthreads();
    }
  }
  route_select(a, smem, lg, t0, BT, 8, w, lane);
}

template <int TG, int TN>
static hipError_t launch_prefill(const RouteArgs& a, int T, const uint16_t* planes, int plane_rows, size_t smem,
                                 hipStream_t s) {
  auto kern = route_prefill_kernel<TG, TN>;
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  constexpr int BT = 16 * TG;
  hipLaunchKernelGGL(kern, dim3((T + BT - 1) / BT), dim3(512), smem, s, a, planes, plane_rows);
  return hipGetLastError();
}

// Second kernel of the split form: a workgroup takes as many tokens as it has waves (phase 2 is
// one wave per token, and with few tokens its latency is the cost), adds the dsplit partial logit
// sums of its tokens in index order and runs phase 2.
__global__ void __launch_bounds__(512) route_finish_kernel(const RouteArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int NW = blockDim.x >> 6;
  const int BT = NW;
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int t0 = blockIdx.x * BT;
  float* lg = reinterpret_cast<float*>(smem + a.region0);         // [BT][NOpad]
  for (int idx = threadIdx.x; idx < BT * a.NO; idx += blockDim.x) {
    const int tl = idx / a.NO, o = idx % a.NO;
    double sum = 0.0;
    if (t0 + tl < a.T)
      for (int sp = 0; sp < a.dsplit; ++sp) sum += a.gpart[((size_t)sp * a.T + t0 + tl) * a.NO + o];
    lg[tl * a.NOpad + o] = (float)sum;
  }
  __syncthreads();
  route_select(a, smem, lg, t0, BT, NW, w, lane);
}

template <bool BF16, int TM, int TN>
static hipError_t launch_one(const RouteArgs& a, dim3 grid, dim3 block, size_t smem, hipStream_t s) {
  auto kern = route_kernel<BF16, TM, TN>;
  static bool attr_done = false;      // more than 64 KB of dynamic LDS needs the opt-in
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  hipLaunchKernelGGL(kern, grid, block, smem, s, a);
  return hipGetLastError();
}

template <bool BF16, int TM>
static hipError_t launch_tn(const RouteArgs& a, int TN, dim3 grid, dim3 block, size_t smem,
                            hipStream_t s) {
  switch (TN) {
    case 1: return launch_one<BF16, TM, 1>(a, grid, block, smem, s);
    case 2: return launch_one<BF16, TM, 2>(a, grid, block, smem, s);
    case 3: return launch_one<BF16, TM, 3>(a, grid, block, smem, s);
    default: return launch_one<BF16, TM, 5>(a, grid, block, smem, s);
  }
}

// Split form: used for at most kSplitMaxT tokens; the workspace holds up to kSplitMax partial
// sums of every logit.
constexpr int kSplitMaxT = 256, kSplitMax = 16;
constexpr int kPrefillMinT = 8192;       // from here on the bf16 matrix-core form (measured: 96 against
                                         // 190 us at 16384 tokens, even at 8192, slower below)

static int tile_cus() {
  static int n = 0;
  if (!n) {
    int dev = 0;
    hipDeviceProp_t p;
    n = (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&p, dev) == hipSuccess && p.multiProcessorCount > 0)
            ? p.multiProcessorCount : 256;
  }
  return n;
}

// the bf16 matrix-core form: bf16 tokens, enough of them, whole 128-deep chunks
static bool prefill_form(const LayerDesc& L, int dtype) {
  return dtype == MOHGE_BF16 && L.T >= kPrefillMinT && L.d % kPfChunk == 0;
}

size_t route_workspace_bytes(const LayerDesc& L, int dtype) {
  if (prefill_form(L, dtype)) {
    // the three bf16 planes of the router rows, rows padded to whole passes of 16 * TN
    const int tiles = (L.Ng + L.Ne + 15) / 16, TNp = tiles >= 5 ? 5 : tiles;
    const size_t rows = (size_t)(tiles + TNp - 1) / TNp * TNp * 16;
    return (3 * rows * L.d * sizeof(uint16_t) + 255) / 256 * 256;
  }
  if (L.T > kSplitMaxT) return 0;
  return ((size_t)kSplitMax * (L.T > 0 ? L.T : 1) * (L.Ng + L.Ne) * sizeof(double) + 255) / 256 * 256;
}

hipError_t launch_route(const LayerDesc& L, int dtype, const void* x, const float* w_group,
                        const float* w_expert, const float* bias, int32_t* group_idx,
                        int32_t* expert_idx, float* gates, float* gs_out, float* es1_out,
                        void* ws, size_t ws_bytes, hipStream_t s) {
  RouteArgs a;
  a.x = x; a.wg = w_group; a.we = w_expert; a.bias = bias;
  a.gidx = group_idx; a.eidx = expert_idx; a.gates = gates; a.gs = gs_out; a.es1 = es1_out;
  a.T = L.T; a.d = L.d; a.Ng = L.Ng; a.N = L.N; a.Ne = L.Ne; a.Kg = L.Kg; a.Ke = L.Ke;
  a.mode = L.select_mode;
  a.NO = L.Ng + L.Ne;
  a.NOpad = ((a.NO + 15) / 16) * 16 + 4;
  a.Nepad = ((L.Ne + 63) / 64) * 64;
  const int NW = (L.d % 256 == 0) ? 8 : (L.d % 128 == 0) ? 4 : 2;
  a.kslice = L.d / NW;
  // few tokens: split the reduction over more workgroups (a slice stays a whole number of
  // 32-element steps) until there are about 128 of them
  a.dsplit = 1;
  a.gpart = nullptr;
  if (ws && L.T <= kSplitMaxT && ws_bytes >= route_workspace_bytes(L, dtype)) {
    const int blocks = (L.T + 15) / 16;
    int ds = 1;
    while (ds * 2 <= kSplitMax && blocks * ds * 2 <= 128 && (a.kslice / (ds * 2)) % 32 == 0 &&
           a.kslice / (ds * 2) >= 32)
      ds *= 2;
    if (ds > 1) {
      a.dsplit = ds;
      a.kslice /= ds;
      a.gpart = static_cast<double*>(ws);
    }
  }
  const int tiles = (a.NO + 15) / 16;
  // many bf16 tokens and a workspace for the split router rows: the bf16 matrix-core form
  if (prefill_form(L, dtype) && ws && ws_bytes >= route_workspace_bytes(L, dtype)) {
    const int TNp = tiles >= 5 ? 5 : tiles;                       // column tiles per pass
    const int plane_rows = (tiles + TNp - 1) / TNp * TNp * 16;
    uint16_t* planes = static_cast<uint16_t*>(ws);
    const long long quads = (long long)plane_rows * (L.d / 4);
    hipLaunchKernelGGL(route_split_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, s, w_group, w_expert,
                       planes, L.Ng, a.NO, plane_rows, L.d);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t buf = (size_t)2 * 3 * 16 * TNp * 256;
    const size_t rows_bytes = (size_t)8 * 5 * a.Nepad * sizeof(float);
    // 64 tokens per workgroup when that still gives every compute unit one, else 32
    for (int TG = (L.T >= 64 * tile_cus()) ? 4 : 2; TG >= 2; TG -= 2) {
      const size_t red = (size_t)16 * TG * 16 * TNp * sizeof(double);
      size_t r0 = buf > rows_bytes ? buf : rows_bytes;
      if (red > r0) r0 = red;
      a.region0 = (int)((r0 + 15) / 16 * 16);
      const size_t smem_p = (size_t)a.region0 + (size_t)16 * TG * a.NOpad * sizeof(float);
      if (smem_p > 160 * 1024) continue;
      switch (TNp * 2 + (TG == 4)) {
        case 2: return launch_prefill<2, 1>(a, L.T, planes, plane_rows, smem_p, s);
        case 3: return launch_prefill<4, 1>(a, L.T, planes, plane_rows, smem_p, s);
        case 4: return launch_prefill<2, 2>(a, L.T, planes, plane_rows, smem_p, s);
        case 5: return launch_prefill<4, 2>(a, L.T, planes, plane_rows, smem_p, s);
        case 6: return launch_prefill<2, 3>(a, L.T, planes, plane_rows, smem_p, s);
        case 7: return launch_prefill<4, 3>(a, L.T, planes, plane_rows, smem_p, s);
        case 8: return launch_prefill<2, 4>(a, L.T, planes, plane_rows, smem_p, s);
        case 9: return launch_prefill<4, 4>(a, L.T, planes, plane_rows, smem_p, s);
        case 10: return launch_prefill<2, 5>(a, L.T, planes, plane_rows, smem_p, s);
        default: return launch_prefill<4, 5>(a, L.T, planes, plane_rows, smem_p, s);
      }
    }
  }
  const int TN = tiles <= 1 ? 1 : tiles == 2 ? 2 : tiles == 3 ? 3 : 5;
  int TM = (L.T >= 16384 && TN <= 2) ? 2 : 1;   // wider combinations would spill registers
  size_t smem = 0;
  for (;; TM = 1) {
    const size_t part_bytes = (size_t)NW * 16 * TM * 16 * TN * sizeof(double);
    const size_t rows_bytes = (size_t)NW * 5 * a.Nepad * sizeof(float);
    a.region0 = (int)(((part_bytes > rows_bytes ? part_bytes : rows_bytes) + 15) / 16 * 16);
    smem = (size_t)a.region0 + (size_t)16 * TM * a.NOpad * sizeof(float);
    if (smem <= 96 * 1024 || TM == 1) break;
  }
  const int BT = 16 * TM;
  dim3 grid((L.T + BT - 1) / BT, a.dsplit), block(64 * NW);
  const bool bf = dtype == MOHGE_BF16;
  hipError_t e;
  if (TM == 2) e = bf ? launch_tn<true, 2>(a, TN, grid, block, smem, s)
                      : launch_tn<false, 2>(a, TN, grid, block, smem, s);
  else e = bf ? launch_tn<true, 1>(a, TN, grid, block, smem, s)
              : launch_tn<false, 1>(a, TN, grid, block, smem, s);
  if (e != hipSuccess || a.dsplit == 1) return e;
  static bool attr_done = false;
  if (!attr_done) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(route_finish_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  hipLaunchKernelGGL(route_finish_kernel, dim3((L.T + NW - 1) / NW), block, smem, s, a);
  return hipGetLastError();
}

}  // namespace mohge
