// Backward pass of the expert networks on gfx950 (bf16 storage, fp32 accumulation).
//
// The paper trains the layer (sections 3.3, 3.4.2 give the loss terms) without spelling out
// the backward pass; it is the chain rule over  y_r = W_down (SiLU(a) * b),  a = W_gate x_r,
// b = W_up x_r  for every routed row r of expert e:
//     dh = W_down^T dy_r
//     da = dh * b * s (1 + a (1 - s)),   db = dh * a * s,   s = sigmoid(a)
//     dx_r = W_gate^T da + W_up^T db
//     dW_down[e] = sum_r dy_r h_r^T,   dW_gate[e] = sum_r da_r x_r^T,   dW_up[e] = sum_r db_r x_r^T
//
// All five products run on the ragged grouped GEMM tile kernel of the forward pass, which
// needs both operands contiguous along the reduction dimension:
//   dH   = dY . (W_down^T)^T     reduction over d     -> needs W_down^T  [N, F, d]
//   dX   = [dA|dB] . (W13^T)^T   reduction over 2F_g  -> needs W13^T     [N, d, 2F]
//   dW2  = dY^T . (H^T)^T        reduction over the expert's rows -> needs dY^T, H^T
//   dW13 = [dA|dB]^T . (X^T)^T   reduction over the expert's rows -> needs [dA|dB]^T, X^T
// The transposed weights are an input (kept by the caller next to the weights, or made with
// the helper below); the transposed activations are written here by a bandwidth-bound
// 64x64 LDS transpose into per-expert windows whose length is rounded up to a multiple of
// 64 rows and zero filled, so that the reduction length of a weight-gradient tile is a whole
// number of 64-deep stages (an expert without rows gets one all-zero stage, which makes its
// gradient come out as zeros through the same path).
#include "common.h"
#include "tiled.h"

namespace mohge {

const void* saved_h(const LayerDesc& L, const void* saved);
const void* saved_pre(const LayerDesc& L, const void* saved);

// ---------------------------------------------------------------------------------------
// padded window offsets
// ---------------------------------------------------------------------------------------
__global__ void __launch_bounds__(64) window_offsets_kernel(const int32_t* __restrict__ offsets,
                                                           int32_t* __restrict__ poff, int Ne) {
  if (threadIdx.x == 0) {
    int p = 0;
    for (int e = 0; e < Ne; ++e) {
      poff[e] = p;
      const int n = offsets[e + 1] - offsets[e];
      p += n > 0 ? (n + 63) / 64 * 64 : 64;
    }
    poff[Ne] = p;
  }
}

// ---------------------------------------------------------------------------------------
// 64 x 64 transposes through LDS
// ---------------------------------------------------------------------------------------
constexpr int kTP = 66;   // padded tile row length in elements (132 bytes)

// thread (i = tid/4, q = tid%4) holds 16 consecutive elements of source row i
__device__ __forceinline__ void tile_put(uint16_t (*tile)[kTP], int i, int q, const uint4 v0,
                                         const uint4 v1) {
  uint32_t* dst = reinterpret_cast<uint32_t*>(&tile[i][q * 16]);
  dst[0] = v0.x; dst[1] = v0.y; dst[2] = v0.z; dst[3] = v0.w;
  dst[4] = v1.x; dst[5] = v1.y; dst[6] = v1.z; dst[7] = v1.w;
}

// thread (f = tid/4, q = tid%4) collects column f of source rows q*16 .. q*16+15
__device__ __forceinline__ void tile_get_t(const uint16_t (*tile)[kTP], int f, int q, uint4& v0,
                                           uint4& v1) {
  uint32_t w[8];
#pragma unroll
  for (int j = 0; j < 8; ++j)
    w[j] = (uint32_t)tile[q * 16 + 2 * j][f] | ((uint32_t)tile[q * 16 + 2 * j + 1][f] << 16);
  v0 = make_uint4(w[0], w[1], w[2], w[3]);
  v1 = make_uint4(w[4], w[5], w[6], w[7]);
}

struct RaggedTransposeArgs {
  const uint16_t* in;       // [rows, ld_in]: sorted positions (or tokens, through perm)
  const int32_t* perm;      // NULL, or sorted position -> pair id (row = pair / Ke)
  const int32_t* offsets;   // [Ne+1]
  const int32_t* poff;      // [Ne+1]
  uint16_t* out;            // [features, ld_out]
  int ld_in, ld_out, Ke, Ne, N;
  int ncols[kMaxGroups];    // valid features of a row of group g
};

// grid.x: 64-wide position blocks of the padded layout, grid.y: 64-wide feature blocks
__global__ void __launch_bounds__(256) ragged_transpose_kernel(const RaggedTransposeArgs a) {
  __shared__ uint16_t tile[64][kTP];
  const int pos0 = blockIdx.x * 64;
  if (pos0 >= a.poff[a.Ne]) return;
  int lo = 0, hi = a.Ne - 1;             // last expert whose window starts at or before pos0
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (a.poff[mid] <= pos0) lo = mid; else hi = mid - 1;
  }
  const int e = lo;
  const int c0 = blockIdx.y * 64;
  if (c0 >= a.ncols[e / a.N]) return;
  const int cnt = a.offsets[e + 1] - a.offsets[e];
  const int local0 = pos0 - a.poff[e];
  const int i = threadIdx.x >> 2, q = threadIdx.x & 3;
  uint4 v0 = make_uint4(0, 0, 0, 0), v1 = v0;
  if (local0 + i < cnt) {
    long long row = a.offsets[e] + local0 + i;
    if (a.perm) row = a.perm[row] / a.Ke;
    const uint4* src = reinterpret_cast<const uint4*>(a.in + row * a.ld_in + c0 + q * 16);
    v0 = src[0];
    v1 = src[1];
  }
  tile_put(tile, i, q, v0, v1);
  __syncthreads();
  tile_get_t(tile, i, q, v0, v1);
  uint4* dst = reinterpret_cast<uint4*>(a.out + (long long)(c0 + i) * a.ld_out + pos0 + q * 16);
  dst[0] = v0;
  dst[1] = v1;
}

// in: [batch, R, C] -> out: [batch, C, R]; R and C are multiples of 64
__global__ void __launch_bounds__(256) weight_transpose_kernel(const uint16_t* __restrict__ in,
                                                               uint16_t* __restrict__ out, int R, int C) {
  __shared__ uint16_t tile[64][kTP];
  const int r0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
  const long long base = (long long)blockIdx.z * R * C;
  const int i = threadIdx.x >> 2, q = threadIdx.x & 3;
  const uint4* src = reinterpret_cast<const uint4*>(in + base + (long long)(r0 + i) * C + c0 + q * 16);
  uint4 v0 = src[0], v1 = src[1];
  tile_put(tile, i, q, v0, v1);
  __syncthreads();
  tile_get_t(tile, i, q, v0, v1);
  uint4* dst = reinterpret_cast<uint4*>(out + base + (long long)(c0 + i) * R + r0 + q * 16);
  dst[0] = v0;
  dst[1] = v1;
}

hipError_t launch_transpose_weights(const LayerDesc& L, const GroupPtrs& W, void* const* w13t,
                                    void* const* w2t, hipStream_t s) {
  for (int g = 0; g < L.Ng; ++g) {
    const int F = L.F[g];
    // W13[g]: N x [2F, d] -> N x [d, 2F];  W2[g]: N x [d, F] -> N x [F, d]
    hipLaunchKernelGGL(weight_transpose_kernel, dim3(2 * F / 64, L.d / 64, L.N), dim3(256), 0, s,
                       static_cast<const uint16_t*>(W.w13[g]), static_cast<uint16_t*>(w13t[g]), 2 * F, L.d);
    hipLaunchKernelGGL(weight_transpose_kernel, dim3(L.d / 64, F / 64, L.N), dim3(256), 0, s,
                       static_cast<const uint16_t*>(W.w2[g]), static_cast<uint16_t*>(w2t[g]), L.d, F);
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// workspace layout and the launch sequence
// ---------------------------------------------------------------------------------------
static size_t up256(size_t b) { return (b + 255) / 256 * 256; }

static int padded_rows(const LayerDesc& L) { return (L.P + 63) / 64 * 64 + 64 * L.Ne; }

struct BwdLayout {
  size_t sched[4], recs[4];   // dgrad-h, dgrad-x, wgrad-2, wgrad-13
  size_t poff, dab, dyt, ht, dabt, xt, total;
};

static BwdLayout bwd_layout(const LayerDesc& L) {
  BwdLayout o;
  const int modes[4] = {kDgradH, kDown, kWgrad, kWgrad};
  size_t p = 0;
  for (int i = 0; i < 4; ++i) {
    o.sched[i] = p; p += 256;
    o.recs[i] = p; p += up256((size_t)tile_capacity(L, modes[i]) * sizeof(TileRec));
  }
  const size_t P = L.P > 0 ? L.P : 1, Pp = padded_rows(L);
  o.poff = p; p += up256((size_t)(L.Ne + 1) * 4);
  o.dab = p;  p += up256(P * 2 * L.Fmax * 2);
  o.dyt = p;  p += up256((size_t)L.d * Pp * 2);
  o.ht = p;   p += up256((size_t)L.Fmax * Pp * 2);
  o.dabt = p; p += up256((size_t)2 * L.Fmax * Pp * 2);
  o.xt = p;   p += up256((size_t)L.d * Pp * 2);
  o.total = p;
  return o;
}

size_t ffn_bwd_workspace_bytes(const LayerDesc& L) { return bwd_layout(L).total; }

hipError_t launch_expert_ffn_bwd(const LayerDesc& L, const void* x, const int32_t* perm,
                                 const int32_t* offsets, const void* const* w13t,
                                 const void* const* w2t, const void* saved, const void* dy_perm,
                                 void* dx_perm, void* const* dw13, void* const* dw2, void* ws,
                                 hipStream_t s) {
  const BwdLayout lay = bwd_layout(L);
  unsigned char* base = static_cast<unsigned char*>(ws);
  int32_t* poff = reinterpret_cast<int32_t*>(base + lay.poff);
  uint16_t* dab = reinterpret_cast<uint16_t*>(base + lay.dab);
  uint16_t* dyt = reinterpret_cast<uint16_t*>(base + lay.dyt);
  uint16_t* ht = reinterpret_cast<uint16_t*>(base + lay.ht);
  uint16_t* dabt = reinterpret_cast<uint16_t*>(base + lay.dabt);
  uint16_t* xt = reinterpret_cast<uint16_t*>(base + lay.xt);
  const int Pp = padded_rows(L);

  TileArgs t{};
  t.offsets = offsets;
  t.Ke = L.Ke; t.Ng = L.Ng; t.N = L.N; t.Ne = L.Ne; t.d = L.d; t.P = L.P;
  t.ncu = tile_num_cus();
  t.ldpre = 2 * L.Fmax;
  for (int g = 0; g < kMaxGroups; ++g) t.order[g] = g;
  for (int i = 1; i < L.Ng; ++i)
    for (int j = i; j > 0 && L.F[t.order[j]] > L.F[t.order[j - 1]]; --j) {
      const int tmp = t.order[j]; t.order[j] = t.order[j - 1]; t.order[j - 1] = tmp;
    }
  auto with_sched = [&](TileArgs a, int i) {
    a.hdr = reinterpret_cast<SchedHeader*>(base + lay.sched[i]);
    a.recs = reinterpret_cast<TileRec*>(base + lay.recs[i]);
    return a;
  };

  hipLaunchKernelGGL(window_offsets_kernel, dim3(1), dim3(64), 0, s, offsets, poff, L.Ne);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;

  // dH = dY W_down, fused with the SwiGLU derivative: [dA|dB] rows
  {
    TileArgs a = with_sched(t, 0);
    a.A = static_cast<const uint16_t*>(dy_perm);
    a.lda = L.d;
    a.pre = const_cast<uint16_t*>(static_cast<const uint16_t*>(saved_pre(L, saved)));
    a.C2 = dab;
    for (int g = 0; g < L.Ng; ++g) { a.F[g] = L.F[g]; a.W[g] = static_cast<const uint16_t*>(w2t[g]); }
    e = launch_tile_gemm(kDgradH, a, s);
    if (e != hipSuccess) return e;
  }
  // dX = [dA|dB] W13: the down-projection form with reduction length 2 F_g
  {
    TileArgs a = with_sched(t, 1);
    a.A = dab;
    a.lda = 2 * L.Fmax;
    a.C = static_cast<uint16_t*>(dx_perm);
    a.ldc = L.d;
    for (int g = 0; g < L.Ng; ++g) { a.F[g] = 2 * L.F[g]; a.W[g] = static_cast<const uint16_t*>(w13t[g]); }
    e = launch_tile_gemm(kDown, a, s);
    if (e != hipSuccess) return e;
  }
  // transposed activations in zero-padded per-expert windows
  {
    RaggedTransposeArgs r{};
    r.offsets = offsets; r.poff = poff; r.Ke = L.Ke; r.Ne = L.Ne; r.N = L.N; r.ld_out = Pp;
    const unsigned pb = (unsigned)(Pp / 64);
    auto run = [&](const void* in, int ld_in, const int32_t* pm, uint16_t* out, int mult, int fixed) {
      RaggedTransposeArgs q = r;
      q.in = static_cast<const uint16_t*>(in); q.ld_in = ld_in; q.perm = pm; q.out = out;
      int cmax = 0;
      for (int g = 0; g < L.Ng; ++g) {
        q.ncols[g] = fixed ? fixed : mult * L.F[g];
        if (q.ncols[g] > cmax) cmax = q.ncols[g];
      }
      hipLaunchKernelGGL(ragged_transpose_kernel, dim3(pb, (unsigned)(cmax / 64)), dim3(256), 0, s, q);
    };
    run(dy_perm, L.d, nullptr, dyt, 0, L.d);
    run(saved_h(L, saved), L.Fmax, nullptr, ht, 1, 0);
    run(dab, 2 * L.Fmax, nullptr, dabt, 2, 0);
    run(x, L.d, perm, xt, 0, L.d);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  // dW_down[e] = dY_e^T H_e : rows d, columns F_g
  {
    TileArgs a = with_sched(t, 2);
    a.A = dyt; a.lda = Pp; a.B2 = ht; a.ldb = Pp; a.poff = poff; a.force_rows = 256;
    for (int g = 0; g < L.Ng; ++g) {
      a.F[g] = L.F[g]; a.Mrows[g] = L.d; a.Ncols[g] = L.F[g];
      a.Wout[g] = static_cast<uint16_t*>(dw2[g]);
    }
    e = launch_tile_gemm(kWgrad, a, s);
    if (e != hipSuccess) return e;
  }
  // dW13[e] = [dA|dB]_e^T X_e : rows 2 F_g (gate rows, then up rows), columns d
  {
    TileArgs a = with_sched(t, 3);
    a.A = dabt; a.lda = Pp; a.B2 = xt; a.ldb = Pp; a.poff = poff; a.force_rows = 256;
    for (int g = 0; g < L.Ng; ++g) {
      a.F[g] = L.F[g]; a.Mrows[g] = 2 * L.F[g]; a.Ncols[g] = L.d;
      a.Wout[g] = static_cast<uint16_t*>(dw13[g]);
    }
    e = launch_tile_gemm(kWgrad, a, s);
  }
  return e;
}

}  // namespace mohge
