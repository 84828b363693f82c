// Expert feed-forward networks for prefill-sized token counts on gfx950: a ragged
// grouped GEMM on the bf16 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulate).
//
// Two launches: "up" computes H = SiLU(X W_gate^T) * (X W_up^T) for every expert's
// rows, "down" computes Y = H W_down^T.  Both have the form C[rows of expert e] =
// A_rows . B_e^T with A and B contiguous along the reduction dimension.  What makes it
// ragged: the row count n_e comes from the router (device memory `offsets`), the width
// F_g differs from group to group (it is N of the up and K of the down projection).
//
// Tile schedule, derived on the device: tile -> (expert, row tile, column tile) by a
// wave-wide prefix sum over the experts' tile counts; workgroup ids are first folded so
// that each of the 8 XCDs (own L2 each) walks a contiguous range of tiles, and inside
// an expert row tiles vary fastest so that neighbours share the weight tile.
//
// Data path: global -> LDS with global_load_lds_dwordx4 (no staging registers), two
// stages; 16-byte chunks are XOR-swizzled inside each 128-byte tile row so that the
// ds_read_b128 operand reads do not collide on banks.  The token gather is fused: a
// tile row's global address is taken through `perm`.  The MFMA is issued with the
// weight fragment as the first operand so that a lane ends up with 4 consecutive
// output features of one token, which pack into one 8-byte store.
#include "common.h"

namespace mohge {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct TileArgs {
  const uint16_t* A;          // up: x [T,d] (gathered through perm) or [P,d]; down: H [P,lda]
  const int32_t* perm;        // up only, may be NULL
  const int32_t* offsets;     // [Ne+1]
  const uint16_t* W[kMaxGroups];   // up: w13[g] [N,2F,d]; down: w2[g] [N,d,F]
  uint16_t* C;                // up: H [P,ldc]; down: y_perm [P,ldc]
  int lda, ldc;
  int Ke, Ng, N, Ne, d;
  int F[kMaxGroups];
  int order[kMaxGroups];      // groups in visiting order
};

template <int BM, int BN, bool UP>
struct TileCoord {
  int e, g, i, row0, rows, m0, n0, F;
  bool valid;
};

__device__ __forceinline__ int wave_incl_scan(int v, int lane) {
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int up = __shfl_up(v, off, 64);
    if (lane >= off) v += up;
  }
  return v;
}

// Maps this workgroup to a tile.  Every wave computes it redundantly (no LDS, no barrier).
template <int BM, int BN, bool UP>
__device__ __forceinline__ TileCoord<BM, BN, UP> find_tile(const TileArgs& a, int lane) {
  TileCoord<BM, BN, UP> tc;
  tc.valid = false;
  // tiles per expert, in visiting order v = position of (group order, expert in group)
  int incl[4], ev[4], cntv[4];
  int carry = 0;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    incl[c] = 0; ev[c] = 0; cntv[c] = 0;
    if (64 * c < a.Ne) {
      const int v = lane + 64 * c;
      int tiles = 0;
      if (v < a.Ne) {
        const int g = a.order[v / a.N];
        const int e = g * a.N + v % a.N;
        const int cnt = a.offsets[e + 1] - a.offsets[e];
        const int ncols = UP ? a.F[g] : a.d;
        constexpr int NCOLS_PER_TILE = UP ? BN / 2 : BN;
        tiles = ((cnt + BM - 1) / BM) * ((ncols + NCOLS_PER_TILE - 1) / NCOLS_PER_TILE);
        ev[c] = e;
        cntv[c] = cnt;
      }
      const int s = wave_incl_scan(tiles, lane);
      incl[c] = carry + s;
      carry += __shfl(s, 63, 64);
    }
  }
  const int total = carry;
  // fold workgroup ids so that XCD x (which receives ids x, x+8, ...) gets a contiguous range
  const int chunk = (total + 7) / 8;
  const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
  const int tile = xcd * chunk + local;
  if (local >= chunk || tile >= total) return tc;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    if (64 * c < a.Ne && !tc.valid) {
      const unsigned long long m = __ballot(tile < incl[c]);
      if (m) {
        const int src = __ffsll((long long)m) - 1;
        const int e = __shfl(ev[c], src, 64);
        const int cnt = __shfl(cntv[c], src, 64);
        const int hi = __shfl(incl[c], src, 64);
        const int mt = (cnt + BM - 1) / BM;
        const int g = e / a.N;
        constexpr int NCOLS_PER_TILE = UP ? BN / 2 : BN;
        const int ncols = UP ? a.F[g] : a.d;
        const int nt = (ncols + NCOLS_PER_TILE - 1) / NCOLS_PER_TILE;
        const int lo = hi - mt * nt;
        const int rel = tile - lo;
        tc.e = e; tc.g = g; tc.i = e % a.N; tc.F = a.F[g];
        tc.row0 = a.offsets[e];
        tc.rows = cnt;
        tc.m0 = (rel % mt) * BM;
        tc.n0 = (rel / mt) * NCOLS_PER_TILE;
        tc.valid = true;
      }
    }
  }
  return tc;
}

__device__ __forceinline__ void async_copy16(const void* gptr, void* lds_uniform_base) {
  __builtin_amdgcn_global_load_lds(
      (const __attribute__((address_space(1))) void*)gptr,
      (__attribute__((address_space(3))) void*)lds_uniform_base, 16, 0, 0);
}

// BM x BN output tile (BM tokens, BN weight rows), BK = 64, WGM x WGN waves, SH = swizzle shift.
template <int BM, int BN, int WGM, int WGN, int SH, bool UP>
__global__ void __launch_bounds__(64 * WGM * WGN) ffn_tile_kernel(const TileArgs a) {
  constexpr int BK = 64;
  constexpr int NWAVES = WGM * WGN, NT = 64 * NWAVES;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;   // wave tile: tokens x weight rows
  constexpr int MF = WTM / 32, NF = WTN / 32;
  constexpr int A_LOADS = BM * 8 / NT, B_LOADS = BN * 8 / NT;
  constexpr int STAGE_BYTES = (BM + BN) * BK * 2;
  static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0, "tile rows must divide over the waves");
  static_assert(!UP || NF % 2 == 0, "gate and up halves per wave");
  extern __shared__ __align__(1024) unsigned char lds[];

  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const TileCoord<BM, BN, UP> tc = find_tile<BM, BN, UP>(a, lane);
  if (!tc.valid) return;
  const int e_i = tc.i, g = tc.g, F = tc.F;
  const int K = UP ? a.d : F;
  const int rows_left = tc.rows - tc.m0;           // valid token rows in this tile (>= 1)

  // ---- global source pointers of this thread's 16-byte chunks -------------------
  // load instruction j of wave w fills LDS tile rows (j*NWAVES + w)*8 .. +7; lane l
  // fills row l/8, physical chunk l%8, which holds logical chunk (l%8) ^ swz(row).
  const int lrow = lane >> 3, lpos = lane & 7;
  const uint16_t* a_src[A_LOADS];
  const uint16_t* b_src[B_LOADS];
#pragma unroll
  for (int j = 0; j < A_LOADS; ++j) {
    const int row = (j * NWAVES + w) * 8 + lrow;
    int rr = tc.m0 + row;
    if (rr > tc.rows - 1) rr = tc.rows - 1;         // rows past the expert's end: any valid row
    const int pos = tc.row0 + rr;
    long long src_row;
    if constexpr (UP) src_row = a.perm ? (long long)(a.perm[pos] / a.Ke) : (long long)pos;
    else src_row = pos;
    const int chunk = lpos ^ ((row >> SH) & 7);
    a_src[j] = a.A + src_row * a.lda + chunk * 8;
  }
#pragma unroll
  for (int j = 0; j < B_LOADS; ++j) {
    const int row = (j * NWAVES + w) * 8 + lrow;
    const int chunk = lpos ^ ((row >> SH) & 7);
    long long wrow;
    if constexpr (UP) {
      // tile rows [0, BN/2): W_gate rows n0.., rows [BN/2, BN): W_up rows n0..
      const int half = row >= BN / 2;
      int f = tc.n0 + (row - half * (BN / 2));
      if (f > F - 1) f = F - 1;
      wrow = (long long)e_i * 2 * F + (long long)half * F + f;
    } else {
      int n = tc.n0 + row;
      if (n > a.d - 1) n = a.d - 1;
      wrow = (long long)e_i * a.d + n;
    }
    b_src[j] = a.W[g] + wrow * K + chunk * 8;
  }

  // ---- LDS read offsets of the MFMA operand fragments ----------------------------
  // fragment row = base + lane%32, logical chunk = 2*kk + lane/32
  const int frow = lane & 31, fh = lane >> 5;
  int foff[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) foff[kk] = frow * 128 + (((2 * kk + fh) ^ ((frow >> SH) & 7)) << 4);
  const int wm = w / WGN, wn = w % WGN;
  // token fragments live in the A part, weight fragments in the B part of a stage
  int xbase[MF], wbase[NF];
#pragma unroll
  for (int ti = 0; ti < MF; ++ti) xbase[ti] = (wm * WTM + ti * 32) * 128;
#pragma unroll
  for (int fi = 0; fi < NF; ++fi) {
    int row;
    if constexpr (UP) {
      constexpr int NFh = NF / 2;
      row = (fi < NFh) ? wn * (WTN / 2) + fi * 32 : BN / 2 + wn * (WTN / 2) + (fi - NFh) * 32;
    } else {
      row = wn * WTN + fi * 32;
    }
    wbase[fi] = BM * 128 + row * 128;
  }

  f32x16 acc[NF][MF];
#pragma unroll
  for (int fi = 0; fi < NF; ++fi)
#pragma unroll
    for (int ti = 0; ti < MF; ++ti)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[fi][ti][r] = 0.f;

  auto issue = [&](int stage, int k0) {
    unsigned char* sb = lds + stage * STAGE_BYTES;
#pragma unroll
    for (int j = 0; j < A_LOADS; ++j)
      async_copy16(a_src[j] + k0, sb + (j * NWAVES + w) * 1024);
#pragma unroll
    for (int j = 0; j < B_LOADS; ++j)
      async_copy16(b_src[j] + k0, sb + BM * 128 + (j * NWAVES + w) * 1024);
  };

  const int KT = K / BK;
  issue(0, 0);
  for (int kt = 0; kt < KT; ++kt) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (kt + 1 < KT) issue((kt + 1) & 1, (kt + 1) * BK);
    const unsigned char* sb = lds + (kt & 1) * STAGE_BYTES;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      bf16x8 xf[MF], wf[NF];
#pragma unroll
      for (int ti = 0; ti < MF; ++ti) xf[ti] = *reinterpret_cast<const bf16x8*>(sb + xbase[ti] + foff[kk]);
#pragma unroll
      for (int fi = 0; fi < NF; ++fi) wf[fi] = *reinterpret_cast<const bf16x8*>(sb + wbase[fi] + foff[kk]);
#pragma unroll
      for (int fi = 0; fi < NF; ++fi)
#pragma unroll
        for (int ti = 0; ti < MF; ++ti)
          acc[fi][ti] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[fi], xf[ti], acc[fi][ti], 0, 0, 0);
    }
  }

  // ---- epilogue: lane holds, per 32x32 block, token lane%32 and weight rows
  // 8*(r/4) + 4*(lane/32) + r%4, i.e. 4 runs of 4 consecutive output features ---------
  const int tok_l = lane & 31, fsub = (lane >> 5) * 4;
  constexpr int NFo = UP ? NF / 2 : NF;
  const int ncols = UP ? F : a.d;
#pragma unroll
  for (int ti = 0; ti < MF; ++ti) {
    const int trow = wm * WTM + ti * 32 + tok_l;
    if (trow >= rows_left) continue;
    uint16_t* crow = a.C + (long long)(tc.row0 + tc.m0 + trow) * a.ldc;
#pragma unroll
    for (int fi = 0; fi < NFo; ++fi) {
      const int cbase = tc.n0 + (UP ? wn * (WTN / 2) : wn * WTN) + fi * 32 + fsub;
#pragma unroll
      for (int blk = 0; blk < 4; ++blk) {
        const int col = cbase + blk * 8;
        float v[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          if constexpr (UP) {
            const float gt = acc[fi][ti][blk * 4 + b], up = acc[fi + NF / 2][ti][blk * 4 + b];
            v[b] = gt / (1.f + __expf(-gt)) * up;
          } else {
            v[b] = acc[fi][ti][blk * 4 + b];
          }
        }
        if (col < ncols) {
          uint2 o;
          o.x = pack_bf16x2(v[0], v[1]);
          o.y = pack_bf16x2(v[2], v[3]);
          *reinterpret_cast<uint2*>(crow + col) = o;
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------
template <int BM, int BN, int WGM, int WGN, int SH, bool UP>
static hipError_t launch_tile(const TileArgs& a, int P, int maxcols, hipStream_t s) {
  constexpr int NCOLS_PER_TILE = UP ? BN / 2 : BN;
  constexpr size_t smem = 2 * (size_t)(BM + BN) * 64 * 2;
  auto kern = ffn_tile_kernel<BM, BN, WGM, WGN, SH, UP>;
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  // upper bound on the number of tiles: every expert adds at most one partial row tile
  const long long mt_bound = (long long)P / BM + a.Ne;
  const long long nt_max = (maxcols + NCOLS_PER_TILE - 1) / NCOLS_PER_TILE;
  long long grid = mt_bound * nt_max;
  grid = (grid + 7) / 8 * 8;
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(64 * WGM * WGN), smem, s, a);
  return hipGetLastError();
}

hipError_t launch_ffn_tiled(const LayerDesc& L, const void* x, const int32_t* perm,
                            const int32_t* offsets, const GroupPtrs& W, void* y_perm, void* ws,
                            hipStream_t s, int stages) {
  TileArgs up;
  up.A = static_cast<const uint16_t*>(x);
  up.perm = perm;
  up.offsets = offsets;
  up.C = static_cast<uint16_t*>(ws);
  up.lda = L.d; up.ldc = L.Fmax;
  up.Ke = L.Ke; up.Ng = L.Ng; up.N = L.N; up.Ne = L.Ne; up.d = L.d;
  // visit groups by decreasing width so that the longest tiles are scheduled first
  int order[kMaxGroups];
  for (int g = 0; g < kMaxGroups; ++g) order[g] = g;
  for (int i = 1; i < L.Ng; ++i)
    for (int j = i; j > 0 && L.F[order[j]] > L.F[order[j - 1]]; --j) {
      int t = order[j]; order[j] = order[j - 1]; order[j - 1] = t;
    }
  for (int g = 0; g < kMaxGroups; ++g) {
    up.F[g] = L.F[g];
    up.order[g] = order[g];
    up.W[g] = static_cast<const uint16_t*>(W.w13[g]);
  }
  TileArgs dn = up;
  dn.A = static_cast<const uint16_t*>(ws);
  dn.perm = nullptr;
  dn.C = static_cast<uint16_t*>(y_perm);
  dn.lda = L.Fmax; dn.ldc = L.d;
  for (int g = 0; g < kMaxGroups; ++g) dn.W[g] = static_cast<const uint16_t*>(W.w2[g]);

  hipError_t e = hipSuccess;
  if (stages & 1) e = launch_tile<256, 256, 2, 2, 1, true>(up, L.P, L.Fmax, s);
  if (e != hipSuccess) return e;
  if (stages & 2) e = launch_tile<256, 256, 2, 2, 1, false>(dn, L.P, L.d, s);
  return e;
}

}  // namespace mohge
