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
#include <type_traits>

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
  long long* dbg;             // timing probe only: 8 timestamps per workgroup, else NULL
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

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Probe modes for tuning runs (results are meaningless in the non-zero modes, every access
// stays in bounds): 1 = global loads only in the prologue (matrix-core + LDS rate with a
// perfect memory system), 2 = no matrix-core work (rate of the global -> LDS feed alone).
enum { PROBE_NONE = 0, PROBE_NO_LOADS = 1, PROBE_NO_MFMA = 2 };

// BM x BN output tile (BM tokens, BN weight rows), BK reduction elements per stage, NST
// LDS stages, WGM x WGN waves.
template <int BM, int BN, int BK, int NST, int WGM, int WGN, bool UP, int PROBE>
__global__ void __launch_bounds__(64 * WGM * WGN) ffn_tile_kernel(const TileArgs a) {
  constexpr int NWAVES = WGM * WGN, NT = 64 * NWAVES;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;   // wave tile: tokens x weight rows
  constexpr int MF = WTM / 32, NF = WTN / 32;
  constexpr int CH = BK / 8;                      // 16-byte chunks per tile row
  constexpr int ROWB = BK * 2;                    // bytes per tile row
  constexpr int RPL = 64 / CH;                    // tile rows filled by one wave-wide load
  constexpr int SH = (CH == 8) ? 1 : 2;           // swizzle: chunk ^= (row >> SH) & (CH-1)
  constexpr int KK = BK / 16;
  constexpr int A_LOADS = BM * CH / NT, B_LOADS = BN * CH / NT, LPS = A_LOADS + B_LOADS;
  constexpr int STAGE_BYTES = (BM + BN) * ROWB;
  static_assert(BM * CH % NT == 0 && BN * CH % NT == 0, "tile rows must divide over the waves");
  static_assert(!UP || NF % 2 == 0, "gate and up halves per wave");
  static_assert(NST >= 2 && NST <= 4 && (NST - 2) * LPS < 64, "stage count");
  extern __shared__ __align__(1024) unsigned char lds[];

  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const TileCoord<BM, BN, UP> tc = find_tile<BM, BN, UP>(a, lane);
  if (!tc.valid) return;
  const int e_i = tc.i, g = tc.g, F = tc.F;
  const int K = UP ? a.d : F;
  const int rows_left = tc.rows - tc.m0;           // valid token rows in this tile (>= 1)

  // ---- global source pointers of this thread's 16-byte chunks -------------------
  // load instruction j of wave w fills LDS tile rows (j*NWAVES + w)*RPL .. +RPL-1; lane l
  // fills row l/CH, physical chunk l%CH, which holds logical chunk (l%CH) ^ swz(row).
  const int lrow = lane / CH, lpos = lane % CH;
  const uint16_t* a_src[A_LOADS];
  const uint16_t* b_src[B_LOADS];
#pragma unroll
  for (int j = 0; j < A_LOADS; ++j) {
    const int row = (j * NWAVES + w) * RPL + lrow;
    int rr = tc.m0 + row;
    if (rr > tc.rows - 1) rr = tc.rows - 1;         // rows past the expert's end: any valid row
    const int pos = tc.row0 + rr;
    long long src_row;
    if constexpr (UP) src_row = a.perm ? (long long)(a.perm[pos] / a.Ke) : (long long)pos;
    else src_row = pos;
    const int chunk = lpos ^ ((row >> SH) & (CH - 1));
    a_src[j] = a.A + src_row * a.lda + chunk * 8;
  }
#pragma unroll
  for (int j = 0; j < B_LOADS; ++j) {
    const int row = (j * NWAVES + w) * RPL + lrow;
    const int chunk = lpos ^ ((row >> SH) & (CH - 1));
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
  int foff[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk)
    foff[kk] = frow * ROWB + (((2 * kk + fh) ^ ((frow >> SH) & (CH - 1))) << 4);
  const int wm = w / WGN, wn = w % WGN;
  // token fragments live in the A part, weight fragments in the B part of a stage
  int xbase[MF], wbase[NF];
#pragma unroll
  for (int ti = 0; ti < MF; ++ti) xbase[ti] = (wm * WTM + ti * 32) * ROWB;
#pragma unroll
  for (int fi = 0; fi < NF; ++fi) {
    int row;
    if constexpr (UP) {
      constexpr int NFh = NF / 2;
      row = (fi < NFh) ? wn * (WTN / 2) + fi * 32 : BN / 2 + wn * (WTN / 2) + (fi - NFh) * 32;
    } else {
      row = wn * WTN + fi * 32;
    }
    wbase[fi] = BM * ROWB + row * ROWB;
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
      async_copy16(b_src[j] + k0, sb + BM * ROWB + (j * NWAVES + w) * 1024);
  };

  // NST-stage pipeline: stage kt+NST-1 is requested while stage kt is consumed
  const int KT = K / BK;
#pragma unroll
  for (int s = 0; s < NST - 1; ++s)
    if (s < KT) issue(s, s * BK);
  for (int kt = 0; kt < KT; ++kt) {
    // wait until this thread's loads of stage kt have landed: at most `ahead` later stages
    // may still be in flight
    int ahead = KT - 1 - kt;
    if (ahead > NST - 2) ahead = NST - 2;
    if (PROBE == PROBE_NO_LOADS && kt >= 1) ahead = 3;
    if (ahead == 0) wait_vmcnt<0>();
    else if (ahead == 1) wait_vmcnt<LPS>();
    else if (ahead == 2) wait_vmcnt<(NST > 3 ? 2 * LPS : 0)>();
    __syncthreads();
    if (kt + NST - 1 < KT && (PROBE != PROBE_NO_LOADS))
      issue((kt + NST - 1) % NST, (kt + NST - 1) * BK);
    const unsigned char* sb = lds + (kt % NST) * STAGE_BYTES;
    if constexpr (PROBE != PROBE_NO_MFMA) {
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
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
// Second generation of the tile kernel: 256 x 256 tile, BK = 32, four LDS stages, and a
// hand-ordered inner loop.  One workgroup barrier per stage sits in the MIDDLE of the
// stage's matrix-core work: operand fragments for the next 16-deep slice are read from LDS
// into a second register set while the current set feeds the MFMAs, and the global -> LDS
// requests for the stage three ahead are issued between MFMAs, so that neither LDS latency
// nor the barrier nor the address arithmetic of the loads leaves the matrix core idle.
//   stage kt, first half : MFMA(set0) interleaved with ds_read(stage kt, k 16..31 -> set1)
//   middle               : wait for this thread's loads of stage kt+1, barrier
//   stage kt, second half: MFMA(set1) interleaved with ds_read(stage kt+1, k 0..15 -> set0)
//                          and the loads of stage kt+3 (its buffer held stage kt-1, which
//                          every wave has left once it passed the barrier)
#define MOHGE_PIN() __builtin_amdgcn_sched_barrier(0)

template <int WGM, int WGN, bool UP, int PROBE>
__global__ void __launch_bounds__(64 * WGM * WGN) ffn_tile_kernel_v2(const TileArgs a) {
  constexpr int BM = 256, BN = 256, BK = 32, NST = 4;
  constexpr int NWAVES = WGM * WGN, NT = 64 * NWAVES;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int MF = WTM / 32, NF = WTN / 32;
  constexpr int CH = 4, ROWB = 64, RPL = 16, SH = 2;
  constexpr int A_LOADS = BM * CH / NT, B_LOADS = BN * CH / NT, LPS = A_LOADS + B_LOADS;
  constexpr int STAGE_BYTES = (BM + BN) * ROWB;
  constexpr int NM = MF * NF;       // MFMAs per half stage
  constexpr int NR = MF + NF;       // fragment reads per half stage
  static_assert(!UP || NF % 2 == 0, "gate and up halves per wave");
  static_assert(NR <= NM && LPS <= NM, "interleave slots");
  extern __shared__ __align__(1024) unsigned char lds[];

  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  long long ts[8];
  ts[0] = __builtin_amdgcn_s_memtime();
  const TileCoord<BM, BN, UP> tc = find_tile<BM, BN, UP>(a, lane);
  if (!tc.valid) return;
  ts[1] = __builtin_amdgcn_s_memtime();
  const int e_i = tc.i, g = tc.g, F = tc.F;
  const int K = UP ? a.d : F;
  const int rows_left = tc.rows - tc.m0;

  const int lrow = lane / CH, lpos = lane % CH;
  const uint16_t* src[LPS];
#pragma unroll
  for (int j = 0; j < A_LOADS; ++j) {
    const int row = (j * NWAVES + w) * RPL + lrow;
    int rr = tc.m0 + row;
    if (rr > tc.rows - 1) rr = tc.rows - 1;
    const int pos = tc.row0 + rr;
    long long src_row;
    if constexpr (UP) src_row = a.perm ? (long long)(a.perm[pos] / a.Ke) : (long long)pos;
    else src_row = pos;
    const int chunk = lpos ^ ((row >> SH) & (CH - 1));
    src[j] = a.A + src_row * a.lda + chunk * 8;
  }
#pragma unroll
  for (int j = 0; j < B_LOADS; ++j) {
    const int row = (j * NWAVES + w) * RPL + lrow;
    const int chunk = lpos ^ ((row >> SH) & (CH - 1));
    long long wrow;
    if constexpr (UP) {
      const int half = row >= BN / 2;
      int f = tc.n0 + (row - half * (BN / 2));
      if (f > F - 1) f = F - 1;
      wrow = (long long)e_i * 2 * F + (long long)half * F + f;
    } else {
      int n = tc.n0 + row;
      if (n > a.d - 1) n = a.d - 1;
      wrow = (long long)e_i * a.d + n;
    }
    src[A_LOADS + j] = a.W[g] + wrow * K + chunk * 8;
  }
  // LDS destination (wave-uniform) of load j inside a stage
  auto dst_off = [&](int j) {
    return j < A_LOADS ? (j * NWAVES + w) * 1024 : BM * ROWB + ((j - A_LOADS) * NWAVES + w) * 1024;
  };

  const int frow = lane & 31, fh = lane >> 5;
  int foff[2];
#pragma unroll
  for (int kk = 0; kk < 2; ++kk)
    foff[kk] = frow * ROWB + (((2 * kk + fh) ^ ((frow >> SH) & (CH - 1))) << 4);
  const int wm = w / WGN, wn = w % WGN;
  int fbase[NR];     // token fragments first, then weight fragments
#pragma unroll
  for (int ti = 0; ti < MF; ++ti) fbase[ti] = (wm * WTM + ti * 32) * ROWB;
#pragma unroll
  for (int fi = 0; fi < NF; ++fi) {
    int row;
    if constexpr (UP) {
      constexpr int NFh = NF / 2;
      row = (fi < NFh) ? wn * (WTN / 2) + fi * 32 : BN / 2 + wn * (WTN / 2) + (fi - NFh) * 32;
    } else {
      row = wn * WTN + fi * 32;
    }
    fbase[MF + fi] = BM * ROWB + row * ROWB;
  }

  f32x16 acc[NF][MF];
#pragma unroll
  for (int fi = 0; fi < NF; ++fi)
#pragma unroll
    for (int ti = 0; ti < MF; ++ti)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[fi][ti][r] = 0.f;

  const int KT = K / BK;
  auto issue_stage = [&](int st) {
    unsigned char* sb = lds + (st & (NST - 1)) * STAGE_BYTES;
#pragma unroll
    for (int j = 0; j < LPS; ++j) async_copy16(src[j] + st * BK, sb + dst_off(j));
  };
  auto read_frag = [&](const unsigned char* sb, int kk, int r) {
    return *reinterpret_cast<const bf16x8*>(sb + fbase[r] + foff[kk]);
  };

  // prologue: request stages 0..2, wait for stage 0, read its first fragments
  ts[2] = __builtin_amdgcn_s_memtime();
#pragma unroll
  for (int st = 0; st < NST - 1; ++st)
    if (st < KT) issue_stage(st);
  if (KT >= 3) wait_vmcnt<2 * LPS>();
  else if (KT == 2) wait_vmcnt<LPS>();
  else wait_vmcnt<0>();
  __builtin_amdgcn_s_barrier();
  MOHGE_PIN();
  ts[3] = __builtin_amdgcn_s_memtime();
  bf16x8 f0[NR], f1[NR];
#pragma unroll
  for (int r = 0; r < NR; ++r) f0[r] = read_frag(lds, 0, r);

  // one half stage: NM MFMAs on `use`; after MFMA i the i-th fragment read into `nxt`; the
  // last LPS MFMAs are each followed by one global -> LDS request when LOADS is set
  auto half = [&](bf16x8 (&use)[NR], bf16x8 (&nxt)[NR], const unsigned char* sb_next, int kk_next,
                  auto LOADS, int st_load) {
#pragma unroll
    for (int i = 0; i < NM; ++i) {
      const int fi = i / MF, ti = i % MF;
      if constexpr (PROBE != PROBE_NO_MFMA)
        acc[fi][ti] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(use[MF + fi], use[ti], acc[fi][ti], 0, 0, 0);
      MOHGE_PIN();
      if (i < NR) {
        if constexpr (PROBE != PROBE_NO_MFMA) nxt[i] = read_frag(sb_next, kk_next, i);
        MOHGE_PIN();
      }
      if constexpr (decltype(LOADS)::value) {
        if (i >= NM - LPS) {
          const int j = i - (NM - LPS);
          unsigned char* sb = lds + (st_load & (NST - 1)) * STAGE_BYTES;
          async_copy16(src[j] + st_load * BK, sb + dst_off(j));
          MOHGE_PIN();
        }
      }
    }
  };

  auto stage = [&](int kt, auto LOADS) {
    const unsigned char* sb = lds + (kt & (NST - 1)) * STAGE_BYTES;
    const unsigned char* sbn = lds + ((kt + 1) & (NST - 1)) * STAGE_BYTES;
    half(f0, f1, sb, 1, std::false_type{}, 0);
    // stage kt+1 must be complete before anyone reads it in the second half
    if (PROBE != PROBE_NO_LOADS) {
      if (kt + 2 < KT) wait_vmcnt<LPS>();
      else wait_vmcnt<0>();
    }
    __builtin_amdgcn_s_barrier();
    MOHGE_PIN();
    half(f1, f0, sbn, 0, LOADS, kt + NST - 1);
  };

  int kt = 0;
  if constexpr (PROBE != PROBE_NO_LOADS) {
    for (; kt + NST - 1 < KT; ++kt) stage(kt, std::true_type{});
  }
  for (; kt < KT; ++kt) stage(kt, std::false_type{});
  ts[4] = __builtin_amdgcn_s_memtime();

  // ---- epilogue: accumulators -> bf16 -> a wave-private LDS patch -> 16-byte stores ------
  // A lane holds, per 32x32 block, token lane%32 and weight rows 8*(r/4) + 4*(lane/32) +
  // r%4: runs of 4 consecutive output features.  Writing those straight to global memory
  // scatters 8-byte pieces over 32 rows per instruction; instead every wave transposes its
  // part through LDS (row stride padded by 16 bytes against bank conflicts) and stores whole
  // 128- or 256-byte row segments.
  __syncthreads();                     // all waves are done reading the stages
  {
    constexpr int OC = UP ? WTN / 2 : WTN;           // output features of this wave
    constexpr int RS = OC * 2 + 16;                  // LDS row stride in bytes
    constexpr int TPP = (NWAVES * WTM * RS <= NST * STAGE_BYTES) ? WTM : WTM / 2;   // tokens per pass
    constexpr int EPI_BYTES = TPP * RS;
    constexpr int CPR = OC * 2 / 16;                 // 16-byte chunks per row
    constexpr int NFo = UP ? NF / 2 : NF;
    static_assert(NWAVES * EPI_BYTES <= NST * STAGE_BYTES, "epilogue patch must fit the stage buffers");
    static_assert(TPP * CPR % 64 == 0 && TPP % 32 == 0, "whole wave-wide copies");
    unsigned char* my = lds + w * EPI_BYTES;
    const int tok_l = lane & 31, fsub = (lane >> 5) * 4;
    const int ncols = UP ? F : a.d;
    const int col0 = tc.n0 + wn * OC;
#pragma unroll
    for (int pass = 0; pass < WTM / TPP; ++pass) {
#pragma unroll
      for (int tl = 0; tl < TPP / 32; ++tl) {
        const int ti = pass * (TPP / 32) + tl;
#pragma unroll
        for (int fi = 0; fi < NFo; ++fi)
#pragma unroll
          for (int blk = 0; blk < 4; ++blk) {
            float v[4];
#pragma unroll
            for (int b = 0; b < 4; ++b) {
              if constexpr (UP) v[b] = swiglu(acc[fi][ti][blk * 4 + b], acc[fi + NF / 2][ti][blk * 4 + b]);
              else v[b] = acc[fi][ti][blk * 4 + b];
            }
            uint2 o;
            o.x = pack_bf16x2(v[0], v[1]);
            o.y = pack_bf16x2(v[2], v[3]);
            *reinterpret_cast<uint2*>(my + (tl * 32 + tok_l) * RS + (fi * 32 + blk * 8 + fsub) * 2) = o;
          }
      }
#pragma unroll
      for (int it = 0; it < TPP * CPR / 64; ++it) {
        const int idx = it * 64 + lane;
        const int row = idx / CPR, c = idx % CPR;
        const uint4 v = *reinterpret_cast<const uint4*>(my + row * RS + c * 16);
        const int trow = wm * WTM + pass * TPP + row;
        const int col = col0 + c * 8;
        if (trow < rows_left && col < ncols)
          *reinterpret_cast<uint4*>(a.C + (long long)(tc.row0 + tc.m0 + trow) * a.ldc + col) = v;
      }
    }
  }
  if (a.dbg) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    ts[5] = __builtin_amdgcn_s_memtime();
    if (threadIdx.x == 0) {
      for (int i = 0; i < 6; ++i) a.dbg[(size_t)blockIdx.x * 8 + i] = ts[i];
      a.dbg[(size_t)blockIdx.x * 8 + 6] = KT;
      a.dbg[(size_t)blockIdx.x * 8 + 7] = __builtin_amdgcn_s_getreg((4 << 0) | (8 << 6) | ((4 - 1) << 11));  // HW_ID bits: cu/se ids
    }
  }
}

template <int WGM, int WGN, bool UP, int PROBE = 0>
static hipError_t launch_tile_v2(const TileArgs& a, int P, int maxcols, hipStream_t s) {
  constexpr int BM = 256, BN = 256;
  constexpr int NCOLS_PER_TILE = UP ? BN / 2 : BN;
  constexpr size_t smem = (size_t)4 * (BM + BN) * 32 * 2;
  auto kern = ffn_tile_kernel_v2<WGM, WGN, UP, PROBE>;
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  const long long mt_bound = (long long)P / BM + a.Ne;
  const long long nt_max = (maxcols + NCOLS_PER_TILE - 1) / NCOLS_PER_TILE;
  long long grid = mt_bound * nt_max;
  grid = (grid + 7) / 8 * 8;
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(64 * WGM * WGN), smem, s, a);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------
template <int BM, int BN, int BK, int NST, int WGM, int WGN, bool UP, int PROBE = 0>
static hipError_t launch_tile(const TileArgs& a, int P, int maxcols, hipStream_t s) {
  constexpr int NCOLS_PER_TILE = UP ? BN / 2 : BN;
  constexpr size_t smem = (size_t)NST * (BM + BN) * BK * 2;
  static_assert(smem <= 160 * 1024, "LDS per workgroup");
  auto kern = ffn_tile_kernel<BM, BN, BK, NST, WGM, WGN, UP, PROBE>;
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

// tile configuration used by the up / down launch; changed through mohge_tune()
static int g_variant[2] = {0, 0};
static long long* g_dbg = nullptr;

void tune_tiled_dbg(void* p) { g_dbg = static_cast<long long*>(p); }

int tune_tiled(int knob, int value) {
  if (knob < 0 || knob > 1 || value < 0 || value > 31) return -1;
  g_variant[knob] = value;
  return 0;
}

template <bool UP>
static hipError_t launch_variant(int v, const TileArgs& a, int P, int maxcols, hipStream_t s) {
  switch (v) {
    case 0: return launch_tile<256, 256, 64, 2, 2, 2, UP>(a, P, maxcols, s);
    case 1: return launch_tile<256, 256, 32, 4, 2, 2, UP>(a, P, maxcols, s);
    case 2: return launch_tile<256, 256, 64, 2, 2, 4, UP>(a, P, maxcols, s);
    case 3: return launch_tile<256, 256, 32, 4, 2, 4, UP>(a, P, maxcols, s);
    case 4: return launch_tile<256, 256, 32, 3, 2, 2, UP>(a, P, maxcols, s);
    case 5: return launch_tile<256, 256, 64, 2, 4, 2, UP>(a, P, maxcols, s);
    case 6: return launch_tile<256, 128, 64, 3, 2, 2, UP>(a, P, maxcols, s);
    case 7: return launch_tile<128, 256, 64, 3, 2, 2, UP>(a, P, maxcols, s);
    case 8: return launch_tile<128, 128, 64, 2, 2, 2, UP>(a, P, maxcols, s);
    case 9: return launch_tile<256, 256, 64, 2, 2, 2, UP, PROBE_NO_LOADS>(a, P, maxcols, s);
    case 10: return launch_tile<256, 256, 64, 2, 2, 2, UP, PROBE_NO_MFMA>(a, P, maxcols, s);
    case 11: return launch_tile<256, 256, 32, 4, 2, 2, UP, PROBE_NO_MFMA>(a, P, maxcols, s);
    case 12: return launch_tile<256, 256, 64, 2, 2, 4, UP, PROBE_NO_LOADS>(a, P, maxcols, s);
    case 13: return launch_tile_v2<2, 2, UP>(a, P, maxcols, s);
    case 14: return launch_tile_v2<4, 2, UP>(a, P, maxcols, s);
    case 15: return launch_tile_v2<2, 4, UP>(a, P, maxcols, s);
    case 16: return launch_tile_v2<2, 2, UP, PROBE_NO_LOADS>(a, P, maxcols, s);
    case 17: return launch_tile_v2<4, 2, UP, PROBE_NO_LOADS>(a, P, maxcols, s);
    case 18: return launch_tile_v2<2, 2, UP, PROBE_NO_MFMA>(a, P, maxcols, s);
    default: return hipErrorInvalidValue;
  }
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
  up.dbg = g_dbg;
  TileArgs dn = up;
  dn.A = static_cast<const uint16_t*>(ws);
  dn.perm = nullptr;
  dn.C = static_cast<uint16_t*>(y_perm);
  dn.lda = L.Fmax; dn.ldc = L.d;
  for (int g = 0; g < kMaxGroups; ++g) dn.W[g] = static_cast<const uint16_t*>(W.w2[g]);

  hipError_t e = hipSuccess;
  if (stages & 1) e = launch_variant<true>(g_variant[0], up, L.P, L.Fmax, s);
  if (e != hipSuccess) return e;
  if (stages & 2) e = launch_variant<false>(g_variant[1], dn, L.P, L.d, s);
  return e;
}

}  // namespace mohge
