// Expert feed-forward networks for prefill-sized token counts on gfx950: a ragged
// grouped GEMM on the bf16 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulate).
//
// Two launches: "up" computes H = SiLU(X W_gate^T) * (X W_up^T) for every expert's
// rows, "down" computes Y = H W_down^T.  Both have the form C[rows of expert e] =
// A_rows . B_e^T with A and B contiguous along the reduction dimension.  What makes it
// ragged: the row count n_e comes from the router (device memory `offsets`), the width
// F_g differs from group to group (it is N of the up and K of the down projection).
//
// Schedule (device side, no host synchronisation).  A one-workgroup kernel turns
// `offsets` into a list of tiles: up to 256 token rows x 256 weight rows (up: 128 W_gate +
// the matching 128 W_up rows).  It picks the tile height (128, 192 or 256 rows) that needs
// the fewest rounds over the compute units, orders tiles so that tiles sharing operands are
// neighbours and every stretch of the list mixes all group widths, and cuts the list into 8 ranges of
// equal cost, one per XCD (each XCD has its own L2).  The GEMM kernel is persistent: one
// workgroup per compute unit, workgroup b serves XCD b%8 (the hardware hands workgroups
// to XCDs round-robin) and draws tiles of that XCD's range from an atomic counter.
//
// Tile kernel.  8 waves as 2 (token) x 4 (weight) with wave tiles of 128 x 64; a wave owns
// the 32-row token fragments {wm, wm+2, wm+4, wm+6}, so a tile with fewer rows keeps both
// wave rows equally busy and simply runs fewer MFMAs (the inner loop is instantiated for
// 1..4 active fragments).  Operands go global -> LDS with global_load_lds_dwordx4 (no
// staging registers) in 128-byte row segments (BK = 64): the texture path handles about one
// 128-byte line per two clocks however little of it is used, so 64-byte segments halve the
// feed rate (measured 24 vs 57 B/clk per CU).  16-byte chunks are XOR-swizzled inside the
// tile rows so that ds_read_b128 fragment reads are conflict free.  All 160 KB of LDS are
// used, asymmetrically: two stages for the token operand (its rows are shared by all column
// tiles of an expert and mostly hit in L2) and three for the weight operand (streamed from
// HBM), which therefore is requested two stages ahead.  The token gather is fused: a tile
// row's global address is taken through `perm`.
// The inner loop is ordered by hand (pinned with sched_barrier): operand fragments of the
// next 16-deep k-step are read from LDS into a second register set and the global -> LDS
// requests are issued between the MFMAs of the current one; one barrier per stage, placed
// after the third of its four k-steps so that the first fragments of the next stage are
// read under MFMAs as well.
// The MFMA takes the weight fragment as first operand: a lane then holds 4 consecutive
// output features of one token; the epilogue packs them to bf16 (hardware conversion),
// transposes through a wave-private LDS patch and stores whole row segments.
//
// Backward products (modes of the same kernel).  Their second operand, and for the weight
// gradients both operands, are stored with the reduction index as the row: dH = dY W_down
// reduces over the rows of W_down[e] ([d, F]), dX = [dA|dB] W13 over the rows of W13[e]
// ([2F, d]), dW_e = A_e^T B_e over the routed rows of expert e.  Such an operand is staged as
// 64 reduction rows x 256 features (512-byte row segments, again through global_load_lds,
// chunks swizzled by the row), and its MFMA fragments are read with ds_read_b64_tr_b16, which
// hands every lane four consecutive reduction indices of one feature.  No operand is
// transposed in memory.  The ragged reduction of the weight gradients needs no padding
// either: rows past the expert's last token are fetched from a row of zeros.  The
// transposing read moves fewer bytes per clock than the 128-bit read (measured about 0.75x),
// which costs these modes 15-20 % against a hypothetical pre-transposed operand; writing and
// re-reading the transposed copies cost more than that.
#include <type_traits>

#include "common.h"
#include "tiled.h"

namespace mohge {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kBM = 256, kBN = 256, kBK = 64;
constexpr int kStagesA = 2, kStagesB = 3;   // 32 KB parts: 2 token + 3 weight = all 160 KB of LDS
constexpr int kWGM = 2, kWGN = 4;
// LDS words for the hand-over between the tiles of a persistent workgroup: beyond the epilogue patches
// (one per wave, at most 32 rows x 144 bytes), inside a stage buffer that is dead between two tiles
constexpr int kHandoverOffset = (kWGM * kWGN * 32 * 144 / 4096 + 1) * 4096;
static_assert(kHandoverOffset == 40960 && kHandoverOffset + 8 <= 2 * kBM * kBK * 2, "inside the second token part");
constexpr int kTileCost = 18;          // cost model of the schedule: fixed part of a tile's stage, in 64-row units

// gate and up rows share a tile in the two up-projection modes
constexpr bool is_up(int mode) { return mode == kUp || mode == kUpSave; }
// operand stored reduction-index major (features contiguous): read through the transposing LDS read
constexpr bool tr_a(int mode) { return mode == kWgrad; }
constexpr bool tr_b(int mode) { return mode == kWgrad || mode == kDgradH || mode == kDgradX; }
// reduction over d, F_g output columns
constexpr bool red_d(int mode) { return is_up(mode) || mode == kDgradH; }

template <int MODE>
struct Shape {
  static constexpr int NCOLS_PER_TILE = is_up(MODE) ? kBN / 2 : kBN;
  // wave grid of the workgroup: 2 x 4 waves with 128 x 64 wave tiles (2 x 2 waves with
  // 128 x 128 wave tiles read a third fewer fragments per MFMA but measured slower in every
  // mode, the weight gradients with their transposing reads included; 4 x 4 waves with 64 x 64
  // wave tiles leave 128 registers a lane, spill, and measured 10 % slower)
  static constexpr int WGM = kWGM, WGN = kWGN;
  static constexpr int THREADS = 64 * WGM * WGN;
};

// ---------------------------------------------------------------------------------------
// schedule: one workgroup of 256 threads per projection; thread v <-> expert at visiting
// position v for the per-expert quantities, then threads stride over the tiles
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ long long wave_incl_scan64(long long v, int lane) {
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const long long up = __shfl_up(v, off, 64);
    if (lane >= off) v += up;
  }
  return v;
}

struct SchedShared {
  long long tp[kMaxExperts + 1];   // tiles before expert v
  long long cp[kMaxExperts + 1];   // cost before expert v
  int e[kMaxExperts], cnt[kMaxExperts], nt[kMaxExperts], kc[kMaxExperts], row0[kMaxExperts];
  int fp[kMaxExperts + 1];         // row blocks before expert v
  int sp[kMaxExperts + 1];         // tiles of the shortest reduction before expert v (see build_schedule)
  long long wsum[4][4];
  int rows;
  int xb[kXcds + 1];               // tile ranges per XCD (copy of the header's)
  int xs[kXcds + 1];               // tiles of the shortest reduction before each range
};

// Per-expert quantities of a mode: rows (`cnt`, starting at `row0`), output columns, and
// reduction length in 64-deep stages.
// Expert at visiting position v.  group_major: all experts of a group are neighbours, groups by
// decreasing width (tiles of one reduction length run together and the shortest come last);
// otherwise expert index major, group minor ("all-size sets": every stretch mixes all widths).
__device__ __forceinline__ void visit(const TileArgs& a, int v, int& e, int& g) {
  if (a.group_major) { g = a.order[v / a.N]; e = g * a.N + v % a.N; }
  else { g = a.order[v % a.Ng]; e = g * a.N + v / a.Ng; }
}

template <int MODE>
__device__ __forceinline__ void expert_dims(const TileArgs& a, int e, int g, int& row0, int& cnt,
                                            int& ncols, int& kc) {
  if constexpr (MODE == kWgrad) {
    row0 = 0;
    cnt = a.Mrows[g];
    ncols = a.Ncols[g];
    kc = (a.offsets[e + 1] - a.offsets[e] + 63) / 64;
    if (kc < 1) kc = 1;          // an expert without tokens still gets its zero gradient written
  } else {
    row0 = a.offsets[e];
    cnt = a.offsets[e + 1] - row0;
    ncols = red_d(MODE) ? a.F[g] : a.d;
    kc = (red_d(MODE) ? a.d : a.F[g]) / 64;
  }
}

// Tile height for a launch of MODE: the candidate with the lowest estimated time.  Called by all
// 256 threads; uses sh.wsum and sh.rows.
template <int MODE>
__device__ __forceinline__ int choose_tile_rows(const TileArgs& a, SchedShared& sh, bool fused = false) {
  constexpr int NCPT = Shape<MODE>::NCOLS_PER_TILE;
  const int v = threadIdx.x, lane = v & 63, w = v >> 6;
  int cnt = 0, nt = 0, kc = 0;
  if (v < a.Ne) {
    int e, g;
    visit(a, v, e, g);
    int ncols, row0;
    expert_dims<MODE>(a, e, g, row0, cnt, ncols, kc);
    nt = (ncols + NCPT - 1) / NCPT;
  }
  long long cand[3];
#pragma unroll
  for (int c = 0; c < 3; ++c) {
    const int h = 256 - 64 * c;
    long long x = (long long)((cnt + h - 1) / h) * nt * kc;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, 64);
    cand[c] = x;
  }
  __syncthreads();
  if (lane == 0) { sh.wsum[w][0] = cand[0]; sh.wsum[w][1] = cand[1]; sh.wsum[w][2] = cand[2]; }
  __syncthreads();
  if (v == 0) {
    long long kmax = 1;
    for (int g = 0; g < a.Ng; ++g)
      kmax = max(kmax, (long long)((red_d(MODE) ? a.d : a.F[g]) / 64));
    float best = 0.f;
    int best_rows = 256;
    for (int c = 0; c < 3; ++c) {
      const long long tot = sh.wsum[0][c] + sh.wsum[1][c] + sh.wsum[2][c] + sh.wsum[3][c];
      const long long rounds = (tot + (long long)a.ncu * kmax - 1) / ((long long)a.ncu * kmax);
      // measured: a stage of a tile costs about 1850 + 100 * (rows / 64) clocks (operand traffic
      // and LDS work do not shrink with the tile height), so rounds count more than height
      // (fused launch: the down tiles fill the last round of up tiles, so the up tiles are
      // costed by their total work rather than by whole rounds)
      const float units = fused ? (float)tot / (float)((long long)a.ncu * kmax) : (float)rounds;
      const float est = units * ((float)(4 - c) + 18.5f);
      if (c == 0 || est < best) { best = est; best_rows = 256 - 64 * c; }
    }
    sh.rows = a.force_rows ? a.force_rows : best_rows;
  }
  __syncthreads();
  const int h = sh.rows;
  __syncthreads();
  return h;
}

// Tile list of a launch of MODE with tile height h.  FUSED: the list belongs to a launch that
// runs up and down tiles together; down tiles then carry the number of up tiles they wait for.
// part / nparts: several workgroups may build one list together: each derives the (cheap) per-expert
// prefix sums itself and writes every nparts-th stretch of 256 records; part 0 writes the header.
template <int MODE>
__device__ __forceinline__ void build_schedule(const TileArgs& a, SchedShared& sh, int h, bool fused,
                                               int part = 0, int nparts = 1) {
  constexpr int NCPT = Shape<MODE>::NCOLS_PER_TILE;
  const int v = threadIdx.x, lane = v & 63, w = v >> 6;
  int e = 0, cnt = 0, nt = 0, kc = 0, row0 = 0;
  if (v < a.Ne) {
    int g;
    visit(a, v, e, g);
    int ncols;
    expert_dims<MODE>(a, e, g, row0, cnt, ncols, kc);
    nt = (ncols + NCPT - 1) / NCPT;
  }
  sh.e[v] = e; sh.cnt[v] = cnt; sh.nt[v] = nt; sh.kc[v] = kc; sh.row0[v] = row0;
  // exclusive prefix sums of tiles, cost and row blocks over the experts
  const long long my_t = (long long)((cnt + h - 1) / h) * nt;
  // cost of a tile = reduction stages x (kTileCost + its 64-row units): measured, a stage of a tile
  // costs about 1850 + 100 * units clocks, so a short tile is almost as expensive as a full one
  const long long my_c = ((long long)kTileCost * ((cnt + h - 1) / h) + (cnt + 63) / 64) * nt * kc;
  const long long my_f = MODE == kWgrad ? 0 : (cnt + h - 1) / h;
  // Second list of a fused launch (its tiles wait for tiles of the first): inside every XCD range
  // the tiles of the groups with the shortest reduction go last, everything else keeps its order.
  // The end of a range is then handed out in its smallest pieces (the launch ends when the slowest
  // workgroup does), and a tile only ever moves to a LATER position, so none meets its row block
  // earlier than before.
  int kmin = 1 << 30, kmax = 0;
  for (int g = 0; g < a.Ng; ++g) {
    const int k = (red_d(MODE) ? a.d : a.F[g]) / 64;
    kmin = min(kmin, k);
    kmax = max(kmax, k);
  }
  const bool short_last = fused && a.short_last && (MODE == kDown || MODE == kDgradX) && kmin < kmax;
  const long long my_s = (short_last && v < a.Ne && kc == kmin) ? my_t : 0;
  const long long it = wave_incl_scan64(my_t, lane), ic = wave_incl_scan64(my_c, lane);
  const long long jf = wave_incl_scan64(my_f, lane), is = wave_incl_scan64(my_s, lane);
  if (lane == 63) { sh.wsum[w][0] = it; sh.wsum[w][1] = ic; sh.wsum[w][2] = jf; sh.wsum[w][3] = is; }
  __syncthreads();
  long long bt = 0, bc = 0, bf = 0, bs = 0;
  for (int ww = 0; ww < w; ++ww) { bt += sh.wsum[ww][0]; bc += sh.wsum[ww][1]; bf += sh.wsum[ww][2]; bs += sh.wsum[ww][3]; }
  sh.tp[v] = bt + it - my_t;
  sh.cp[v] = bc + ic - my_c;
  sh.fp[v] = (int)(bf + jf - my_f);
  sh.sp[v] = (int)(bs + is - my_s);
  if (v == 255) { sh.tp[256] = bt + it; sh.cp[256] = bc + ic; sh.fp[256] = (int)(bf + jf); sh.sp[256] = (int)(bs + is); }
  __syncthreads();
  const int total = (int)sh.tp[256];
  const long long ctot = sh.cp[256];
  // expert (visiting position) of tile t: last v with tp[v] <= t
  auto expert_of = [&](int t) {
    int lo = 0, hi = 255;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (sh.tp[mid] <= t) lo = mid; else hi = mid - 1;
    }
    return lo;
  };
  // Inside an expert the tiles run in bands of `band` row blocks: band after band, inside a band
  // column tile major, row block minor.  The workgroups of an XCD draw consecutive tiles, so at any
  // moment they work on a few row blocks x a few column tiles of one expert and share both operand
  // panels through that XCD's L2 (an expert's whole column of row blocks per column tile would
  // share the weight panel only).
  const int RB = a.band > 0 ? a.band : 1;
  // XCD x starts at the first tile whose preceding cost is >= x/8 of the total.  The cost before
  // the tile at position rel of an expert follows from the band order in closed form, so the tile
  // is found by bisection once the expert is known.
  if (v <= kXcds) {
    int tile = total;
    if (v < kXcds) {
      const long long target = (ctot * v + kXcds - 1) / kXcds;
      int lo = 0, hi = 255;                  // last expert with cp[ve] <= target
      while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (sh.cp[mid] <= target) lo = mid; else hi = mid - 1;
      }
      const int ve = lo;
      const int c = sh.cnt[ve], kcv = sh.kc[ve], ntv = sh.nt[ve];
      const long long rem = target - sh.cp[ve];
      if (rem <= 0 || c == 0 || kcv == 0 || ntv == 0) {
        tile = (int)sh.tp[ve];               // (cp[ve] == target: the expert's first tile)
        if (rem > 0) tile = (int)sh.tp[ve + 1];
      } else {
        const int mt = (c + h - 1) / h, units = (c + 63) / 64, hu = h / 64;
        auto cost_before = [&](int rel) -> long long {
          if (rel >= mt * ntv) return ((long long)kTileCost * mt + units) * ntv * kcv;
          const int bnd = rel / (RB * ntv), rel2 = rel - bnd * RB * ntv;
          const int rb = min(RB, mt - bnd * RB);
          const int ni = rel2 / rb, mi2 = rel2 % rb;
          const int ub = min(units - bnd * RB * hu, RB * hu);       // 64-row units of this band
          return ((long long)kTileCost * rel + (long long)bnd * RB * hu * ntv + (long long)ni * ub +
                  min(mi2 * hu, ub)) * kcv;
        };
        int rl = 0, rh = mt * ntv;           // smallest rel with cost_before(rel) >= rem
        while (rl < rh) {
          const int mid = (rl + rh) >> 1;
          if (cost_before(mid) >= rem) rh = mid; else rl = mid + 1;
        }
        tile = (int)sh.tp[ve] + rl;
        if (tile > (int)sh.tp[ve + 1]) tile = (int)sh.tp[ve + 1];
      }
    }
    if (part == 0) a.hdr->xcd_begin[v] = tile;
    sh.xb[v] = tile;
  }
  __syncthreads();
  // tiles of the shortest reduction before tile t (t may be `total`)
  auto short_before = [&](int t) {
    if (t >= total) return sh.sp[256];
    const int ve = expert_of(t);
    return sh.sp[ve] + ((sh.sp[ve + 1] > sh.sp[ve]) ? t - (int)sh.tp[ve] : 0);
  };
  if (v <= kXcds) sh.xs[v] = short_last ? short_before(sh.xb[v]) : 0;
  __syncthreads();
  for (int t = v + 256 * part; t < total; t += 256 * nparts) {
    const int ve = expert_of(t);
    const int c = sh.cnt[ve], mt = (c + h - 1) / h, ntv = sh.nt[ve];
    const int rel = t - (int)sh.tp[ve];
    const int bnd = rel / (RB * ntv), rel2 = rel - bnd * RB * ntv;
    const int rb = min(RB, mt - bnd * RB);
    const int ni = rel2 / rb, mi = bnd * RB + rel2 % rb;
    TileRec r;
    r.e = sh.e[ve];
    r.row_start = sh.row0[ve] + mi * h;
    r.rows = min(h, c - mi * h);
    r.n0 = ni * NCPT;
    r.fam = sh.fp[ve] + mi;
    // a down tile of the fused forward waits for the up tiles of its row block: one per 128
    // hidden units of the expert's group (F holds the group's width in kDown)
    // (kDown: F holds the group's width, the up tiles are 128 hidden units wide; kDgradX: F holds
    // twice the width, the dH tiles are 256 hidden units wide)
    r.need = !fused ? 0
             : MODE == kDown ? (a.F[r.e / a.N] + kBN / 2 - 1) / (kBN / 2)
             : MODE == kDgradX ? (a.F[r.e / a.N] / 2 + kBN - 1) / kBN : 0;
    int pos = t;
    if (short_last) {
      int x = 0;                                   // the tile's XCD range
      while (x + 1 < kXcds && t >= sh.xb[x + 1]) ++x;
      const int sb = short_before(t) - sh.xs[x];   // short tiles of the range before t
      const int nlong = (sh.xb[x + 1] - sh.xb[x]) - (sh.xs[x + 1] - sh.xs[x]);
      const bool is_short = sh.sp[ve + 1] > sh.sp[ve];
      pos = is_short ? sh.xb[x] + nlong + sb : sh.xb[x] + (t - sh.xb[x]) - sb;
    }
    a.recs[pos] = r;
  }
  if (part != 0) return;                     // (workgroup-uniform: everything below is part 0's)
  // tail[x]: the tiles at the end of range x that belong to an expert whose tiles continue in
  // range x+1.  The fused launch computes them first (see fused_phase).
  if (v < kXcds) {
    const int cut = sh.xb[v + 1];
    int n = 0;
    if (cut > 0 && cut < total) {
      const int ve = expert_of(cut);                 // expert of the first tile of range x+1
      n = cut - (int)sh.tp[ve];                      // its tiles before the cut ...
      n = min(n, cut - sh.xb[v]);                    // ... that lie inside range x
      if (n < 0) n = 0;
    }
    a.hdr->tail[v] = n;
  }
  // the first ncu/8 tiles of a range are taken statically, one per workgroup (fused launch:
  // every tile is handed out by the counter, so that the tiles a waiting workgroup depends on
  // never sit with a workgroup that has not started yet)
  if (v < kXcds) a.hdr->counters[v] = fused ? 0 : a.ncu / kXcds;
  if (v == 0) { a.hdr->tile_rows = h; a.hdr->total = total; a.hdr->pad[0] = 0; }
  // fused forward: the row-block counters start at zero (the up list's workgroup clears them)
  if (fused && (is_up(MODE) || MODE == kDgradH))
    for (int i = v; i < sh.fp[256]; i += 256) a.fam_done[i] = 0;
}

template <int MODE>
__device__ __forceinline__ void build_schedule(const TileArgs& a, SchedShared& sh) {
  const int h = choose_tile_rows<MODE>(a, sh);
  build_schedule<MODE>(a, sh, h, false);
}

// workgroup 0 schedules the up projection, workgroup 1 the down projection (mask bits 0 / 1).
// mask 7: both lists for the fused launch, which needs one tile height for both (the up
// projection's choice, it is the larger part) so that row blocks coincide.
__global__ void __launch_bounds__(256) ffn_schedule_kernel(const TileArgs up, const TileArgs dn, int mask) {
  __shared__ SchedShared sh;
  if (mask == 7) {
    // four workgroups per list (blockIdx.x = list + 2 * part)
    const int h = choose_tile_rows<kUp>(up, sh, true);
    const int part = blockIdx.x >> 1, nparts = gridDim.x >> 1;
    if ((blockIdx.x & 1) == 0) build_schedule<kUp>(up, sh, h, true, part, nparts);
    else build_schedule<kDown>(dn, sh, h, true, part, nparts);
    return;
  }
  const int which = (mask == 3) ? (int)blockIdx.x : (mask == 2 ? 1 : 0);
  if (which == 0) build_schedule<kUp>(up, sh);
  else build_schedule<kDown>(dn, sh);
}

// the four schedules of the expert backward pass in one launch: workgroup i <-> launch i
// fused: the lists are for two fused launches (dH then dX, which waits for dH's row blocks and
// so shares its tile height; the two weight gradients one after the other)
__global__ void __launch_bounds__(256) bwd_schedule_kernel(const TileArgs dh, const TileArgs dx,
                                                           const TileArgs w2, const TileArgs w13, int fused,
                                                           const GatherArgs ga) {
  if (blockIdx.x >= 4) {
    // rows of x in sorted order, one wave per row; the first of these workgroups also clears the
    // row of zeros the weight-gradient tiles read past an expert's last row
    const int b = blockIdx.x - 4;
    if (b == 0 && threadIdx.x < 32) ga.zero_row[threadIdx.x] = make_uint4(0u, 0u, 0u, 0u);
    const int p = b * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (p >= ga.P || ga.perm == nullptr) return;
    const long long row = ga.perm[p] / ga.Ke;
    for (int c = lane; c < ga.chunks; c += 64) ga.xs[(long long)p * ga.chunks + c] = ga.x[row * ga.chunks + c];
    return;
  }
  __shared__ SchedShared sh;
  if (fused) {
    if (blockIdx.x < 2) {
      const int h = choose_tile_rows<kDgradH>(dh, sh, true);
      if (blockIdx.x == 0) build_schedule<kDgradH>(dh, sh, h, true);
      else build_schedule<kDgradX>(dx, sh, h, true);
    } else if (blockIdx.x == 2) {
      const int h = choose_tile_rows<kWgrad>(w2, sh);
      build_schedule<kWgrad>(w2, sh, h, true);
    } else {
      const int h = choose_tile_rows<kWgrad>(w13, sh);
      build_schedule<kWgrad>(w13, sh, h, true);
    }
    return;
  }
  if (blockIdx.x == 0) build_schedule<kDgradH>(dh, sh);
  else if (blockIdx.x == 1) build_schedule<kDgradX>(dx, sh);
  else if (blockIdx.x == 2) build_schedule<kWgrad>(w2, sh);
  else build_schedule<kWgrad>(w13, sh);
}

// schedule of one launch
template <int MODE>
__global__ void __launch_bounds__(256) tile_schedule_kernel(const TileArgs a) {
  __shared__ SchedShared sh;
  build_schedule<MODE>(a, sh);
}

// ---------------------------------------------------------------------------------------
// tile kernel
// ---------------------------------------------------------------------------------------
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

__device__ __forceinline__ void async_copy16(const void* gptr, void* lds_uniform_base) {
  __builtin_amdgcn_global_load_lds(
      (const __attribute__((address_space(1))) void*)gptr,
      (__attribute__((address_space(3))) void*)lds_uniform_base, 16, 0, 0);
}

#define MOHGE_PIN() __builtin_amdgcn_sched_barrier(0)

// 16-byte store performed at device scope (the sc1 cache policy of a vector store): written
// through the XCD's L2, so that once the store has completed (vmcnt) a workgroup on any XCD
// that has not cached the line before reads the new data.
__device__ __forceinline__ void store16_device_scope(void* p, const uint4 v) {
  typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 q = {v.x, v.y, v.z, v.w};
  asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(p), "v"(q) : "memory");
}

// SwiGLU backward for 8 packed bf16 values.  The training forward stored, per hidden unit,
//   p = b * SiLU'(a) = b * s * (1 + a*(1-s))   and   q = SiLU(a) = a * s,   s = sigmoid(a),
// so that  dA = dh * p,  dB = dh * q.
__device__ __forceinline__ void swiglu_bwd8(const uint4 dh, const uint4 pv, const uint4 qv, uint4& da,
                                            uint4& db) {
  const uint32_t hw[4] = {dh.x, dh.y, dh.z, dh.w};
  const uint32_t pw[4] = {pv.x, pv.y, pv.z, pv.w};
  const uint32_t qw[4] = {qv.x, qv.y, qv.z, qv.w};
  uint32_t oa[4], ob[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    float ra[2], rb[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const float g = __uint_as_float(h ? (hw[i] & 0xffff0000u) : (hw[i] << 16));
      ra[h] = g * __uint_as_float(h ? (pw[i] & 0xffff0000u) : (pw[i] << 16));
      rb[h] = g * __uint_as_float(h ? (qw[i] & 0xffff0000u) : (qw[i] << 16));
    }
    oa[i] = pack_bf16x2(ra[0], ra[1]);
    ob[i] = pack_bf16x2(rb[0], rb[1]);
  }
  da = make_uint4(oa[0], oa[1], oa[2], oa[3]);
  db = make_uint4(ob[0], ob[1], ob[2], ob[3]);
}

// One tile with NACT active 32-row token fragments per wave (tile rows <= 64*NACT).
// phase clocks for the optional counters of the benchmark library (a.cycles)
#define PROBE_T(i) do { if (a.cycles) ts[i] = __builtin_amdgcn_s_memtime(); } while (0)

template <int MODE, int NACT>
__device__ __forceinline__ void run_tile(const TileArgs& a, const TileRec rec, unsigned char* lds,
                                         int lane, int w, int* signal = nullptr) {
  constexpr bool UP = is_up(MODE);
  constexpr bool TRA = tr_a(MODE), TRB = tr_b(MODE);   // operand read by transposing LDS reads
  constexpr bool WG = MODE == kWgrad;
  constexpr bool DH = MODE == kDgradH;
  long long ts[6] = {0, 0, 0, 0, 0, 0};
  PROBE_T(0);
  constexpr int BM = kBM, BN = kBN, BK = kBK;
  constexpr int WGM = Shape<MODE>::WGM, WGN = Shape<MODE>::WGN, NWAVES = WGM * WGN, NT = 64 * NWAVES;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int MF = WTM / 32, NF = WTN / 32;
  constexpr int CH = BK / 8, ROWB = BK * 2, RPL = 64 / CH, SH = 1;   // 8 chunks, 128-byte rows
  constexpr int KK = BK / 16;                                        // MFMA k-steps per stage
  constexpr int B_LOADS = BN * CH / NT;
  // wave-wide load j of the token part fills tile rows [64j, 64j+64): only NACT of them matter
  // (token-major operands: a part is 64 tokens x 256 features, all of it is loaded)
  // (NACT active fragments per wave cover the tile rows [0, NACT * 32 * WGM))
  constexpr int A_LOADS = TRA ? BM * CH / NT : NACT * (32 * WGM / (NWAVES * RPL));
  static_assert((32 * WGM) % (NWAVES * RPL) == 0 && B_LOADS * NWAVES * RPL == BN, "whole wave-wide loads");
  constexpr int PART = BM * ROWB;                 // 32 KB: one token part or one weight part
  constexpr int NM = NACT * NF;     // MFMAs per k-step
  constexpr int NR = NACT + NF;     // fragment reads per k-step
  static_assert(NACT >= 1 && NACT <= MF, "active fragments");
  static_assert(!UP || NF % 2 == 0, "gate and up halves per wave");
  // LDS map: token parts A0, A1 (two stages), then weight parts B0, B1, B2 (three stages)
  auto a_part = [&](int stage) { return lds + (stage & 1) * PART; };
  auto b_part = [&](int slot) { return lds + (kStagesA + slot) * PART; };

  const int g = rec.e / a.N, e_i = rec.e % a.N, F = a.F[g];
  int K;
  int tok0 = 0, ntok = 0;       // kWgrad: the expert's routed rows [tok0, tok0 + ntok)
  if constexpr (WG) {
    tok0 = a.offsets[rec.e];
    ntok = a.offsets[rec.e + 1] - tok0;
    K = (ntok + BK - 1) / BK * BK;
    if (K < BK) K = BK;
  } else {
    K = red_d(MODE) ? a.d : F;
  }
  const int wm = w / WGN, wn = w % WGN;

  // ---- global source pointers of this thread's 16-byte chunks -------------------------
  // wave-wide load j fills tile rows (j*NWAVES + w)*RPL .. +RPL-1; lane l fills row l/CH,
  // physical chunk l%CH, which holds logical chunk (l%CH) ^ ((row >> SH) & (CH-1)).
  const int lrow = lane / CH, lpos = lane % CH;
  const uint16_t* src_a[TRA ? 1 : A_LOADS];
  const uint16_t* src_b[TRB ? 1 : B_LOADS];
  // Operands stored reduction-index major (rows = reduction index, features contiguous): a part
  // holds 64 reduction rows x 256 features, 512 bytes a row.  Wave-wide load j fills rows
  // 2*(j*NWAVES + w) and the next one; lane l fills physical chunk l%32 of row t = that + l/32,
  // which holds logical chunk (l%32) ^ (4*(t&3)): the four rows a transposing read touches at
  // once then sit in different banks.
  static_assert(!(TRA || TRB) || (NWAVES % 2 == 0 && B_LOADS == BM * CH / NT), "part layout");
  const int trow0 = 2 * w + (lane >> 5);          // row of load 0; load j: + 2*NWAVES*j
  const int tr_lc = (lane & 31) ^ (4 * (trow0 & 3));
  const uint16_t* zsrc = nullptr;
  unsigned tr_ldb = 0;                            // row pitch of the B operand in elements
  if constexpr (TRA) {
    int ma = rec.row_start + tr_lc * 8;
    // feature chunks past the matrix edge: any chunk inside the row (never stored)
    if (ma > a.Mrows[g] - 8) ma = a.Mrows[g] - 8;
    src_a[0] = a.A + (long long)(tok0 + trow0) * a.lda + ma;      // load 0 of stage 0
  }
  if constexpr (TRB) {
    int nb = rec.n0 + tr_lc * 8;
    if constexpr (WG) {
      if (nb > a.Ncols[g] - 8) nb = a.Ncols[g] - 8;
      zsrc = a.zero_row + (lane & 31) * 8;
      tr_ldb = a.ldb;
      src_b[0] = a.B2 + (long long)(tok0 + trow0) * a.ldb + nb;
    } else if constexpr (DH) {
      if (nb > F - 8) nb = F - 8;                 // W_down[e]: [d, F]
      tr_ldb = a.ldw[g];
      src_b[0] = a.W[g] + ((long long)e_i * a.d + trow0) * a.ldw[g] + nb;
    } else {
      if (nb > a.d - 8) nb = a.d - 8;             // W13[e]: [2F, d]; F holds 2 F_g here
      tr_ldb = a.ldw[g];
      src_b[0] = a.W[g] + ((long long)e_i * F + trow0) * a.ldw[g] + nb;
    }
  }
#pragma unroll
  for (int j = 0; j < (TRA ? 0 : A_LOADS); ++j) {
    const int row = (j * NWAVES + w) * RPL + lrow;
    const int rr = row < rec.rows ? row : rec.rows - 1;     // rows past the end: any valid row
    const int pos = rec.row_start + rr;
    long long src_row;
    if constexpr (UP) src_row = a.perm ? (long long)(a.perm[pos] / a.Ke) : (long long)pos;
    else src_row = pos;
    const int chunk = lpos ^ ((row >> SH) & (CH - 1));
    src_a[j] = a.A + src_row * a.lda + chunk * 8;
  }
#pragma unroll
  for (int j = 0; j < (TRB ? 0 : B_LOADS); ++j) {
    const int row = (j * NWAVES + w) * RPL + lrow;
    const int chunk = lpos ^ ((row >> SH) & (CH - 1));
    long long wrow;
    if constexpr (UP) {
      // tile rows [0, BN/2): W_gate rows n0.., rows [BN/2, BN): W_up rows n0..
      const int half = row >= BN / 2;
      int f = rec.n0 + (row - half * (BN / 2));
      if (f > F - 1) f = F - 1;
      wrow = (long long)e_i * 2 * F + (long long)half * F + f;
    } else {
      int n = rec.n0 + row;
      if (n > a.d - 1) n = a.d - 1;
      wrow = (long long)e_i * a.d + n;
    }
    src_b[j] = a.W[g] + wrow * a.ldw[g] + chunk * 8;
  }
  const int ld_off = w * 1024;      // + j * NWAVES * 1024: wave-uniform destination inside a part

  // ---- LDS offsets of the MFMA operand fragments ---------------------------------------
  // fragment row = base + lane%32, logical chunk = 2*kk + lane/32
  // Token-major parts: the transposing read works on groups of 16 lanes.  Lane 4*a + b of a
  // group passes the address of 4 features (8 bytes) of token k0 + a at feature m0 + 4*b and
  // gets back tokens k0..k0+3 of feature m0 + (its index in the group).  Group q of the wave
  // covers features 16*(q&1).. of the fragment and tokens 8*(q>>1).. of the k-step, so two
  // reads (k0, k0 + 4) give a lane its 8 consecutive reduction indices of one fragment row.
  const int frow = lane & 31, fh = lane >> 5;
  const int tq = lane >> 4, ta = (lane & 15) >> 2, tb = lane & 3;
  int foff[KK], foff_t[KK];       // plain parts / reduction-major parts (only one is live
                                  // unless the two operands differ)
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    foff_t[kk] = (16 * kk + 8 * (tq >> 1) + ta) * 512 + (2 * (tq & 1) + (tb >> 1)) * 16 + (tb & 1) * 8;
    foff[kk] = frow * ROWB + (((2 * kk + fh) ^ ((frow >> SH) & (CH - 1))) << 4);
  }
  // first feature of a fragment -> its 16-byte chunk, swizzled like the loads wrote it
  auto tr_base = [&](int feat) { return (((feat >> 3) ^ (4 * ta)) << 4); };
  int fbase[NR];     // token fragments first (interleaved over the wave rows), then weights
#pragma unroll
  for (int ti = 0; ti < NACT; ++ti)
    fbase[ti] = TRA ? tr_base((ti * WGM + wm) * 32) : ((ti * WGM + wm) * 32) * ROWB;
#pragma unroll
  for (int fi = 0; fi < NF; ++fi) {
    int row;
    if constexpr (UP) {
      constexpr int NFh = NF / 2;
      row = (fi < NFh) ? wn * (WTN / 2) + fi * 32 : BN / 2 + wn * (WTN / 2) + (fi - NFh) * 32;
    } else {
      row = wn * WTN + fi * 32;
    }
    fbase[NACT + fi] = TRB ? tr_base(row) : row * ROWB;
  }

  f32x16 acc[NF][NACT];
#pragma unroll
  for (int fi = 0; fi < NF; ++fi)
#pragma unroll
    for (int ti = 0; ti < NACT; ++ti)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[fi][ti][r] = 0.f;

  const int KT = K / BK;
  // fragment r of k-step kk of the stage whose parts are pa (tokens) / pb (weights)
  auto read_frag = [&](const unsigned char* pa, const unsigned char* pb, int kk, int r) {
    const bool tr = r < NACT ? TRA : TRB;
    const unsigned char* p = (r < NACT ? pa : pb) + fbase[r] + (tr ? foff_t[kk] : foff[kk]);
    if (tr) {
      typedef short s16x4 __attribute__((ext_vector_type(4)));
      typedef short s16x8 __attribute__((ext_vector_type(8)));
      typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * 512));
      const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      return __builtin_bit_cast(bf16x8, v);
    } else {
      return *reinterpret_cast<const bf16x8*>(p);
    }
  };
  // reduction-major operands: load j of a stage starts 2*NWAVES*j rows further down; in
  // kWgrad the rows are routed tokens, and those at or past the expert's count read the zero
  // row instead
  auto tr_src = [&](const uint16_t* base, unsigned ld, int stage, int j) {
    const int t = stage * BK + 2 * NWAVES * j;      // row of this load, less trow0
    // wave-uniform 32 x 32 -> 64 bit product: stays in scalar registers
    const uint16_t* p = base + (unsigned long long)(unsigned)t * ld;
    if constexpr (WG) return t + trow0 < ntok ? p : zsrc;
    else return p;
  };
  auto issue_a = [&](int stage, int j) {
    const uint16_t* src;
    if constexpr (TRA) src = tr_src(src_a[0], a.lda, stage, j);
    else src = src_a[j] + stage * BK;
    async_copy16(src, a_part(stage) + j * NWAVES * 1024 + ld_off);
  };
  auto issue_b = [&](int stage, int slot, int j) {
    const uint16_t* src;
    if constexpr (TRB) src = tr_src(src_b[0], tr_ldb, stage, j);
    else src = src_b[j] + stage * BK;
    async_copy16(src, b_part(slot) + j * NWAVES * 1024 + ld_off);
  };

  // prologue: request B(0), A(0), B(1), A(1), B(2) (those that exist), wait for the first
  // two, read the first fragments
  PROBE_T(1);
  __syncthreads();                  // the previous tile's epilogue has left the LDS
#pragma unroll
  for (int j = 0; j < B_LOADS; ++j) issue_b(0, 0, j);
#pragma unroll
  for (int j = 0; j < A_LOADS; ++j) issue_a(0, j);
  if (KT > 1) {
#pragma unroll
    for (int j = 0; j < B_LOADS; ++j) issue_b(1, 1, j);
#pragma unroll
    for (int j = 0; j < A_LOADS; ++j) issue_a(1, j);
    if (KT > 2) {
#pragma unroll
      for (int j = 0; j < B_LOADS; ++j) issue_b(2, 2, j);
      wait_vmcnt<2 * B_LOADS + A_LOADS>();
    } else {
      wait_vmcnt<B_LOADS + A_LOADS>();
    }
  } else {
    wait_vmcnt<0>();
  }
  __builtin_amdgcn_s_barrier();
  MOHGE_PIN();
  // Fused launches: the counter of the row block that this workgroup's PREVIOUS tile completed.
  // Vector memory operations of a wave complete in issue order, so a wave whose first-stage loads
  // have landed has seen all its earlier stores complete, and the barrier above makes that true
  // of every wave: the previous tile's rows are in memory.  (Waiting for those stores at the end of
  // the previous tile instead cost a memory round trip with nothing to overlap it.)
  if (signal != nullptr && threadIdx.x == 0)
    __hip_atomic_fetch_add(signal, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  PROBE_T(2);
  bf16x8 f0[NR], f1[NR];
#pragma unroll
  for (int r = 0; r < NR; ++r) f0[r] = read_frag(a_part(0), b_part(0), 0, r);

  // One k-step: NM MFMAs on `use`; after MFMA i the extra instructions of this k-step are
  // placed round-robin: first the NR fragment reads of the next k-step into `nxt`, then the
  // global -> LDS requests handed in as `nld` callables.
  auto kstep = [&](bf16x8 (&use)[NR], bf16x8 (&nxt)[NR], auto READ_NEXT, const unsigned char* pa,
                   const unsigned char* pb, int kk_next, auto NLD, auto&& issue_one) {
    constexpr bool RN = decltype(READ_NEXT)::value;
    constexpr int NL = decltype(NLD)::value;
    constexpr int NX = (RN ? NR : 0) + NL;
    constexpr int PER = (NX + NM - 1) / NM;
#pragma unroll
    for (int i = 0; i < NM; ++i) {
      const int fi = i / NACT, ti = i % NACT;
      acc[fi][ti] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(use[NACT + fi], use[ti], acc[fi][ti], 0, 0, 0);
      MOHGE_PIN();
#pragma unroll
      for (int q = 0; q < PER; ++q) {
        const int x = i * PER + q;
        if (RN && x < NR) {
          // in order of first use by the next k-step's MFMAs: weight fragment 0, the token
          // fragments, then the other weight fragments
          const int fr = x == 0 ? NACT : (x <= NACT ? x - 1 : x);
          nxt[fr] = read_frag(pa, pb, kk_next, fr);
          MOHGE_PIN();
        } else if (x < NX) {
          issue_one(x - (RN ? NR : 0));
          MOHGE_PIN();
        }
      }
    }
  };

  // Stage kt: token part kt&1, weight slot `slot` = kt%3.  The one barrier of the stage comes
  // after its third k-step, when every wave holds the fragments of the fourth in registers:
  // from then on nobody reads the stage's LDS parts again, so the token part of stage kt+2 and
  // the weight part of stage kt+3 are requested into them during the fourth k-step (tokens
  // first, so that "all but the newest B_LOADS requests have landed" certifies stage kt+1 at
  // the next barrier), and the first fragments of stage kt+1 are read under the fourth
  // k-step's MFMAs instead of after a barrier.
  int slot = 0;
  auto stage = [&](int kt, auto LA, auto LB, auto LAST) {
    // la: stage kt+2 exists (so A(kt+2) is requested and B(kt+2) may be in flight at the
    // barrier); lb: stage kt+3 exists; last: no stage kt+1
    constexpr bool la = decltype(LA)::value, lb = decltype(LB)::value, last = decltype(LAST)::value;
    const unsigned char* pa = a_part(kt);
    const unsigned char* pb = b_part(slot);
    const int slot1 = slot == kStagesB - 1 ? 0 : slot + 1;     // stage kt+1
    using c0 = std::integral_constant<int, 0>;
    using cAB = std::integral_constant<int, (la ? A_LOADS : 0) + (lb ? B_LOADS : 0)>;
    kstep(f0, f1, std::true_type{}, pa, pb, 1, c0{}, [&](int) {});
    kstep(f1, f0, std::true_type{}, pa, pb, 2, c0{}, [&](int) {});
    kstep(f0, f1, std::true_type{}, pa, pb, 3, c0{}, [&](int) {});
    if constexpr (!last) {
      // my reads of this stage are complete; my requests for stage kt+1 have landed
      if constexpr (la) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(B_LOADS) : "memory");
      else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
      __builtin_amdgcn_s_barrier();
      MOHGE_PIN();
      kstep(f1, f0, std::true_type{}, a_part(kt + 1), b_part(slot1), 0, cAB{}, [&](int j) {
        if (la && j < A_LOADS) issue_a(kt + 2, j);
        else issue_b(kt + 3, slot, j - (la ? A_LOADS : 0));
      });
    } else {
      kstep(f1, f0, std::false_type{}, pa, pb, 0, c0{}, [&](int) {});
    }
    slot = slot1;
  };

  {
    using T = std::true_type;
    using Fa = std::false_type;
    int kt = 0;
    for (; kt + 3 < KT; ++kt) stage(kt, T{}, T{}, Fa{});
    if (kt + 2 < KT) { stage(kt, T{}, Fa{}, Fa{}); ++kt; }
    if (kt + 1 < KT) { stage(kt, Fa{}, Fa{}, Fa{}); ++kt; }
    stage(kt, Fa{}, Fa{}, T{});
  }
  PROBE_T(3);

  // ---- epilogue: accumulators -> bf16 -> a wave-private LDS patch -> 16-byte stores ------
  // A lane holds, per 32x32 block, token lane%32 and weight rows 8*(r/4) + 4*(lane/32) +
  // r%4: runs of 4 consecutive output features.  Every wave transposes its part through
  // LDS (row stride padded by 16 bytes against bank conflicts) and stores row segments.
  __syncthreads();                     // all waves are done reading the stages
  {
    constexpr int OC = UP ? WTN / 2 : WTN;           // output features of this wave
    constexpr int RS = OC * 2 + 16;                  // LDS row stride in bytes
    constexpr int EPI_BYTES = 32 * RS;               // one 32-token fragment at a time
    constexpr int CPR = OC * 2 / 16;                 // 16-byte chunks per row
    constexpr int NFo = UP ? NF / 2 : NF;
    static_assert(NWAVES * EPI_BYTES <= (kStagesA + kStagesB) * PART, "epilogue patch must fit the stage buffers");
    static_assert(32 * CPR % 64 == 0, "whole wave-wide copies");
    unsigned char* my = lds + w * EPI_BYTES;
    const int tok_l = lane & 31, fsub = (lane >> 5) * 4;
    const int ncols = red_d(MODE) ? F : (WG ? a.Ncols[g] : a.d);
    const int col0 = rec.n0 + wn * OC;
    // kUpSave makes three passes over the patch: h, then the backward factors p and q
    constexpr int NPASS = MODE == kUpSave ? 3 : 1;
    constexpr int NIT = 32 * CPR / 64;     // row-segment copies per lane and fragment
    // kDgradH: the stored factor chunks a lane will meet in the copy loop are requested before
    // the transposition through LDS (rows / columns past the tile edge: any valid chunk)
    auto load_pre = [&](int ti, uint4 (&pa)[NIT], uint4 (&pb)[NIT]) {
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        const int idx = it * 64 + lane;
        int trow = (ti * WGM + wm) * 32 + idx / CPR, col = col0 + (idx % CPR) * 8;
        if (trow > rec.rows - 1) trow = rec.rows - 1;
        if (col > ncols - 8) col = ncols - 8;
        const long long at = (long long)(rec.row_start + trow) * a.ldpre + col;
        pa[it] = *reinterpret_cast<const uint4*>(a.pre + at);
        pb[it] = *reinterpret_cast<const uint4*>(a.pre + at + F);
      }
    };
#pragma unroll
    for (int ti = 0; ti < NACT; ++ti) {
      uint4 pre_a[DH ? NIT : 1], pre_b[DH ? NIT : 1];
      if constexpr (DH) load_pre(ti, pre_a, pre_b);
      // kUpSave: the two factors the backward pass multiplies dh with, computed along with h
      // (one sigmoid per element) and kept packed until their pass
      uint2 keep_p[MODE == kUpSave ? NFo * 4 : 1], keep_q[MODE == kUpSave ? NFo * 4 : 1];
#pragma unroll
      for (int pass = 0; pass < NPASS; ++pass) {
#pragma unroll
        for (int fi = 0; fi < NFo; ++fi)
#pragma unroll
          for (int blk = 0; blk < 4; ++blk) {
            uint2 o;
            if (MODE == kUpSave && pass > 0) {
              o = pass == 1 ? keep_p[fi * 4 + blk] : keep_q[fi * 4 + blk];
            } else {
              float v[4], vp[4], vq[4];
#pragma unroll
              for (int b = 0; b < 4; ++b) {
                if constexpr (MODE == kUpSave) {
                  const float ga = acc[fi][ti][blk * 4 + b], ub = acc[fi + NF / 2][ti][blk * 4 + b];
                  const float sg = __builtin_amdgcn_rcpf(1.f + __expf(-ga));
                  vq[b] = ga * sg;                                   // SiLU(a)
                  v[b] = ga * ub * sg;                               // h, rounded as in kUp
                  vp[b] = ub * sg * (1.f + ga * (1.f - sg));         // b * SiLU'(a)
                } else if constexpr (UP) {
                  v[b] = swiglu(acc[fi][ti][blk * 4 + b], acc[fi + NF / 2][ti][blk * 4 + b]);
                } else {
                  v[b] = acc[fi][ti][blk * 4 + b];
                }
              }
              o.x = pack_bf16x2(v[0], v[1]);
              o.y = pack_bf16x2(v[2], v[3]);
              if constexpr (MODE == kUpSave) {
                keep_p[fi * 4 + blk] = make_uint2(pack_bf16x2(vp[0], vp[1]), pack_bf16x2(vp[2], vp[3]));
                keep_q[fi * 4 + blk] = make_uint2(pack_bf16x2(vq[0], vq[1]), pack_bf16x2(vq[2], vq[3]));
              }
            }
            *reinterpret_cast<uint2*>(my + tok_l * RS + (fi * 32 + blk * 8 + fsub) * 2) = o;
          }
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
          const int idx = it * 64 + lane;
          const int row = idx / CPR, c = idx % CPR;
          const uint4 v = *reinterpret_cast<const uint4*>(my + row * RS + c * 16);
          const int trow = (ti * WGM + wm) * 32 + row;
          const int col = col0 + c * 8;
          if (trow < rec.rows && col < ncols) {
            if constexpr (WG) {
              uint16_t* dst = a.Wout[g] + ((long long)e_i * a.Mrows[g] + rec.row_start + trow) * ncols + col;
              *reinterpret_cast<uint4*>(dst) = v;
            } else if constexpr (DH) {
              // v holds dh; the stored factors turn it into the gradients of the pre-activations
              const long long at = (long long)(rec.row_start + trow) * a.ldpre + col;
              uint4 da, db;
              swiglu_bwd8(v, pre_a[it], pre_b[it], da, db);
              if (a.coherent_out) {
                store16_device_scope(a.C2 + at, da);
                store16_device_scope(a.C2 + at + F, db);
              } else {
                *reinterpret_cast<uint4*>(a.C2 + at) = da;
                *reinterpret_cast<uint4*>(a.C2 + at + F) = db;
              }
            } else if (pass == 0) {
              uint16_t* dst = a.C + (long long)(rec.row_start + trow) * a.ldc + col;
              if (UP && a.coherent_out) store16_device_scope(dst, v);
              else *reinterpret_cast<uint4*>(dst) = v;
            } else {
              const long long at = (long long)(rec.row_start + trow) * a.ldpre + (pass == 2 ? F : 0) + col;
              *reinterpret_cast<uint4*>(a.pre + at) = v;
            }
          }
        }
      }
    }
  }
  PROBE_T(4);
  if (a.cycles && threadIdx.x == 0) {
    // setup, wait for the first stages, main loop, epilogue; tiles; stages
    long long* d = a.cycles + (size_t)blockIdx.x * 8;
    for (int i = 0; i < 4; ++i) d[i] += ts[i + 1] - ts[i];
    d[4] += 1;
    d[5] += KT;
  }
}

// The instantiation of run_tile for the tile's row count: a wave's k-th fragment serves the tile
// rows [32 * WGM * k, 32 * WGM * (k + 1)) together with the other wave rows.
template <int MODE>
__device__ __forceinline__ void run_tile_rows(const TileArgs& a, const TileRec& rec, unsigned char* lds, int lane,
                                              int w, int* signal) {
  constexpr int UNIT = 32 * Shape<MODE>::WGM, MF = kBM / UNIT;
  static_assert(MF == 2 || MF == 4, "two or four token fragments per wave");
  const int nact = (rec.rows + UNIT - 1) / UNIT;
  if constexpr (MF == 4) {
    if (nact == 4) { run_tile<MODE, 4>(a, rec, lds, lane, w, signal); return; }
    if (nact == 3) { run_tile<MODE, 3>(a, rec, lds, lane, w, signal); return; }
  }
  if (nact >= 2) run_tile<MODE, 2>(a, rec, lds, lane, w, signal);
  else run_tile<MODE, 1>(a, rec, lds, lane, w, signal);
}

// Persistent tile kernel: workgroup b serves XCD b % 8.  Its first tile is fixed (range start
// + b / 8); further tiles are handed out by an atomic counter per range, so a workgroup that
// drew cheap tiles simply takes more of them.  The counter is read one tile ahead (the
// atomic's latency hides behind the tile) and the result is passed to the other waves
// through one LDS word between the tiles.  Which workgroup computes a tile has no influence
// on the tile's result, so the output stays bit-identical from run to run.
template <int MODE>
__global__ void __launch_bounds__(Shape<MODE>::THREADS) ffn_tile_kernel(const TileArgs a) {
  extern __shared__ __align__(1024) unsigned char lds[];
  // LDS word for the hand-over: beyond the epilogue patches, inside a stage buffer that is
  // dead between a tile's last barrier and the first barrier of the next tile
  constexpr int kBcastOffset = kHandoverOffset;
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int xcd = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
  int tbeg = a.hdr->xcd_begin[xcd], tend = a.hdr->xcd_begin[xcd + 1];
  const int total = a.hdr->total;
  if (tbeg < 0) tbeg = 0;
  if (tend > total) tend = total;
  int t = tbeg + slot;
  while (t < tend) {
    int t_next = 0;
    if (threadIdx.x == 0) t_next = tbeg + atomicAdd(&a.hdr->counters[xcd], 1);
    TileRec rec = a.recs[t];
    rec.e = __builtin_amdgcn_readfirstlane(rec.e);
    rec.row_start = __builtin_amdgcn_readfirstlane(rec.row_start);
    rec.rows = __builtin_amdgcn_readfirstlane(rec.rows);
    rec.n0 = __builtin_amdgcn_readfirstlane(rec.n0);
    // a record that does not describe rows of this call would mean a corrupted schedule:
    // skip it rather than touch memory through it
    bool ok = !(rec.e < 0 || rec.e >= a.Ne || rec.rows < 1 || rec.rows > kBM ||
                rec.row_start < 0 || rec.n0 < 0);
    if (ok) {
      if constexpr (MODE == kWgrad) {
        ok = rec.row_start + rec.rows <= a.Mrows[rec.e / a.N] && rec.n0 < a.Ncols[rec.e / a.N] &&
             a.zero_row != nullptr && a.offsets[rec.e] >= 0 && a.offsets[rec.e + 1] <= a.P &&
             a.offsets[rec.e] <= a.offsets[rec.e + 1];
      } else {
        ok = rec.row_start + rec.rows <= a.P;
      }
    }
    if (ok) {
      run_tile_rows<MODE>(a, rec, lds, lane, w, nullptr);
    }
    __syncthreads();       // every wave is past its epilogue (and past reading the old word)
    if (threadIdx.x == 0) *reinterpret_cast<volatile int*>(lds + kBcastOffset) = t_next;
    __syncthreads();
    t = __builtin_amdgcn_readfirstlane(*reinterpret_cast<volatile int*>(lds + kBcastOffset));
  }
}

// Fused forward: the up tiles and the down tiles of a layer call in one persistent launch.
// Workgroup b serves XCD b % 8: first the up tiles of that XCD's range of the up list, then the
// down tiles of its range of the down list, each range with its own hand-out counter as in
// ffn_tile_kernel.  A down tile reads the H rows of one (expert, row block), which the up tiles
// of that row block write: every finished up tile adds one to the row block's counter
// (fam_done), a down tile waits until the counter has reached the number of up tiles of the
// block.  What makes the hand-over sound on any XCD:
//  * H is stored at device scope (coherent_out), and every wave waits for its stores (vmcnt)
//    before the workgroup barrier that precedes the counter increment;
//  * the consumer reads the counter at device scope and reads H only after that; no cache on
//    its path can hold an older copy of these lines, since nothing reads H rows of a row block
//    in this launch before the block's counter is complete, and launch boundaries invalidate
//    the caches.
// Waiting cannot deadlock: tiles are handed out in list order, all up tiles of an XCD come
// before its down tiles, and an up tile never waits for anything; a down tile whose row block
// belongs to another XCD's range waits for tiles that were handed out there before any of
// that XCD's down tiles.  The wait is bounded all the same (kSpinLimit polls, about a second);
// if it ever expires the tile is computed regardless and a flag is left in the header of the
// waiting list, which mohge_fused_status reports.  A negative limit (test hook, mohge_tune knob
// 3) makes every dependent tile give up without looking.
constexpr int kSpinLimit = 1 << 22;

// Output region of a tile of a token mode (rows x 256 columns of C) filled with bf16 NaNs.
__device__ __forceinline__ void poison_tile(const TileArgs& a, const TileRec& rec) {
  if (a.C == nullptr) return;
  const int ncols = min(kBN, a.ldc - rec.n0);
  for (int i = threadIdx.x; i < rec.rows * (kBN / 2); i += blockDim.x) {
    const int r = i / (kBN / 2), c = (i % (kBN / 2)) * 2;
    if (c < ncols)
      *reinterpret_cast<uint32_t*>(a.C + (long long)(rec.row_start + r) * a.ldc + rec.n0 + c) = 0x7FC07FC0u;
  }
}

// One phase of a fused launch: the tiles of one list in MODE.  ROLE 1: producer (every finished
// tile adds one to its row block's counter; the range's straddling tail goes first), ROLE 2:
// consumer (a tile waits until its row block's counter has reached rec.need), ROLE 0: neither.
template <int MODE, int ROLE>
__device__ __forceinline__ void fused_phase(const TileArgs& a, unsigned char* lds, int lane, int w) {
  constexpr int PHASE = ROLE == 1 ? 0 : 1;
  constexpr int kBcastOffset = kHandoverOffset;
  const int home = blockIdx.x % kXcds;
  const int total = a.hdr->total;
  // The counter of a range hands out positions 0, 1, 2, ...  Up phase: the positions map to the
  // range's tail first (tiles of an expert that continues in the next XCD's range: down tiles of
  // both ranges wait for them), then to the rest in list order.  Down phase: list order, the order
  // in which the up tiles they depend on were handed out.
  // A workgroup serves its own XCD's range until the counter runs past its end and then (steal)
  // whichever other range still has tiles, so the launch ends when all tiles are done rather than
  // when the slowest range is.  (The number of rounds is bounded for form's sake: every round but
  // the last exhausts a range, and counters only grow.)  A stolen tile is an ordinary draw from that range's counter, so the
  // argument about waiting below holds for it as well.
  int* pending = nullptr;      // ROLE 1: counter of the row block of the tile just finished, not yet added to
  int cur = home;
  for (int round = 0; round <= 4 * kXcds; ++round) {
    if (round > 0) {
      // Own range exhausted: look at the counters of all other ranges at once (one memory round
      // trip: looking at them one after the other cost a round trip each at the moment when the
      // workgroup has nothing to do, 15-30 us where the whole launch takes 230) and go to the first
      // one, in ring order, that still has tiles.  (A counter is looked at before it is drawn
      // from, so that an exhausted one is left alone.)
      // (only where a compute unit sees several tiles of this list: with fewer, what a stolen tile
      // saves at the end does not pay for fetching its operands into another XCD's L2)
      if (!(a.steal & (PHASE == 0 ? 1 : 2)) || total < 4 * a.ncu) break;
      __syncthreads();
      if (threadIdx.x == 0) {
        int c[kXcds];
#pragma unroll
        for (int x = 0; x < kXcds; ++x)
          c[x] = __hip_atomic_load(&a.hdr->counters[x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        int pick = -1;
#pragma unroll
        for (int k = kXcds - 1; k >= 1; --k) {
          const int x = (home + k) % kXcds;
          int b = a.hdr->xcd_begin[x], e = a.hdr->xcd_begin[x + 1];
          if (b < 0) b = 0;
          if (e > total) e = total;
          int cx = 0;
#pragma unroll
          for (int y = 0; y < kXcds; ++y) cx = y == x ? c[y] : cx;
          if (cx < e - b) pick = x;
        }
        *reinterpret_cast<volatile int*>(lds + kBcastOffset) = pick;
      }
      __syncthreads();
      cur = __builtin_amdgcn_readfirstlane(*reinterpret_cast<volatile int*>(lds + kBcastOffset));
      if (cur < 0 || cur >= kXcds) break;
    }
    int tbeg = a.hdr->xcd_begin[cur], tend = a.hdr->xcd_begin[cur + 1];
    if (tbeg < 0) tbeg = 0;
    if (tend > total) tend = total;
    const int n = tend - tbeg;
    int ntail = PHASE == 0 ? a.hdr->tail[cur] : 0;
    ntail = ntail < 0 ? 0 : (ntail > n ? n : ntail);
    __syncthreads();         // everybody has read the last hand-over word
    if (threadIdx.x == 0) *reinterpret_cast<volatile int*>(lds + kBcastOffset) = atomicAdd(&a.hdr->counters[cur], 1);
    __syncthreads();
    int pos = __builtin_amdgcn_readfirstlane(*reinterpret_cast<volatile int*>(lds + kBcastOffset));
    while (pos >= 0 && pos < n) {
      const int t = pos < ntail ? tend - ntail + pos : tbeg + (pos - ntail);
      int t_next = 0;
      if (threadIdx.x == 0) t_next = atomicAdd(&a.hdr->counters[cur], 1);
      TileRec rec = a.recs[t];
      rec.e = __builtin_amdgcn_readfirstlane(rec.e);
      rec.row_start = __builtin_amdgcn_readfirstlane(rec.row_start);
      rec.rows = __builtin_amdgcn_readfirstlane(rec.rows);
      rec.n0 = __builtin_amdgcn_readfirstlane(rec.n0);
      rec.fam = __builtin_amdgcn_readfirstlane(rec.fam);
      rec.need = __builtin_amdgcn_readfirstlane(rec.need);
      bool ok = !(rec.e < 0 || rec.e >= a.Ne || rec.rows < 1 || rec.rows > kBM || rec.row_start < 0 ||
                  rec.n0 < 0 || rec.fam < 0);
      if (ok) {
        if constexpr (MODE == kWgrad) {
          ok = rec.row_start + rec.rows <= a.Mrows[rec.e / a.N] && rec.n0 < a.Ncols[rec.e / a.N] &&
               a.zero_row != nullptr && a.offsets[rec.e] >= 0 && a.offsets[rec.e + 1] <= a.P &&
               a.offsets[rec.e] <= a.offsets[rec.e + 1];
        } else {
          ok = rec.row_start + rec.rows <= a.P && rec.fam <= a.P;
        }
      }
      if (ok) {
        bool gave_up = false;
        if constexpr (ROLE == 2) {
          if (threadIdx.x == 0) {
            const long long w0 = a.cycles ? __builtin_amdgcn_s_memtime() : 0;
            int polls = 0, bad = 0;
            if (a.spin_limit < 0) bad = 1;
            else
              while (__hip_atomic_load(&a.fam_done[rec.fam], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < rec.need) {
                if (++polls > a.spin_limit) { bad = 1; break; }
                __builtin_amdgcn_s_sleep(8);
              }
            if (bad) a.hdr->pad[0] = 1;
            *reinterpret_cast<volatile int*>(lds + kBcastOffset + 4) = bad;
            if (a.cycles) {
              a.cycles[(size_t)blockIdx.x * 8 + 6] += __builtin_amdgcn_s_memtime() - w0;
              a.cycles[(size_t)blockIdx.x * 8 + 7] += polls > 0;
            }
          }
          __syncthreads();
          gave_up = __builtin_amdgcn_readfirstlane(*reinterpret_cast<volatile int*>(lds + kBcastOffset + 4)) != 0;
        }
        if (gave_up) {
          // the rows this tile depends on never became complete: its output is written as NaN, so
          // that nothing downstream can take it for a result (the header flag says why)
          poison_tile(a, rec);
        } else {
          run_tile_rows<MODE>(a, rec, lds, lane, w, pending);
        }
        // ROLE 1: this tile's row-block counter is added to by the workgroup's next tile once its
        // first stage has landed, or after the loop (a tile of ROLE 1 is never one that gave up);
        // without `defer_signal` at once, after a wait for this tile's stores
        if constexpr (ROLE == 1) {
          pending = &a.fam_done[rec.fam];
          if (!a.defer_signal) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
      }
      __syncthreads();       // every wave is past its epilogue
      if (threadIdx.x == 0) {
        if (ROLE == 1 && !a.defer_signal && pending != nullptr)
          __hip_atomic_fetch_add(pending, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *reinterpret_cast<volatile int*>(lds + kBcastOffset) = t_next;
      }
      if (ROLE == 1 && !a.defer_signal) pending = nullptr;
      __syncthreads();
      pos = __builtin_amdgcn_readfirstlane(*reinterpret_cast<volatile int*>(lds + kBcastOffset));
    }
  }
  if constexpr (ROLE == 1) {
    // the last tile of this workgroup in this list: wait for its stores, then add to its counter
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (pending != nullptr && threadIdx.x == 0)
      __hip_atomic_fetch_add(pending, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

// first: the tiles of list `p` in mode M0, then those of list `q` in mode M1; DEP: the second
// list's tiles wait for row blocks of the first
template <int M0, int M1, bool DEP>
__global__ void __launch_bounds__(Shape<M0>::THREADS) ffn_fused_kernel(const TileArgs p, const TileArgs q) {
  static_assert(Shape<M0>::THREADS == Shape<M1>::THREADS, "one workgroup shape");
  extern __shared__ __align__(1024) unsigned char lds[];
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  long long k0 = 0, r0 = 0, k1 = 0, r1 = 0;
  if (p.cycles) { k0 = __builtin_amdgcn_s_memtime(); r0 = __builtin_amdgcn_s_memrealtime(); }
  fused_phase<M0, DEP ? 1 : 0>(p, lds, lane, w);
  if (p.cycles) { k1 = __builtin_amdgcn_s_memtime(); r1 = __builtin_amdgcn_s_memrealtime(); }
  fused_phase<M1, DEP ? 2 : 0>(q, lds, lane, w);
  if (p.cycles && threadIdx.x == 0) {
    // second half of the buffer: [workgroup][8] = core clocks and 100 MHz ticks of the two
    // lists, then the 100 MHz time stamps of the workgroup's start and end
    long long* d = p.cycles + (size_t)(gridDim.x + blockIdx.x) * 8;
    const long long k2 = __builtin_amdgcn_s_memtime(), r2 = __builtin_amdgcn_s_memrealtime();
    d[0] = k1 - k0; d[1] = r1 - r0; d[2] = k2 - k1; d[3] = r2 - r1; d[4] = r0; d[5] = r2;
  }
}

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------
void apply_options(TileArgs& t, const FfnOptions& o) {
  t.band = o.band > 0 ? o.band : 1;
  t.group_major = o.group_major != 0;
  t.steal = o.steal;
  t.short_last = o.short_last != 0;
  t.defer_signal = o.defer_signal != 0;
  t.spin_limit = o.spin_limit == 0 ? kSpinLimit : o.spin_limit;
}

static long long max_tiles(const LayerDesc& L, bool up) {
  // smallest tile height 64 (forced) / 128 (chosen): every expert adds at most one partial tile
  const long long mt = (long long)L.P / 64 + L.Ne;
  const int ncols = up ? L.Fmax : L.d;
  const int ncpt = up ? kBN / 2 : kBN;
  return mt * ((ncols + ncpt - 1) / ncpt);
}

// row-block counters of the fused launch: at most one row block per 64 routed rows plus a
// partial one per expert
static size_t fam_bytes(const LayerDesc& L) {
  return ((size_t)(L.P / 64 + L.Ne + 1) * sizeof(int) + 255) / 256 * 256;
}

// bytes at the start of the workspace reserved for the two schedules and the row-block counters
size_t tiled_sched_bytes(const LayerDesc& L) {
  size_t b = 0;
  for (int up = 0; up < 2; ++up) {
    const size_t n = (size_t)max_tiles(L, up);
    b += 256 + (n * sizeof(TileRec) + 255) / 256 * 256;
  }
  return b + fam_bytes(L);
}

long long tile_capacity(const LayerDesc& L, int mode) {
  if (mode == kUp || mode == kUpSave) return max_tiles(L, true);
  if (mode == kDown || mode == kDgradX) return max_tiles(L, false);
  if (mode == kDgradH) return ((long long)L.P / 64 + L.Ne) * ((L.Fmax + kBN - 1) / kBN);
  const int m = L.d > 2 * L.Fmax ? L.d : 2 * L.Fmax, n = L.d > L.Fmax ? L.d : L.Fmax;
  return (long long)L.Ne * ((m + 63) / 64) * ((n + kBN - 1) / kBN);
}

int tile_num_cus() {
  static int n = 0;
  if (!n) {
    int dev = 0;
    hipDeviceProp_t p;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&p, dev) == hipSuccess)
      n = p.multiProcessorCount;
    if (n < kXcds) n = 256;
    n = n / kXcds * kXcds;
  }
  return n;
}

template <int MODE>
static hipError_t launch_stage(const TileArgs& a, hipStream_t s) {
  constexpr size_t smem = (size_t)(kStagesA * kBM + kStagesB * kBN) * kBK * 2;
  auto kern = ffn_tile_kernel<MODE>;
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  hipLaunchKernelGGL(kern, dim3(a.ncu), dim3(Shape<MODE>::THREADS), smem, s, a);
  return hipGetLastError();
}

template <int M0, int M1, bool DEP>
static hipError_t launch_fused(const TileArgs& up, const TileArgs& dn_in, hipStream_t s) {
  const TileArgs& dn = dn_in;
  constexpr size_t smem = (size_t)(kStagesA * kBM + kStagesB * kBN) * kBK * 2;
  auto kern = ffn_fused_kernel<M0, M1, DEP>;
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  hipLaunchKernelGGL(kern, dim3(up.ncu), dim3(Shape<M0>::THREADS), smem, s, up, dn);
  return hipGetLastError();
}

template <int MODE>
static hipError_t sched_and_run(const TileArgs& a, hipStream_t s) {
  hipLaunchKernelGGL((tile_schedule_kernel<MODE>), dim3(1), dim3(256), 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_stage<MODE>(a, s);
}

hipError_t launch_bwd_schedules(const TileArgs& dh, const TileArgs& dx, const TileArgs& w2,
                                const TileArgs& w13, const GatherArgs& ga, bool fused, hipStream_t s) {
  // at least one gather workgroup, so that the row of zeros gets written
  const unsigned gather_blocks = ga.P > 0 && ga.perm ? (unsigned)((ga.P + 3) / 4) : 1u;
  hipLaunchKernelGGL(bwd_schedule_kernel, dim3(4 + gather_blocks), dim3(256), 0, s, dh, dx, w2, w13,
                     fused ? 1 : 0, ga);
  return hipGetLastError();
}


// byte offset, inside the workspace of the forward, of the header of the list whose tiles wait
size_t tiled_waiting_header_offset(const LayerDesc& L) {
  return 256 + ((size_t)max_tiles(L, true) * sizeof(TileRec) + 255) / 256 * 256;
}

// dH and dX in one launch (dX tiles wait for the dH tiles of their row block)
hipError_t launch_dgrad_pair(const TileArgs& dh, const TileArgs& dx, hipStream_t s) {
  return launch_fused<kDgradH, kDgradX, true>(dh, dx, s);
}

// the two weight-gradient products in one launch
hipError_t launch_wgrad_pair(const TileArgs& w2, const TileArgs& w13, hipStream_t s) {
  return launch_fused<kWgrad, kWgrad, false>(w2, w13, s);
}

hipError_t launch_tiles(int mode, const TileArgs& a, hipStream_t s) {
  switch (mode) {
    case kDgradH: return launch_stage<kDgradH>(a, s);
    case kDgradX: return launch_stage<kDgradX>(a, s);
    case kWgrad: return launch_stage<kWgrad>(a, s);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_tile_gemm(int mode, const TileArgs& a, hipStream_t s) {
  switch (mode) {
    case kUpSave: return sched_and_run<kUpSave>(a, s);
    case kDgradH: return sched_and_run<kDgradH>(a, s);
    case kDgradX: return sched_and_run<kDgradX>(a, s);
    case kWgrad: return sched_and_run<kWgrad>(a, s);
    default: return hipErrorInvalidValue;
  }
}

// `pre` != NULL (training): the up projection also stores the backward factors b SiLU'(a) and
// SiLU(a) as rows of [P, 2*Fmax] for the backward pass.
hipError_t launch_ffn_tiled(const LayerDesc& L, const void* x, const int32_t* perm,
                            const int32_t* offsets, const GroupPtrs& W, void* y_perm, void* ws,
                            hipStream_t s, int stages, void* pre, int parts, const FfnOptions& o) {
  unsigned char* base = static_cast<unsigned char*>(ws);
  uint16_t* H = reinterpret_cast<uint16_t*>(base + tiled_sched_bytes(L));
  TileArgs up{};
  up.pre = static_cast<uint16_t*>(pre);
  up.ldpre = 2 * L.Fmax;
  up.A = static_cast<const uint16_t*>(x);
  up.perm = perm;
  up.offsets = offsets;
  up.C = H;
  up.lda = L.d; up.ldc = L.Fmax;
  up.Ke = L.Ke; up.Ng = L.Ng; up.N = L.N; up.Ne = L.Ne; up.d = L.d; up.P = L.P;
  up.ncu = tile_num_cus();
  apply_options(up, o);
  up.cycles = o.cycles;
  // visit groups by decreasing width: the down projection's longest reductions come first
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
    up.ldw[g] = L.d;
  }
  TileArgs dn = up;
  dn.A = H;
  dn.perm = nullptr;
  dn.C = static_cast<uint16_t*>(y_perm);
  dn.lda = L.Fmax; dn.ldc = L.d;
  for (int g = 0; g < kMaxGroups; ++g) {
    dn.W[g] = static_cast<const uint16_t*>(W.w2[g]);
    dn.ldw[g] = L.F[g];
  }
  // schedule areas: [header 256 B][records][cost prefix] for up, then the same for down
  unsigned char* p = base;
  for (int st = 0; st < 2; ++st) {
    TileArgs& t = st == 0 ? up : dn;
    const size_t n = (size_t)max_tiles(L, st == 0);
    t.hdr = reinterpret_cast<SchedHeader*>(p);
    p += 256;
    t.recs = reinterpret_cast<TileRec*>(p);
    p += (n * sizeof(TileRec) + 255) / 256 * 256;
    t.force_rows = o.tile_rows[st];
  }
  up.fam_done = dn.fam_done = reinterpret_cast<int*>(p);
  // the whole forward in one launch: up and down tiles share the persistent workgroups
  if (stages == 3 && o.fused) {
    up.coherent_out = 1;
    // parts: 1 = the tile schedule only, 2 = the product launch only (on a schedule that no
    // launch has consumed yet), 3 = both
    if (parts & 1) {
      hipLaunchKernelGGL(ffn_schedule_kernel, dim3(8), dim3(256), 0, s, up, dn, 7);
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
    }
    if (!(parts & 2)) return hipSuccess;
    return pre ? launch_fused<kUpSave, kDown, true>(up, dn, s) : launch_fused<kUp, kDown, true>(up, dn, s);
  }
  if (parts != 3) return hipErrorInvalidValue;       // (the API checks this before it gets here)
  // both schedules depend only on `offsets`: one launch builds whichever are needed
  hipLaunchKernelGGL(ffn_schedule_kernel, dim3(stages == 3 ? 2 : 1), dim3(256), 0, s, up, dn, stages);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (stages & 1) e = pre ? launch_stage<kUpSave>(up, s) : launch_stage<kUp>(up, s);
  if (e != hipSuccess) return e;
  if (stages & 2) e = launch_stage<kDown>(dn, s);
  return e;
}

}  // namespace mohge
