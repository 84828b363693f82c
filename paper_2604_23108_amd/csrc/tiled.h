// Argument block and schedule records of the ragged grouped GEMM tile kernel (bf16 matrix
// cores), shared by the forward launcher and the backward launcher.
#pragma once
#include "common.h"

namespace mohge {

constexpr int kXcds = 8;

// What a launch of the tile kernel computes: C = A . B with fp32 accumulation.  An operand is
// either contiguous along the reduction dimension ("plain": its LDS rows feed the matrix cores
// through 128-bit reads) or stored reduction-index major, i.e. with its features contiguous
// ("reduction-major": the fragments come out of LDS through the transposing 64-bit read).
enum TileMode {
  kUp = 0,       // H = SiLU(X Wg^T) * (X Wu^T): rows = routed tokens, reduction over d
  kDown = 1,     // Y = A W^T: rows = routed tokens, reduction over F[g]
  kUpSave = 2,   // kUp that also stores p = b SiLU'(a) and q = SiLU(a) for the backward pass
  kDgradH = 3,   // dH = dY W_down, then (dA, dB) = dH (p, q): reduction over d, B = W_down
                 //   as stored ([N, d, F]: reduction-major)
  kDgradX = 4,   // dX = [dA|dB] W13: reduction over F[g] := 2 F_g, B = W13 as stored ([N, 2F, d])
  kWgrad = 5     // dW_e = A_e^T B_e over the routed rows of expert e: both operands token-major
                 //   ([P, features]), i.e. reduction-major
};

struct TileRec {
  int e;          // expert
  int row_start;  // first row of the tile: sorted position / row of dW_e (kWgrad)
  int rows;       // valid rows (1..256)
  int n0;         // first output column
  int fam;        // token modes: index of the tile's (expert, row block) among all row blocks
  int need;       // fused forward, down tiles: up tiles that must have finished (else 0)
};

struct SchedHeader {
  int tile_rows;             // chosen tile height
  int total;                 // number of tiles
  int xcd_begin[kXcds + 1];  // tile ranges per XCD
  int counters[kXcds];       // next tile of each range not yet handed out
  int tail[kXcds];           // tiles at the end of each range whose expert continues in the next range
  int pad[5];                // pad[0]: set by a tile of a fused launch that gave up waiting for its row block
};
static_assert(sizeof(SchedHeader) <= 256, "header area");

struct TileArgs {
  const uint16_t* A;          // token modes: [rows, lda] (kUp*: x, gathered through perm if given)
                              // kWgrad: [P, lda] in sorted order, its columns are the rows of dW
  const int32_t* perm;        // kUp* only, may be NULL
  const int32_t* offsets;     // [Ne+1] routed rows per expert (exclusive prefix sum)
  const uint16_t* W[kMaxGroups];   // weight operand per group (all modes but kWgrad)
  int ldw[kMaxGroups];        // row pitch of W[g] in elements
  uint16_t* C;                // token modes: output [P, ldc]
  int lda, ldc;
  int Ke, Ng, N, Ne, d, P;
  int F[kMaxGroups];          // kUp*, kDgradH: output width F_g; kDown: reduction length
  int order[kMaxGroups];      // groups in visiting order (longest reduction first)
  SchedHeader* hdr;
  TileRec* recs;
  int ncu;                    // compute units = persistent workgroups
  int force_rows;             // 0 = choose, else 64/128/192/256
  int group_major;            // visiting order of the experts (see visit())
  int steal;                  // fused launches: workgroups whose range is exhausted help the other ranges
  int short_last;             // fused launches, second list: shortest reductions last inside every XCD range
  int defer_signal;           // fused launches, first list: a tile's row-block counter is added to in the next tile's prologue
  int band;                   // row blocks per band of the tile order inside an expert (>= 1)
  // --- fused forward (up and down tiles in one launch) ------------------------------------
  int* fam_done;              // [row blocks] finished up tiles per row block (zeroed by the schedule)
  int spin_limit;             // fused launches: polls a dependent tile waits (set by launch_fused)
  int coherent_out;           // kUp*: store H at device scope, so that a down tile running on
                              //   another XCD reads what an up tile wrote in the same launch
  // --- backward extensions -------------------------------------------------------------
  uint16_t* pre;              // kUpSave: out, kDgradH: in; [P, ldpre], row = p[0..F_g) q[0..F_g)
  uint16_t* C2;               // kDgradH: out [P, ldpre], row = dA[0..F_g) dB[0..F_g)
  int ldpre;
  const uint16_t* B2;         // kWgrad: [P, ldb] in sorted order, its columns are the columns of dW
  int ldb;
  const uint16_t* zero_row;   // kWgrad: 512 bytes of zeros (stands in for the rows past an
                              //   expert's last token in its final 64-token stage)
  uint16_t* Wout[kMaxGroups]; // kWgrad: dW per group, [N, Mrows[g], Ncols[g]]
  int Mrows[kMaxGroups], Ncols[kMaxGroups];
  long long* cycles;          // NULL, or [2 * workgroups][8] counters of the fused launches (tile_cycles.md
                              //   layout in mohge_bench.h): clock sums per tile phase, tiles, stages, waits
};

// One schedule launch + one tile-kernel launch for `mode` (backward modes and kUpSave).
hipError_t launch_tile_gemm(int mode, const TileArgs& a, hipStream_t s);
// The expert backward pass: all four schedules in one launch, then the tile launches alone.
// The same launch also gathers the rows of x into sorted order (xs[p] = x[perm[p] / Ke], nothing
// if perm == NULL) and clears the 512-byte row of zeros: workgroups beyond the first four.
struct GatherArgs {
  const uint4* x;
  const int32_t* perm;
  uint4* xs;
  uint4* zero_row;
  int P, Ke, chunks;          // chunks = 16-byte pieces of a row
};
hipError_t launch_bwd_schedules(const TileArgs& dh, const TileArgs& dx, const TileArgs& w2,
                                const TileArgs& w13, const GatherArgs& ga, bool fused, hipStream_t s);
hipError_t launch_tiles(int mode, const TileArgs& a, hipStream_t s);
// Fused launches (the default form): dH then dX in one launch, the two weight gradients in one
// launch.  The schedules must have been built in the same form (`fused`).
void apply_options(TileArgs& t, const FfnOptions& o);
size_t tiled_waiting_header_offset(const LayerDesc& L);
hipError_t launch_dgrad_pair(const TileArgs& dh, const TileArgs& dx, hipStream_t s);
hipError_t launch_wgrad_pair(const TileArgs& w2, const TileArgs& w13, hipStream_t s);
// Largest number of tiles a schedule of `mode` can hold for layer L (sizes the record area).
long long tile_capacity(const LayerDesc& L, int mode);
int tile_num_cus();

}  // namespace mohge
