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
// All of it runs as four launches of the ragged grouped GEMM tile kernel of the forward pass:
//   dH   = dY . W_down        reduction over d        (SwiGLU derivative fused: writes [dA|dB])
//   dX   = [dA|dB] . W13      reduction over 2 F_g
//   dW2  = dY^T . H           reduction over the expert's routed rows
//   dW13 = [dA|dB]^T . X      reduction over the expert's routed rows
// In every one of them the second operand (in the last two, both) is stored with the reduction
// index as the row; the tile kernel reads such operands through the transposing LDS read, so
// the weights are used as the forward pass stores them and no activation is transposed in
// memory.  The only helper pass gathers the rows of x into sorted order for the last product
// (the other three activations already are in sorted order); it shares a launch with the tile
// schedules.
#include "common.h"
#include "tiled.h"

namespace mohge {

const void* saved_h(const LayerDesc& L, const void* saved);
const void* saved_pre(const LayerDesc& L, const void* saved);

// ---------------------------------------------------------------------------------------
// workspace layout and the launch sequence
// ---------------------------------------------------------------------------------------
static size_t up256(size_t b) { return (b + 255) / 256 * 256; }

struct BwdLayout {
  size_t sched[4], recs[4];   // dgrad-h, dgrad-x, wgrad-2, wgrad-13
  size_t zero, fam, dab, xs, total;
};

static BwdLayout bwd_layout(const LayerDesc& L) {
  BwdLayout o;
  const int modes[4] = {kDgradH, kDgradX, kWgrad, kWgrad};
  size_t p = 0;
  for (int i = 0; i < 4; ++i) {
    o.sched[i] = p; p += 256;
    o.recs[i] = p; p += up256((size_t)tile_capacity(L, modes[i]) * sizeof(TileRec));
  }
  const size_t P = L.P > 0 ? L.P : 1;
  o.zero = p; p += 512;
  o.fam = p;  p += up256((size_t)(L.P / 64 + L.Ne + 1) * sizeof(int));     // row-block counters
  o.dab = p;  p += up256(P * 2 * L.Fmax * 2);
  o.xs = p;   p += up256(P * L.d * 2);
  o.total = p;
  return o;
}

size_t ffn_bwd_workspace_bytes(const LayerDesc& L) { return bwd_layout(L).total; }
// header of the list whose tiles wait in the fused dH / dX launch
size_t ffn_bwd_waiting_header_offset(const LayerDesc& L) { return bwd_layout(L).sched[1]; }

hipError_t launch_expert_ffn_bwd(const LayerDesc& L, const void* x, const int32_t* perm,
                                 const int32_t* offsets, const GroupPtrs& W, const void* saved,
                                 const void* dy_perm, void* dx_perm, void* const* dw13,
                                 void* const* dw2, void* ws, hipStream_t s, const FfnOptions& o) {
  const BwdLayout lay = bwd_layout(L);
  unsigned char* base = static_cast<unsigned char*>(ws);
  uint16_t* zero_row = reinterpret_cast<uint16_t*>(base + lay.zero);
  uint16_t* dab = reinterpret_cast<uint16_t*>(base + lay.dab);
  uint16_t* xs = reinterpret_cast<uint16_t*>(base + lay.xs);

  TileArgs t{};
  t.offsets = offsets;
  t.Ke = L.Ke; t.Ng = L.Ng; t.N = L.N; t.Ne = L.Ne; t.d = L.d; t.P = L.P;
  t.ncu = tile_num_cus();
  apply_options(t, o);
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

  TileArgs dh = with_sched(t, 0), dxa = with_sched(t, 1), w2a = with_sched(t, 2), w13a = with_sched(t, 3);
  // dH = dY W_down, fused with the SwiGLU derivative: [dA|dB] rows
  dh.A = static_cast<const uint16_t*>(dy_perm);
  dh.lda = L.d;
  dh.pre = const_cast<uint16_t*>(static_cast<const uint16_t*>(saved_pre(L, saved)));
  dh.C2 = dab;
  // dX = [dA|dB] W13: reduction length 2 F_g
  dxa.A = dab;
  dxa.lda = 2 * L.Fmax;
  dxa.C = static_cast<uint16_t*>(dx_perm);
  dxa.ldc = L.d;
  // dW_down[e] = dY_e^T H_e : rows d, columns F_g
  w2a.A = static_cast<const uint16_t*>(dy_perm); w2a.lda = L.d;
  w2a.B2 = static_cast<const uint16_t*>(saved_h(L, saved)); w2a.ldb = L.Fmax;
  // dW13[e] = [dA|dB]_e^T X_e : rows 2 F_g (gate rows, then up rows), columns d
  w13a.A = dab; w13a.lda = 2 * L.Fmax; w13a.ldb = L.d;
  w13a.B2 = perm ? xs : static_cast<const uint16_t*>(x);
  w2a.zero_row = w13a.zero_row = zero_row;
  w2a.force_rows = w13a.force_rows = 256;
  for (int g = 0; g < L.Ng; ++g) {
    dh.F[g] = L.F[g]; dh.W[g] = static_cast<const uint16_t*>(W.w2[g]); dh.ldw[g] = L.F[g];
    dxa.F[g] = 2 * L.F[g]; dxa.W[g] = static_cast<const uint16_t*>(W.w13[g]); dxa.ldw[g] = L.d;
    w2a.F[g] = L.F[g]; w2a.Mrows[g] = L.d; w2a.Ncols[g] = L.F[g];
    w2a.Wout[g] = static_cast<uint16_t*>(dw2[g]);
    w13a.F[g] = L.F[g]; w13a.Mrows[g] = 2 * L.F[g]; w13a.Ncols[g] = L.d;
    w13a.Wout[g] = static_cast<uint16_t*>(dw13[g]);
  }

  // optional clock counters of one of the two fused launches (both lists of a launch share them)
  if (o.cycles) {
    if (o.cycles_launch == 0) dh.cycles = dxa.cycles = o.cycles;
    else w2a.cycles = w13a.cycles = o.cycles;
  }
  // fused form: dX tiles wait for the row-block counters the dH tiles increment
  const bool fused = o.fused != 0;
  if (fused) {
    dh.coherent_out = 1;
    dh.fam_done = dxa.fam_done = reinterpret_cast<int*>(base + lay.fam);
  }
  // one launch: all four tile schedules (they depend on `offsets` only) and, on further
  // workgroups, x in sorted order and the row of zeros; then the products
  GatherArgs ga;
  ga.x = static_cast<const uint4*>(x); ga.perm = perm; ga.xs = reinterpret_cast<uint4*>(xs);
  ga.zero_row = reinterpret_cast<uint4*>(zero_row); ga.P = L.P; ga.Ke = L.Ke; ga.chunks = L.d / 8;
  hipError_t e = launch_bwd_schedules(dh, dxa, w2a, w13a, ga, fused, s);
  if (e != hipSuccess) return e;
  if (fused) {
    if ((e = launch_dgrad_pair(dh, dxa, s)) != hipSuccess) return e;
    return launch_wgrad_pair(w2a, w13a, s);
  }
  if ((e = launch_tiles(kDgradH, dh, s)) != hipSuccess) return e;
  if ((e = launch_tiles(kDgradX, dxa, s)) != hipSuccess) return e;
  if ((e = launch_tiles(kWgrad, w2a, s)) != hipSuccess) return e;
  e = launch_tiles(kWgrad, w13a, s);
  return e;
}

}  // namespace mohge
