/*
 * mohge_bench.h — measurement and test aids around the MoHGE layer library (libmohge_bench.so,
 * which links against libmohge.so).  Nothing here is needed to run the layer: mohge.h is the
 * layer.  These calls expose how the matrix-core path of the expert networks is launched, so that
 * benchmarks can time its parts and tests can compare its launch forms bit by bit, and two kernels
 * that measure what the machine delivers.  Conventions (return codes, DEVICE / HOST pointers,
 * alignment, streams, mohge_last_error) are those of mohge.h.
 */
#ifndef MOHGE_BENCH_H
#define MOHGE_BENCH_H

#include "mohge.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Launch options of the bf16 matrix-core path (T > 32; ignored by the other paths).  They belong
 * to one call: there is no process-wide state.  Results do not depend on any of them, except a
 * negative spin_limit.  mohge_ffn_default_options fills in what the calls of mohge.h use.
 */
typedef struct mohge_ffn_options {
  int32_t tile_rows_up;    /* token-tile height of the up-projection list (forward) / of dH and dX
                              (backward): 0 = chosen per call from the routed counts, else 64, 128,
                              192 or 256                                                           */
  int32_t tile_rows_down;  /* the same for the down-projection list when the two projections are
                              separate launches (the fused launch uses one height for both)        */
  int32_t fused;           /* 1: up and down projection (backward: dH and dX; the two weight
                              gradients) as one launch each; 0: one launch per product             */
  int32_t spin_limit;      /* polls a dependent tile of a fused launch waits for its row block:
                              0 = default (about a second); > 0 = that many; < 0 = give up without
                              looking (test hook: the tiles then write NaN and mohge_fused_status
                              reports MOHGE_ETIMEOUT)                                              */
  int32_t band_rows;       /* row blocks per band of the tile order inside an expert (0 = default) */
  int32_t group_major;     /* 1: experts visited group by group (widest first); 0: by all-size sets */
  int32_t steal;           /* workgroups whose XCD range is exhausted draw from the other ranges:
                              bit 0 in the first list of a fused launch, bit 1 in the second (and
                              only where a list has at least four tiles per compute unit)          */
  int32_t short_last;      /* 1: in the second list of a fused launch the tiles with the shortest
                              reduction come last inside every XCD range                          */
  int32_t defer_signal;    /* 1: a tile of the first list is announced to its dependents from the
                              workgroup's next tile (when that tile's first loads have landed, the
                              stores before them are complete), 0: after waiting for its stores   */
  int32_t cycles_launch;   /* mohge_bench_expert_ffn_bwd: which fused launch fills `cycles`
                              (0 = dH / dX, 1 = the weight gradients)                              */
  void* cycles;            /* DEVICE or NULL: int64 counters of the fused launch, zeroed by the
                              caller, mohge_bench_cycles_bytes() bytes: [2][workgroups][8].
                              [0][w]: core clocks summed over w's tiles in tile setup, wait for the
                              first operand stages, main loop, epilogue; then tiles, reduction
                              stages, clocks spent waiting for row blocks, tiles that waited.
                              [1][w]: core clocks and 100 MHz ticks of w's first list, of its
                              second list, then the 100 MHz time stamps of w's start and end      */
  size_t cycles_bytes;
} mohge_ffn_options;

void mohge_ffn_default_options(mohge_ffn_options* options);
size_t mohge_bench_cycles_bytes(void);

/*
 * mohge_expert_ffn / mohge_expert_ffn_train / mohge_expert_ffn_bwd (same arguments, same kernels)
 * with explicit launch options (NULL = the defaults).
 * mohge_bench_expert_ffn, parts: on the fused matrix-core path the call is two launches: a small
 * kernel that turns `offsets` into the tile lists and hand-out counters (kept in the workspace),
 * and the launch that computes both projections from them.  parts = 1 issues the first, parts = 2
 * the second, parts = 3 both.  A parts = 2 call consumes the lists: each needs a parts = 1 call
 * with the same cfg, offsets, options and workspace before it, on the same stream or ordered after
 * it; without one it writes nothing useful to y_perm (no other harm).  parts 1 and 2 exist only
 * where the two launches do (MOHGE_BF16, T > 32, fused != 0); MOHGE_EINVAL otherwise.
 */
int mohge_bench_expert_ffn(const mohge_config* cfg, const void* x, const int32_t* perm,
                           const int32_t* offsets, const void* const* w13, const void* const* w2,
                           void* y_perm, void* workspace, size_t workspace_bytes,
                           const mohge_ffn_options* options, int parts, void* stream);
int mohge_bench_expert_ffn_train(const mohge_config* cfg, const void* x, const int32_t* perm,
                                 const int32_t* offsets, const void* const* w13, const void* const* w2,
                                 void* y_perm, void* saved, size_t saved_bytes,
                                 const mohge_ffn_options* options, void* stream);
int mohge_bench_expert_ffn_bwd(const mohge_config* cfg, const void* x, const int32_t* perm,
                               const int32_t* offsets, const void* const* w13, const void* const* w2,
                               const void* saved, const void* dy_perm, void* dx_perm, void* const* dw13,
                               void* const* dw2, void* workspace, size_t workspace_bytes,
                               const mohge_ffn_options* options, void* stream);

/*
 * mohge_decode_layer (same arguments, same kernel) with
 *  - spin_limit: the number of polls a waiting workgroup makes: 0 = the default (about a second),
 *    > 0 = that many, < 0 = give up without waiting (test hook: the launch drains, y is NaN and
 *    mohge_fused_status reports MOHGE_ETIMEOUT);
 *  - trace: NULL, or DEVICE int64 [pieces][4], mohge_bench_decode_trace_bytes(cfg) bytes, zeroed by
 *    the caller: 100 MHz time stamps of every piece of work of the launch.  Pieces are numbered in
 *    queue order: the route tasks, the select tasks, then the units of the experts that have rows
 *    (up units expert by expert, then down units in the order in which the experts' up units became
 *    complete).  [0] the piece was taken up, [1] down units: its expert was available, [3] done.
 */
int mohge_bench_decode_layer(const mohge_config* cfg, const void* x, const float* w_group,
                             const float* w_expert, const float* expert_logit_bias,
                             const void* const* w13, const void* const* w2, int32_t* group_idx,
                             int32_t* expert_idx, float* gates, void* y, void* workspace,
                             size_t workspace_bytes, int spin_limit, void* trace, size_t trace_bytes, void* stream);
size_t mohge_bench_decode_trace_bytes(const mohge_config* cfg);

/*
 * What the box delivers, for reading the kernels' fractions against measured ceilings.
 * mohge_probe_read enqueues a kernel that reads the first *bytes_read <= bytes bytes of buf
 * (DEVICE) exactly once and does nothing else: row_bytes = 0 as contiguous streams; otherwise
 * (a multiple of 512) with the access pattern of the decode kernels on rows of that size, the
 * waves walking their rows in step (staggered = 0) or each from a different start (1).  out:
 * DEVICE, at least 16 bytes, may receive a dummy value.  bytes_read: HOST.
 * mohge_probe_mfma enqueues 1024 workgroups that issue nothing but independent chains of
 * v_mfma_f32_32x32x16_bf16, `iters` per chain; *flops (HOST) receives the FLOPs of the launch;
 * out: DEVICE, at least 1 MiB.  Time either with events on `stream`.
 */
int mohge_probe_read(const void* buf, size_t bytes, int row_bytes, int staggered, void* out,
                     size_t* bytes_read, void* stream);
int mohge_probe_mfma(void* out, size_t out_bytes, int iters, double* flops, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MOHGE_BENCH_H */
