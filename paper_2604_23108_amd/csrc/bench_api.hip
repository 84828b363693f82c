// Host side of the benchmark library (mohge_bench.h): the expert-network calls with their launch
// options exposed, and the two ceiling probes.  Links against libmohge.so and uses its launchers;
// nothing here is needed to run the layer.
#include <string.h>

#include "common.h"
#include "mohge_bench.h"

namespace mohge {
hipError_t launch_probe_read(const void* buf, size_t bytes, int row_bytes, int staggered, void* out,
                             size_t* bytes_read, hipStream_t s);
hipError_t launch_probe_mfma(void* out, int blocks, int iters, double* flops, hipStream_t s);
}  // namespace mohge

using namespace mohge;

#define NEED(p) do { int rc_ = need((p), #p, true); if (rc_) return rc_; } while (0)
#define OPT(p) do { int rc_ = need((p), #p, false); if (rc_) return rc_; } while (0)

static int to_options(const mohge_ffn_options* in, const LayerDesc& L, FfnOptions* o) {
  if (!in) return MOHGE_OK;
  for (int i = 0; i < 2; ++i) {
    const int v = i == 0 ? in->tile_rows_up : in->tile_rows_down;
    if (v != 0 && v != 64 && v != 128 && v != 192 && v != 256) {
      set_error("mohge_ffn_options: tile rows = %d (0, 64, 128, 192 or 256)", v);
      return MOHGE_EINVAL;
    }
    o->tile_rows[i] = v;
  }
  if (in->band_rows < 0 || in->band_rows > (1 << 20)) { set_error("mohge_ffn_options: band_rows = %d", in->band_rows); return MOHGE_EINVAL; }
  o->fused = in->fused != 0;
  o->spin_limit = in->spin_limit;
  if (in->band_rows > 0) o->band = in->band_rows;
  o->group_major = in->group_major != 0;
  o->steal = in->steal & 3;
  o->short_last = in->short_last != 0;
  o->defer_signal = in->defer_signal != 0;
  if (in->cycles) {
    if (((uintptr_t)in->cycles) & 15) { set_error("mohge_ffn_options: cycles is not 16-byte aligned"); return MOHGE_EALIGN; }
    if (in->cycles_bytes < mohge_bench_cycles_bytes()) {
      set_error("mohge_ffn_options: cycles holds %zu bytes, %zu needed", in->cycles_bytes, mohge_bench_cycles_bytes());
      return MOHGE_EWORKSPACE;
    }
    o->cycles = static_cast<long long*>(in->cycles);
    o->cycles_launch = in->cycles_launch != 0;
  }
  (void)L;
  return MOHGE_OK;
}

static int weight_tables(const LayerDesc& L, const void* const* w13, const void* const* w2, GroupPtrs* W) {
  if (!w13 || !w2) { set_error("w13 / w2 pointer table is NULL"); return MOHGE_ENULL; }
  memset(W, 0, sizeof(*W));
  for (int g = 0; g < L.Ng; ++g) {
    NEED(w13[g]); NEED(w2[g]);
    W->w13[g] = w13[g];
    W->w2[g] = w2[g];
  }
  return MOHGE_OK;
}

extern "C" {

void mohge_ffn_default_options(mohge_ffn_options* o) {
  if (!o) return;
  const FfnOptions d;
  memset(o, 0, sizeof(*o));
  o->fused = d.fused;
  o->band_rows = d.band;
  o->group_major = d.group_major;
  o->steal = d.steal;
  o->short_last = d.short_last;
  o->defer_signal = d.defer_signal;
}

size_t mohge_bench_cycles_bytes(void) {
  int dev = 0, cus = 256;
  hipDeviceProp_t p;
  if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&p, dev) == hipSuccess && p.multiProcessorCount > 0)
    cus = p.multiProcessorCount;
  return (size_t)2 * cus * 8 * sizeof(long long);
}

int mohge_bench_expert_ffn(const mohge_config* cfg, const void* x, const int32_t* perm,
                           const int32_t* offsets, const void* const* w13, const void* const* w2,
                           void* y_perm, void* workspace, size_t workspace_bytes,
                           const mohge_ffn_options* options, int parts, void* stream) {
  LayerDesc L;
  int rc = check_config(cfg, &L);
  if (rc) return rc;
  FfnOptions o;
  if ((rc = to_options(options, L, &o))) return rc;
  if (parts < 1 || parts > 3) { set_error("mohge_bench_expert_ffn: parts = %d (1, 2 or 3)", parts); return MOHGE_EINVAL; }
  if (parts != 3 && (!ffn_parts_supported(L, cfg->dtype) || !o.fused)) {
    set_error("mohge_bench_expert_ffn: schedule and product launch are separate launches only in the fused form "
              "of the matrix-core path (MOHGE_BF16, T > 32, options->fused != 0)");
    return MOHGE_EINVAL;
  }
  NEED(x); OPT(perm); NEED(offsets); NEED(y_perm); NEED(workspace);
  GroupPtrs W;
  if ((rc = weight_tables(L, w13, w2, &W))) return rc;
  if (workspace_bytes < ffn_workspace_bytes(L, cfg->dtype)) {
    set_error("expert_ffn workspace: %zu bytes given, %zu needed", workspace_bytes, ffn_workspace_bytes(L, cfg->dtype));
    return MOHGE_EWORKSPACE;
  }
  if (L.T == 0) return MOHGE_OK;
  return hip_rc(launch_expert_ffn(L, cfg->dtype, x, perm, offsets, W, y_perm, workspace, (hipStream_t)stream, 3, parts, o),
                "mohge_bench_expert_ffn");
}

int mohge_bench_expert_ffn_train(const mohge_config* cfg, const void* x, const int32_t* perm,
                                 const int32_t* offsets, const void* const* w13, const void* const* w2,
                                 void* y_perm, void* saved, size_t saved_bytes,
                                 const mohge_ffn_options* options, void* stream) {
  LayerDesc L;
  int rc = check_config(cfg, &L);
  if (rc) return rc;
  if (cfg->dtype != MOHGE_BF16) { set_error("mohge_bench_expert_ffn_train is implemented for dtype MOHGE_BF16 only"); return MOHGE_EINVAL; }
  FfnOptions o;
  if ((rc = to_options(options, L, &o))) return rc;
  NEED(x); OPT(perm); NEED(offsets); NEED(y_perm); NEED(saved);
  GroupPtrs W;
  if ((rc = weight_tables(L, w13, w2, &W))) return rc;
  if (saved_bytes < ffn_saved_bytes(L)) {
    set_error("expert_ffn_train: saved has %zu bytes, %zu needed", saved_bytes, ffn_saved_bytes(L));
    return MOHGE_EWORKSPACE;
  }
  if (L.T == 0) return MOHGE_OK;
  return hip_rc(launch_expert_ffn_train(L, x, perm, offsets, W, y_perm, saved, (hipStream_t)stream, o),
                "mohge_bench_expert_ffn_train");
}

int mohge_bench_expert_ffn_bwd(const mohge_config* cfg, const void* x, const int32_t* perm,
                               const int32_t* offsets, const void* const* w13, const void* const* w2,
                               const void* saved, const void* dy_perm, void* dx_perm, void* const* dw13,
                               void* const* dw2, void* workspace, size_t workspace_bytes,
                               const mohge_ffn_options* options, void* stream) {
  LayerDesc L;
  int rc = check_config(cfg, &L);
  if (rc) return rc;
  if (cfg->dtype != MOHGE_BF16) { set_error("mohge_bench_expert_ffn_bwd is implemented for dtype MOHGE_BF16 only"); return MOHGE_EINVAL; }
  FfnOptions o;
  if ((rc = to_options(options, L, &o))) return rc;
  NEED(x); OPT(perm); NEED(offsets); NEED(saved); NEED(dy_perm); NEED(dx_perm); NEED(workspace);
  GroupPtrs W;
  if ((rc = weight_tables(L, w13, w2, &W))) return rc;
  if (!dw13 || !dw2) { set_error("dw13 / dw2 pointer table is NULL"); return MOHGE_ENULL; }
  void* g13[kMaxGroups];
  void* g2[kMaxGroups];
  for (int g = 0; g < L.Ng; ++g) { NEED(dw13[g]); NEED(dw2[g]); g13[g] = dw13[g]; g2[g] = dw2[g]; }
  if (workspace_bytes < ffn_bwd_workspace_bytes(L)) {
    set_error("expert_ffn_bwd workspace: %zu bytes given, %zu needed", workspace_bytes, ffn_bwd_workspace_bytes(L));
    return MOHGE_EWORKSPACE;
  }
  return hip_rc(launch_expert_ffn_bwd(L, x, perm, offsets, W, saved, dy_perm, dx_perm, g13, g2, workspace,
                                      (hipStream_t)stream, o),
                "mohge_bench_expert_ffn_bwd");
}

int mohge_probe_read(const void* buf, size_t bytes, int row_bytes, int staggered, void* out,
                     size_t* bytes_read, void* stream) {
  NEED(buf); NEED(out);
  if (!bytes_read) { set_error("bytes_read is NULL"); return MOHGE_ENULL; }
  if (row_bytes < 0 || (row_bytes != 0 && (row_bytes % 512 != 0 || row_bytes > (1 << 20)))) {
    set_error("mohge_probe_read: row_bytes = %d (0, or a multiple of 512 up to 1 MiB)", row_bytes);
    return MOHGE_EINVAL;
  }
  return hip_rc(launch_probe_read(buf, bytes, row_bytes, staggered != 0, out, bytes_read, (hipStream_t)stream),
                "mohge_probe_read");
}

int mohge_probe_mfma(void* out, size_t out_bytes, int iters, double* flops, void* stream) {
  NEED(out);
  if (!flops) { set_error("flops is NULL"); return MOHGE_ENULL; }
  const int blocks = 1024;
  if (out_bytes < (size_t)blocks * 256 * sizeof(float)) {
    set_error("mohge_probe_mfma: out holds %zu bytes, %zu needed", out_bytes, (size_t)blocks * 256 * sizeof(float));
    return MOHGE_EWORKSPACE;
  }
  if (iters < 1 || iters > (1 << 20)) { set_error("mohge_probe_mfma: iters = %d outside 1..2^20", iters); return MOHGE_EINVAL; }
  return hip_rc(launch_probe_mfma(out, blocks, iters, flops, (hipStream_t)stream), "mohge_probe_mfma");
}

size_t mohge_bench_decode_trace_bytes(const mohge_config* cfg) {
  LayerDesc L;
  if (check_config(cfg, &L) || !decode_layer_supported(L, cfg->dtype)) return 0;
  return (size_t)decode_layer_trace_entries(L) * 4 * sizeof(long long);
}

int mohge_bench_decode_layer(const mohge_config* cfg, const void* x, const float* w_group,
                             const float* w_expert, const float* expert_logit_bias,
                             const void* const* w13, const void* const* w2, int32_t* group_idx,
                             int32_t* expert_idx, float* gates, void* y, void* workspace,
                             size_t workspace_bytes, int spin_limit, void* trace, size_t trace_bytes, void* stream) {
  LayerDesc L;
  int rc = check_config(cfg, &L);
  if (rc) return rc;
  if (!decode_layer_supported(L, cfg->dtype)) {
    set_error("mohge_bench_decode_layer: bf16 calls of at most 32 tokens only");
    return MOHGE_EINVAL;
  }
  NEED(x); NEED(w_group); NEED(w_expert); OPT(expert_logit_bias);
  NEED(group_idx); NEED(expert_idx); NEED(gates); NEED(y); NEED(workspace);
  GroupPtrs W;
  if ((rc = weight_tables(L, w13, w2, &W))) return rc;
  if (workspace_bytes < decode_layer_workspace_bytes(L)) {
    set_error("decode_layer workspace: %zu bytes given, %zu needed", workspace_bytes, decode_layer_workspace_bytes(L));
    return MOHGE_EWORKSPACE;
  }
  OPT(trace);
  if (trace && trace_bytes < (size_t)decode_layer_trace_entries(L) * 4 * sizeof(long long)) {
    set_error("mohge_bench_decode_layer: trace of %zu bytes, mohge_bench_decode_trace_bytes says %zu", trace_bytes,
              (size_t)decode_layer_trace_entries(L) * 4 * sizeof(long long));
    return MOHGE_EWORKSPACE;
  }
  if (L.T == 0) return MOHGE_OK;
  return hip_rc(launch_decode_layer(L, x, w_group, w_expert, expert_logit_bias, W, group_idx, expert_idx, gates, y,
                                    workspace, spin_limit, static_cast<long long*>(trace), (hipStream_t)stream),
                "mohge_bench_decode_layer");
}

}  // extern "C"
