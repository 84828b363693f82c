// Host side of the C boundary: argument checking, error strings, dispatch to launchers.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include "common.h"
#include "tiled.h"

namespace mohge {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

int check_config(const mohge_config* c, LayerDesc* L) {
  if (!c) { set_error("cfg is NULL"); return MOHGE_ENULL; }
  if (!c->d_ff) { set_error("cfg->d_ff is NULL"); return MOHGE_ENULL; }
  if (c->T < 0) { set_error("T = %d is negative", c->T); return MOHGE_EINVAL; }
  if (c->d < 64 || c->d % 64) { set_error("d = %d must be a positive multiple of 64", c->d); return MOHGE_EINVAL; }
  if (c->n_groups < 1 || c->n_groups > kMaxGroups) {
    set_error("n_groups = %d outside 1..%d", c->n_groups, kMaxGroups); return MOHGE_EINVAL; }
  if (c->experts_per_group < 1 || (int64_t)c->experts_per_group * c->n_groups > kMaxExperts) {
    set_error("n_groups*experts_per_group = %lld outside 1..%d",
              (long long)c->experts_per_group * c->n_groups, kMaxExperts); return MOHGE_EINVAL; }
  if (c->k_groups < 1 || c->k_groups > c->n_groups) {
    set_error("k_groups = %d outside 1..n_groups", c->k_groups); return MOHGE_EINVAL; }
  if (c->k_experts < 1 || c->k_experts > c->k_groups * c->experts_per_group) {
    set_error("k_experts = %d outside 1..k_groups*experts_per_group", c->k_experts); return MOHGE_EINVAL; }
  if (c->select_mode == MOHGE_SELECT_PER_GROUP) {
    if (c->k_experts % c->k_groups || c->k_experts / c->k_groups > c->experts_per_group) {
      set_error("per-group selection needs k_experts %% k_groups == 0 and k_experts/k_groups <= experts_per_group");
      return MOHGE_EINVAL; }
  } else if (c->select_mode != MOHGE_SELECT_GLOBAL) {
    set_error("select_mode = %d unknown", c->select_mode); return MOHGE_EINVAL; }
  if (c->dtype != MOHGE_F32 && c->dtype != MOHGE_BF16) {
    set_error("dtype = %d unknown", c->dtype); return MOHGE_EINVAL; }
  if ((int64_t)c->T * c->k_experts >= (int64_t)1 << 31) {
    set_error("T*k_experts does not fit int32"); return MOHGE_EINVAL; }
  int fmax = 0;
  for (int g = 0; g < c->n_groups; ++g) {
    int F = c->d_ff[g];
    if (F < 64 || F % 64) { set_error("d_ff[%d] = %d must be a positive multiple of 64", g, F); return MOHGE_EINVAL; }
    if (F > fmax) fmax = F;
  }
  if (L) {
    memset(L, 0, sizeof(*L));
    L->T = c->T; L->d = c->d; L->Ng = c->n_groups; L->N = c->experts_per_group;
    L->Ne = L->Ng * L->N; L->Kg = c->k_groups; L->Ke = c->k_experts; L->P = c->T * c->k_experts;
    L->select_mode = c->select_mode; L->Fmax = fmax;
    for (int g = 0; g < L->Ng; ++g) L->F[g] = c->d_ff[g];
  }
  return MOHGE_OK;
}

int need(const void* p, const char* name, bool required) {
  if (!p) {
    if (!required) return MOHGE_OK;
    set_error("%s is NULL", name);
    return MOHGE_ENULL;
  }
  if (((uintptr_t)p) & 15) { set_error("%s is not 16-byte aligned", name); return MOHGE_EALIGN; }
  return MOHGE_OK;
}

int hip_rc(hipError_t e, const char* what) {
  if (e == hipSuccess) return MOHGE_OK;
  set_error("%s: %s", what, hipGetErrorString(e));
  return MOHGE_EHIP;
}

}  // namespace mohge

using namespace mohge;

#define NEED(p) do { int rc_ = need((p), #p, true); if (rc_) return rc_; } while (0)
#define OPT(p) do { int rc_ = need((p), #p, false); if (rc_) return rc_; } while (0)

extern "C" {

const char* mohge_last_error(void) { return g_err; }

int mohge_fused_status(const mohge_config* cfg, int which_call, const void* workspace,
                       size_t workspace_bytes, void* stream) {
  LayerDesc L;
  int rc = check_config(cfg, &L);
  if (rc) return rc;
  if (which_call == MOHGE_CALL_DECODE_LAYER) {
    if (!decode_layer_supported(L, cfg->dtype) || L.T == 0) return MOHGE_OK;
    NEED(workspace);
    if (workspace_bytes < decode_layer_workspace_bytes(L)) {
      set_error("mohge_fused_status: workspace of %zu bytes, the call uses %zu", workspace_bytes,
                decode_layer_workspace_bytes(L));
      return MOHGE_EWORKSPACE;
    }
    hipError_t e = hipStreamSynchronize((hipStream_t)stream);
    if (e != hipSuccess) return hip_rc(e, "mohge_fused_status (synchronise)");
    int st = 0;
    e = hipMemcpy(&st, static_cast<const unsigned char*>(workspace) + decode_layer_status_offset(L), sizeof(st),
                  hipMemcpyDeviceToHost);
    if (e != hipSuccess) return hip_rc(e, "mohge_fused_status (copy)");
    if (st & 2) {
      set_error("mohge_decode_layer: the counters at the start of the workspace were not zero when the call started");
      return MOHGE_EINVAL;
    }
    if (st != 0) {
      set_error("mohge_decode_layer: a workgroup gave up waiting for the work it depends on: y holds NaN");
      return MOHGE_ETIMEOUT;
    }
    return MOHGE_OK;
  }
  if (which_call != MOHGE_CALL_EXPERT_FFN && which_call != MOHGE_CALL_FFN_SAVED &&
      which_call != MOHGE_CALL_EXPERT_FFN_BWD) {
    set_error("mohge_fused_status: call id %d has no fused launch", which_call);
    return MOHGE_EINVAL;
  }
  const long long off = fused_flag_offset(L, cfg->dtype, which_call);
  if (off < 0 || L.T == 0) return MOHGE_OK;
  NEED(workspace);
  if (workspace_bytes < mohge_workspace_size(cfg, which_call)) {
    set_error("mohge_fused_status: workspace of %zu bytes, the call uses %zu", workspace_bytes,
              mohge_workspace_size(cfg, which_call));
    return MOHGE_EWORKSPACE;
  }
  hipError_t e = hipStreamSynchronize((hipStream_t)stream);
  if (e != hipSuccess) return hip_rc(e, "mohge_fused_status (synchronise)");
  SchedHeader h;
  e = hipMemcpy(&h, static_cast<const unsigned char*>(workspace) + off, sizeof(h), hipMemcpyDeviceToHost);
  if (e != hipSuccess) return hip_rc(e, "mohge_fused_status (copy)");
  if (h.pad[0] != 0) {
    set_error("a dependent tile of the fused launch gave up waiting for its row block: output unreliable");
    return MOHGE_ETIMEOUT;
  }
  return MOHGE_OK;
}

size_t mohge_workspace_size(const mohge_config* cfg, int which_call) {
  LayerDesc L;
  if (check_config(cfg, &L)) return 0;
  switch (which_call) {
    case MOHGE_CALL_PERMUTE: return permute_workspace_bytes(L);
    case MOHGE_CALL_EXPERT_FFN: return ffn_workspace_bytes(L, cfg->dtype);
    case MOHGE_CALL_AUX_LOSS: return aux_workspace_bytes(L);
    case MOHGE_CALL_FFN_SAVED: return ffn_saved_bytes(L);
    case MOHGE_CALL_EXPERT_FFN_BWD: return ffn_bwd_workspace_bytes(L);
    case MOHGE_CALL_ROUTE_BWD: return route_bwd_workspace_bytes(L);
    case MOHGE_CALL_ROUTE: return route_workspace_bytes(L, cfg->dtype);
    case MOHGE_CALL_DECODE_LAYER: return decode_layer_supported(L, cfg->dtype) ? decode_layer_workspace_bytes(L) : 0;
    default: set_error("unknown call id %d", which_call); return 0;
  }
}

int mohge_route(const mohge_config* cfg, const void* x, const float* w_group,
                const float* w_expert, const float* expert_logit_bias, int32_t* group_idx,
                int32_t* expert_idx, float* gates, float* gs_out, float* es1_out,
                void* workspace, size_t workspace_bytes, void* stream) {
  LayerDesc L;
  int rc = check_config(cfg, &L);
  if (rc) return rc;
  NEED(x); NEED(w_group); NEED(w_expert); OPT(expert_logit_bias);
  NEED(group_idx); NEED(expert_idx); NEED(gates); OPT(gs_out); OPT(es1_out); OPT(workspace);
  if (L.T == 0) return MOHGE_OK;
  return hip_rc(launch_route(L, cfg->dtype, x, w_group, w_expert, expert_logit_bias, group_idx,
                             expert_idx, gates, gs_out, es1_out, workspace, workspace_bytes,
                             (hipStream_t)stream),
                "mohge_route");
}

int mohge_permute(const mohge_config* cfg, const int32_t* expert_idx, int32_t* counts,
                  int32_t* offsets, int32_t* perm, int32_t* inv_perm, const void* x,
                  void* x_perm, void* workspace, size_t workspace_bytes, void* stream) {
  LayerDesc L;
  int rc = check_config(cfg, &L);
  if (rc) return rc;
  NEED(expert_idx); NEED(counts); NEED(offsets); NEED(perm); NEED(inv_perm);
  OPT(x); OPT(x_perm); NEED(workspace);
  if (x_perm && !x) { set_error("x_perm requested but x is NULL"); return MOHGE_ENULL; }
  if (workspace_bytes < permute_workspace_bytes(L)) {
    set_error("permute workspace: %zu bytes given, %zu needed", workspace_bytes,
              permute_workspace_bytes(L));
    return MOHGE_EWORKSPACE;
  }
  return hip_rc(launch_permute(L, cfg->dtype, expert_idx, counts, offsets, perm, inv_perm, x,
                               x_perm, workspace, (hipStream_t)stream),
                "mohge_permute");
}

int mohge_permute_static(const mohge_config* cfg, const int32_t* expert_idx, int32_t* counts,
                         int32_t* offsets, int32_t* perm, int32_t* inv_perm, const void* x,
                         void* x_perm, void* stream) {
  LayerDesc L;
  int rc = check_config(cfg, &L);
  if (rc) return rc;
  NEED(expert_idx); NEED(counts); NEED(offsets); NEED(perm); NEED(inv_perm);
  OPT(x); OPT(x_perm);
  if (x_perm && !x) { set_error("x_perm requested but x is NULL"); return MOHGE_ENULL; }
  if (permute_workspace_bytes(L) > (size_t)MOHGE_PERMUTE_STATIC_BYTES) {
    set_error("mohge_permute_static: this configuration needs %zu bytes of scratch, the static buffer holds %zu "
              "(use mohge_permute with a workspace)", permute_workspace_bytes(L),
              (size_t)MOHGE_PERMUTE_STATIC_BYTES);
    return MOHGE_EWORKSPACE;
  }
  return hip_rc(launch_permute_static(L, cfg->dtype, expert_idx, counts, offsets, perm, inv_perm, x,
                                      x_perm, (hipStream_t)stream),
                "mohge_permute_static");
}

int mohge_expert_ffn(const mohge_config* cfg, const void* x, const int32_t* perm,
                     const int32_t* offsets, const void* const* w13, const void* const* w2,
                     void* y_perm, void* workspace, size_t workspace_bytes, void* stream) {
  LayerDesc L;
  int rc = check_config(cfg, &L);
  if (rc) return rc;
  NEED(x); OPT(perm); NEED(offsets); NEED(y_perm); NEED(workspace);
  if (!w13 || !w2) { set_error("w13 / w2 pointer table is NULL"); return MOHGE_ENULL; }
  GroupPtrs W;
  memset(&W, 0, sizeof(W));
  for (int g = 0; g < L.Ng; ++g) {
    NEED(w13[g]); NEED(w2[g]);
    W.w13[g] = w13[g];
    W.w2[g] = w2[g];
  }
  if (workspace_bytes < ffn_workspace_bytes(L, cfg->dtype)) {
    set_error("expert_ffn workspace: %zu bytes given, %zu needed", workspace_bytes,
              ffn_workspace_bytes(L, cfg->dtype));
    return MOHGE_EWORKSPACE;
  }
  if (L.T == 0) return MOHGE_OK;
  return hip_rc(launch_expert_ffn(L, cfg->dtype, x, perm, offsets, W, y_perm, workspace,
                                  (hipStream_t)stream, 3),
                "mohge_expert_ffn");
}

static int decode_layer_args(const mohge_config* cfg, LayerDesc& L, const void* x, const float* w_group,
                             const float* w_expert, const float* expert_logit_bias, const void* const* w13,
                             const void* const* w2, int32_t* group_idx, int32_t* expert_idx, float* gates,
                             void* y, void* workspace, size_t workspace_bytes, GroupPtrs& W) {
  int rc = check_config(cfg, &L);
  if (rc) return rc;
  if (!decode_layer_supported(L, cfg->dtype)) {
    set_error("mohge_decode_layer serves bf16 calls of at most 32 tokens and 2048 (token, expert) pairs: "
              "dtype = %d, T = %d, T*K_e = %d", cfg->dtype, L.T, L.P);
    return MOHGE_EINVAL;
  }
  NEED(x); NEED(w_group); NEED(w_expert); OPT(expert_logit_bias);
  NEED(group_idx); NEED(expert_idx); NEED(gates); NEED(y); NEED(workspace);
  if (!w13 || !w2) { set_error("w13 / w2 pointer table is NULL"); return MOHGE_ENULL; }
  memset(&W, 0, sizeof(W));
  for (int g = 0; g < L.Ng; ++g) {
    NEED(w13[g]); NEED(w2[g]);
    W.w13[g] = w13[g];
    W.w2[g] = w2[g];
  }
  if (workspace_bytes < decode_layer_workspace_bytes(L)) {
    set_error("decode_layer workspace: %zu bytes given, %zu needed", workspace_bytes, decode_layer_workspace_bytes(L));
    return MOHGE_EWORKSPACE;
  }
  return MOHGE_OK;
}

int mohge_decode_layer(const mohge_config* cfg, const void* x, const float* w_group,
                       const float* w_expert, const float* expert_logit_bias,
                       const void* const* w13, const void* const* w2, int32_t* group_idx,
                       int32_t* expert_idx, float* gates, void* y, void* workspace,
                       size_t workspace_bytes, void* stream) {
  LayerDesc L;
  GroupPtrs W;
  int rc = decode_layer_args(cfg, L, x, w_group, w_expert, expert_logit_bias, w13, w2, group_idx, expert_idx,
                             gates, y, workspace, workspace_bytes, W);
  if (rc) return rc;
  if (L.T == 0) return MOHGE_OK;
  return hip_rc(launch_decode_layer(L, x, w_group, w_expert, expert_logit_bias, W, group_idx, expert_idx, gates,
                                    y, workspace, 0, nullptr, (hipStream_t)stream),
                "mohge_decode_layer");
}

size_t mohge_decode_layer_ctl_bytes(const mohge_config* cfg) {
  LayerDesc L;
  if (check_config(cfg, &L) || !decode_layer_supported(L, cfg->dtype)) return 0;
  return decode_layer_ctl_bytes(L);
}

static int need_bf16(const mohge_config* cfg, const char* what) {
  if (cfg->dtype != MOHGE_BF16) {
    set_error("%s is implemented for dtype MOHGE_BF16 only", what);
    return MOHGE_EINVAL;
  }
  return MOHGE_OK;
}

int mohge_expert_ffn_w8(const mohge_config* cfg, const void* x, const int32_t* perm,
                        const int32_t* offsets, const void* const* w13q, const float* const* w13_scale,
                        const void* const* w2q, const float* const* w2_scale, void* y_perm,
                        void* workspace, size_t workspace_bytes, void* stream) {
  LayerDesc L;
  int rc = check_config(cfg, &L);
  if (rc) return rc;
  if ((rc = need_bf16(cfg, "mohge_expert_ffn_w8"))) return rc;
  if (!ffn_w8_supported(L)) {
    set_error("mohge_expert_ffn_w8: FP8 weights are served by the decode path only (T <= 32), T = %d", L.T);
    return MOHGE_EINVAL;
  }
  NEED(x); OPT(perm); NEED(offsets); NEED(y_perm); NEED(workspace);
  if (!w13q || !w2q || !w13_scale || !w2_scale) { set_error("a weight / scale pointer table is NULL"); return MOHGE_ENULL; }
  GroupPtrs W;
  memset(&W, 0, sizeof(W));
  const float* s13[kMaxGroups];
  const float* s2[kMaxGroups];
  for (int g = 0; g < L.Ng; ++g) {
    NEED(w13q[g]); NEED(w2q[g]); NEED(w13_scale[g]); NEED(w2_scale[g]);
    W.w13[g] = w13q[g];
    W.w2[g] = w2q[g];
    s13[g] = w13_scale[g];
    s2[g] = w2_scale[g];
  }
  if (workspace_bytes < ffn_workspace_bytes(L, cfg->dtype)) {
    set_error("expert_ffn_w8 workspace: %zu bytes given, %zu needed", workspace_bytes,
              ffn_workspace_bytes(L, cfg->dtype));
    return MOHGE_EWORKSPACE;
  }
  if (L.T == 0) return MOHGE_OK;
  return hip_rc(launch_expert_ffn_w8(L, x, perm, offsets, W, s13, s2, y_perm, workspace, (hipStream_t)stream),
                "mohge_expert_ffn_w8");
}

int mohge_fp8_decode(const void* codes, float* out, size_t n, void* stream) {
  if (n == 0) return MOHGE_OK;
  NEED(codes); NEED(out);
  return hip_rc(launch_fp8_decode(codes, out, (long long)n, (hipStream_t)stream), "mohge_fp8_decode");
}

int mohge_expert_ffn_w4(const mohge_config* cfg, const void* x, const int32_t* perm,
                        const int32_t* offsets, const void* const* w13q, const void* const* w13_scale,
                        const void* const* w2q, const void* const* w2_scale, void* y_perm,
                        void* workspace, size_t workspace_bytes, void* stream) {
  LayerDesc L;
  int rc = check_config(cfg, &L);
  if (rc) return rc;
  if ((rc = need_bf16(cfg, "mohge_expert_ffn_w4"))) return rc;
  if (!ffn_w8_supported(L)) {
    set_error("mohge_expert_ffn_w4: MXFP4 weights are served by the decode path only (T <= 32), T = %d", L.T);
    return MOHGE_EINVAL;
  }
  NEED(x); OPT(perm); NEED(offsets); NEED(y_perm); NEED(workspace);
  if (!w13q || !w2q || !w13_scale || !w2_scale) { set_error("a weight / scale pointer table is NULL"); return MOHGE_ENULL; }
  GroupPtrs W;
  memset(&W, 0, sizeof(W));
  const void* b13[kMaxGroups];
  const void* b2[kMaxGroups];
  for (int g = 0; g < L.Ng; ++g) {
    NEED(w13q[g]); NEED(w2q[g]); NEED(w13_scale[g]); NEED(w2_scale[g]);
    W.w13[g] = w13q[g];
    W.w2[g] = w2q[g];
    b13[g] = w13_scale[g];
    b2[g] = w2_scale[g];
  }
  if (workspace_bytes < ffn_workspace_bytes(L, cfg->dtype)) {
    set_error("expert_ffn_w4 workspace: %zu bytes given, %zu needed", workspace_bytes,
              ffn_workspace_bytes(L, cfg->dtype));
    return MOHGE_EWORKSPACE;
  }
  if (L.T == 0) return MOHGE_OK;
  return hip_rc(launch_expert_ffn_w4(L, x, perm, offsets, W, b13, b2, y_perm, workspace, (hipStream_t)stream),
                "mohge_expert_ffn_w4");
}

int mohge_mxfp4_decode(const void* packed, const void* scales, float* out, size_t n, void* stream) {
  if (n == 0) return MOHGE_OK;
  if (n % 32) { set_error("mohge_mxfp4_decode: n = %zu is not a multiple of the block size 32", n); return MOHGE_EINVAL; }
  NEED(packed); NEED(scales); NEED(out);
  return hip_rc(launch_mxfp4_decode(packed, scales, out, (long long)n, (hipStream_t)stream), "mohge_mxfp4_decode");
}

int mohge_expert_ffn_up(const mohge_config* cfg, const void* x, const int32_t* perm,
                        const int32_t* offsets, const void* const* w13, void* h, size_t h_bytes,
                        void* stream) {
  LayerDesc L;
  int rc = check_config(cfg, &L);
  if (rc) return rc;
  NEED(x); OPT(perm); NEED(offsets); NEED(h);
  if (!w13) { set_error("w13 pointer table is NULL"); return MOHGE_ENULL; }
  GroupPtrs W;
  memset(&W, 0, sizeof(W));
  for (int g = 0; g < L.Ng; ++g) { NEED(w13[g]); W.w13[g] = w13[g]; }
  if (h_bytes < ffn_workspace_bytes(L, cfg->dtype)) {
    set_error("expert_ffn_up: h has %zu bytes, %zu needed", h_bytes, ffn_workspace_bytes(L, cfg->dtype));
    return MOHGE_EWORKSPACE;
  }
  if (L.T == 0) return MOHGE_OK;
  return hip_rc(launch_expert_ffn(L, cfg->dtype, x, perm, offsets, W, nullptr, h,
                                  (hipStream_t)stream, 1),
                "mohge_expert_ffn_up");
}

int mohge_expert_ffn_down(const mohge_config* cfg, const void* h, size_t h_bytes, const int32_t* offsets,
                          const void* const* w2, void* y_perm, void* stream) {
  LayerDesc L;
  int rc = check_config(cfg, &L);
  if (rc) return rc;
  NEED(h); NEED(offsets); NEED(y_perm);
  if (!w2) { set_error("w2 pointer table is NULL"); return MOHGE_ENULL; }
  GroupPtrs W;
  memset(&W, 0, sizeof(W));
  for (int g = 0; g < L.Ng; ++g) { NEED(w2[g]); W.w2[g] = w2[g]; }
  if (h_bytes < ffn_workspace_bytes(L, cfg->dtype)) {
    set_error("expert_ffn_down: h has %zu bytes, %zu needed", h_bytes, ffn_workspace_bytes(L, cfg->dtype));
    return MOHGE_EWORKSPACE;
  }
  if (L.T == 0) return MOHGE_OK;
  return hip_rc(launch_expert_ffn(L, cfg->dtype, nullptr, nullptr, offsets, W, y_perm,
                                  const_cast<void*>(h), (hipStream_t)stream, 2),
                "mohge_expert_ffn_down");
}

int mohge_combine(const mohge_config* cfg, const void* y_perm, const int32_t* inv_perm,
                  const float* gates, void* y, void* stream) {
  LayerDesc L;
  int rc = check_config(cfg, &L);
  if (rc) return rc;
  NEED(y_perm); NEED(inv_perm); NEED(gates); NEED(y);
  if (L.T == 0) return MOHGE_OK;
  return hip_rc(launch_combine(L, cfg->dtype, y_perm, inv_perm, gates, nullptr, y, (hipStream_t)stream),
                "mohge_combine");
}

int mohge_combine_add(const mohge_config* cfg, const void* y_perm, const int32_t* inv_perm,
                      const float* gates, const void* y_add, void* y, void* stream) {
  LayerDesc L;
  int rc = check_config(cfg, &L);
  if (rc) return rc;
  NEED(y_perm); NEED(inv_perm); NEED(gates); NEED(y_add); NEED(y);
  if (L.T == 0) return MOHGE_OK;
  return hip_rc(launch_combine(L, cfg->dtype, y_perm, inv_perm, gates, y_add, y, (hipStream_t)stream),
                "mohge_combine_add");
}

int mohge_shared_routing(const mohge_config* cfg, int32_t* expert_idx, float* gates, int32_t* counts,
                         int32_t* offsets, int32_t* perm, int32_t* inv_perm, void* stream) {
  LayerDesc L;
  int rc = check_config(cfg, &L);
  if (rc) return rc;
  if (L.Ng != 1 || L.Kg != 1 || L.Ke != L.N) {
    set_error("shared routing needs n_groups = k_groups = 1 and k_experts = experts_per_group");
    return MOHGE_EINVAL;
  }
  NEED(expert_idx); NEED(gates); NEED(counts); NEED(offsets); NEED(perm); NEED(inv_perm);
  if (L.T == 0) return MOHGE_OK;
  return hip_rc(launch_shared_routing(L, expert_idx, gates, counts, offsets, perm, inv_perm,
                                      (hipStream_t)stream),
                "mohge_shared_routing");
}

int mohge_aux_loss(const mohge_config* cfg, const float* gs, const float* es1,
                   const int32_t* group_idx, const int32_t* expert_idx, float* losses,
                   float* stats, void* workspace, size_t workspace_bytes, void* stream) {
  LayerDesc L;
  int rc = check_config(cfg, &L);
  if (rc) return rc;
  NEED(gs); NEED(es1); NEED(group_idx); NEED(expert_idx); NEED(losses); OPT(stats);
  NEED(workspace);
  if (L.T < 1) { set_error("aux_loss needs T >= 1"); return MOHGE_EINVAL; }
  if (workspace_bytes < aux_workspace_bytes(L)) {
    set_error("aux_loss workspace: %zu bytes given, %zu needed", workspace_bytes,
              aux_workspace_bytes(L));
    return MOHGE_EWORKSPACE;
  }
  return hip_rc(launch_aux_loss(L, *cfg, gs, es1, group_idx, expert_idx, losses, stats, workspace,
                                (hipStream_t)stream),
                "mohge_aux_loss");
}

// ---- training -------------------------------------------------------------------------

#define PTR_TABLE(dst, src, name)                                              \
  do {                                                                         \
    if (!(src)) { set_error(name " pointer table is NULL"); return MOHGE_ENULL; } \
    for (int g_ = 0; g_ < L.Ng; ++g_) { NEED((src)[g_]); (dst)[g_] = (src)[g_]; }  \
  } while (0)

int mohge_expert_ffn_train(const mohge_config* cfg, const void* x, const int32_t* perm,
                           const int32_t* offsets, const void* const* w13, const void* const* w2,
                           void* y_perm, void* saved, size_t saved_bytes, void* stream) {
  LayerDesc L;
  int rc = check_config(cfg, &L);
  if (rc) return rc;
  if ((rc = need_bf16(cfg, "mohge_expert_ffn_train"))) return rc;
  NEED(x); OPT(perm); NEED(offsets); NEED(y_perm); NEED(saved);
  GroupPtrs W;
  memset(&W, 0, sizeof(W));
  PTR_TABLE(W.w13, w13, "w13");
  PTR_TABLE(W.w2, w2, "w2");
  if (saved_bytes < ffn_saved_bytes(L)) {
    set_error("expert_ffn_train: saved has %zu bytes, %zu needed", saved_bytes, ffn_saved_bytes(L));
    return MOHGE_EWORKSPACE;
  }
  if (L.T == 0) return MOHGE_OK;
  return hip_rc(launch_expert_ffn_train(L, x, perm, offsets, W, y_perm, saved, (hipStream_t)stream),
                "mohge_expert_ffn_train");
}

int mohge_combine_bwd(const mohge_config* cfg, const void* dy, const void* y_perm,
                      const int32_t* inv_perm, const float* gates, float* dgates, void* dy_perm,
                      void* stream) {
  LayerDesc L;
  int rc = check_config(cfg, &L);
  if (rc) return rc;
  if ((rc = need_bf16(cfg, "mohge_combine_bwd"))) return rc;
  NEED(dy); NEED(y_perm); NEED(inv_perm); NEED(gates); NEED(dgates); NEED(dy_perm);
  if (L.T == 0) return MOHGE_OK;
  return hip_rc(launch_combine_bwd(L, dy, y_perm, inv_perm, gates, dgates, dy_perm, (hipStream_t)stream),
                "mohge_combine_bwd");
}

int mohge_expert_ffn_bwd(const mohge_config* cfg, const void* x, const int32_t* perm,
                         const int32_t* offsets, const void* const* w13, const void* const* w2,
                         const void* saved, const void* dy_perm, void* dx_perm, void* const* dw13,
                         void* const* dw2, void* workspace, size_t workspace_bytes, void* stream) {
  LayerDesc L;
  int rc = check_config(cfg, &L);
  if (rc) return rc;
  if ((rc = need_bf16(cfg, "mohge_expert_ffn_bwd"))) return rc;
  NEED(x); OPT(perm); NEED(offsets); NEED(saved); NEED(dy_perm); NEED(dx_perm); NEED(workspace);
  GroupPtrs W;
  memset(&W, 0, sizeof(W));
  void* g13[kMaxGroups];
  void* g2[kMaxGroups];
  PTR_TABLE(W.w13, w13, "w13");
  PTR_TABLE(W.w2, w2, "w2");
  PTR_TABLE(g13, dw13, "dw13");
  PTR_TABLE(g2, dw2, "dw2");
  if (workspace_bytes < ffn_bwd_workspace_bytes(L)) {
    set_error("expert_ffn_bwd workspace: %zu bytes given, %zu needed", workspace_bytes,
              ffn_bwd_workspace_bytes(L));
    return MOHGE_EWORKSPACE;
  }
  return hip_rc(launch_expert_ffn_bwd(L, x, perm, offsets, W, saved, dy_perm, dx_perm, g13, g2,
                                      workspace, (hipStream_t)stream),
                "mohge_expert_ffn_bwd");
}

int mohge_route_bwd(const mohge_config* cfg, const void* x, const float* w_group,
                    const float* w_expert, const float* gs, const float* es1,
                    const int32_t* group_idx, const int32_t* expert_idx, const float* gates,
                    const float* dgates, const float* stats, const void* dx_perm,
                    const int32_t* inv_perm, void* dx, float* dw_group, float* dw_expert,
                    float* dz_out, void* workspace, size_t workspace_bytes, void* stream) {
  LayerDesc L;
  int rc = check_config(cfg, &L);
  if (rc) return rc;
  if ((rc = need_bf16(cfg, "mohge_route_bwd"))) return rc;
  NEED(x); NEED(w_group); NEED(w_expert); NEED(gs); NEED(es1); NEED(group_idx); NEED(expert_idx);
  NEED(gates); NEED(dgates); OPT(stats); OPT(dx_perm); OPT(inv_perm); NEED(dx); NEED(dw_group);
  NEED(dw_expert); OPT(dz_out); NEED(workspace);
  if (dx_perm && !inv_perm) { set_error("dx_perm given but inv_perm is NULL"); return MOHGE_ENULL; }
  if (L.T < 1) { set_error("route_bwd needs T >= 1"); return MOHGE_EINVAL; }
  if (workspace_bytes < route_bwd_workspace_bytes(L)) {
    set_error("route_bwd workspace: %zu bytes given, %zu needed", workspace_bytes,
              route_bwd_workspace_bytes(L));
    return MOHGE_EWORKSPACE;
  }
  return hip_rc(launch_route_bwd(L, *cfg, x, w_group, w_expert, gs, es1, group_idx, expert_idx, gates,
                                 dgates, stats, dx_perm, inv_perm, dx, dw_group, dw_expert, dz_out,
                                 workspace, (hipStream_t)stream),
                "mohge_route_bwd");
}

}  // extern "C"
