/*
 * mohge.h — C boundary of the MI355X (gfx950) implementation of one MoHGE layer
 * (Mixture of Heterogeneous Grouped Experts): forward pass on one GPU's share of
 * the experts, the two auxiliary losses of the training variant, and the backward pass.
 *
 * Notation follows the paper (section 3):
 *   T    tokens in the call,            d    hidden size,
 *   N_g  expert groups,                 N    experts per group (held by this GPU),
 *   N_e = N_g*N experts, expert e = g*N + i (group-major, 0-based),
 *   F_g  SwiGLU intermediate width of every expert of group g (section 3.1),
 *   K_g  groups kept per token (3.2.1), K_e experts kept per token (3.2.2),
 *   P = T*K_e (token, slot) pairs, pair p = t*K_e + slot.
 *
 * Conventions for every call
 *   - Returns MOHGE_OK (0) or a negative error code; mohge_last_error() gives the
 *     message of the last failing call on the calling thread.
 *   - "DEVICE" pointers are device memory owned by the caller; the library never
 *     allocates, frees or keeps them.  "HOST" pointers are read during the call only.
 *   - DEVICE pointers must be 16-byte aligned (MOHGE_EALIGN otherwise).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     only enqueue kernels: no host synchronisation, no device-to-host copy.  The
 *     tile schedules of the expert networks are derived on the device from `offsets`.
 *   - Activations and expert weights are fp32 or bf16 as `dtype` says; router
 *     weights, gates, scores and losses are always fp32; indices are int32.
 *   - All matrices are row-major with the innermost (reduction) dimension contiguous.
 *   - Limits: 1 <= N_g <= 16, N_e <= 256, d % 64 == 0, F_g % 64 == 0, T*K_e < 2^31.
 *     With the All-size Group-decoupling Allocation (section 3.4.1) a GPU holds the
 *     same expert indices i of every group, so its share is itself an N_g x N layer
 *     and `experts_per_group` is the local count.
 */
#ifndef MOHGE_H
#define MOHGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  MOHGE_OK = 0,
  MOHGE_EINVAL = -1,      /* configuration outside the documented limits            */
  MOHGE_ENULL = -2,       /* a required pointer is NULL                             */
  MOHGE_EALIGN = -3,      /* a device pointer is not 16-byte aligned                */
  MOHGE_EWORKSPACE = -4,  /* workspace smaller than mohge_workspace_size()          */
  MOHGE_EHIP = -5,        /* the HIP runtime reported an error at launch            */
  MOHGE_ETIMEOUT = -6     /* mohge_fused_status: a tile gave up waiting for the tiles it depends on */
};

enum { MOHGE_SELECT_GLOBAL = 0, MOHGE_SELECT_PER_GROUP = 1 };
enum { MOHGE_F32 = 0, MOHGE_BF16 = 1 };
enum {
  MOHGE_CALL_PERMUTE = 0, MOHGE_CALL_EXPERT_FFN = 1, MOHGE_CALL_AUX_LOSS = 2,
  MOHGE_CALL_FFN_SAVED = 3,       /* `saved` of mohge_expert_ffn_train                      */
  MOHGE_CALL_EXPERT_FFN_BWD = 4, MOHGE_CALL_ROUTE_BWD = 5,
  MOHGE_CALL_ROUTE = 6,           /* optional workspace of mohge_route (0 when it has no use) */
  MOHGE_CALL_DECODE_LAYER = 7     /* workspace of mohge_decode_layer                          */
};

typedef struct mohge_config {
  int32_t T;                  /* tokens                                              */
  int32_t d;                  /* hidden size                                         */
  int32_t n_groups;           /* N_g                                                 */
  int32_t experts_per_group;  /* N                                                   */
  const int32_t* d_ff;        /* HOST [N_g]: F_g                                     */
  int32_t k_groups;           /* K_g, 1..N_g                                         */
  int32_t k_experts;          /* K_e, 1..K_g*N                                       */
  int32_t select_mode;        /* MOHGE_SELECT_GLOBAL: K_e best ES'' over all kept
                                 groups (section 3.2.2, step 2);
                                 MOHGE_SELECT_PER_GROUP: K_e/K_g best in each kept
                                 group (K_e % K_g == 0, K_e/K_g <= N)               */
  int32_t dtype;              /* MOHGE_F32 or MOHGE_BF16: x, expert weights, y       */
  float alpha_g;              /* coefficient of L_G                                  */
  float alpha_e;              /* coefficient of L_E                                  */
  float eps;                  /* epsilon in the denominator of S^E (section 3.4.2)   */
  int32_t aux_freq_norm;      /* 1: routing frequencies f carry 1/T; 0: as printed   */
} mohge_config;

/*
 * Two-level router (section 3.2).
 *   GS_{g,t}  = sigmoid(x_t . w_group[g])                          (3.2.1)
 *   kept groups = the K_g largest (taken on the logit; ties to the lowest g)
 *   ES'_{g,i,t} = softmax_i(x_t . w_expert[g*N+i] + bias) for kept g, else 0   (3.2.2 step 1)
 *   ES'' = ES' * GS; kept experts per select_mode (ties to the lowest e)       (step 2)
 *   gates = kept ES'' / sum of kept ES''                                        (step 3)
 * In:  x DEVICE [T,d] (dtype), w_group DEVICE [N_g,d] f32, w_expert DEVICE [N_e,d]
 *      f32, expert_logit_bias DEVICE [N_e] f32 or NULL.
 * Out: group_idx DEVICE [T,K_g] and expert_idx DEVICE [T,K_e], ascending ids;
 *      gates DEVICE [T,K_e] aligned with expert_idx; gs_out DEVICE [T,N_g] (GS) and
 *      es1_out DEVICE [T,N_e] (ES', zero outside kept groups), each may be NULL.
 * Logits are accumulated in fp32 over 64 hidden elements at a time and in fp64 across those
 * slices (error about 1e-7).
 * workspace DEVICE, optional (NULL / 0 allowed), mohge_workspace_size(cfg, MOHGE_CALL_ROUTE) bytes
 * (0 where it has no use).  Without it the logits come from the fp32 matrix cores, one workgroup
 * per 16 tokens.  With it, two other forms are chosen by size: for few tokens (decode) the
 * reduction over d is spread over many workgroups, which leave partial sums there; from 8192
 * bf16 tokens on, the router rows are first split there into three bf16 parts that add up to the
 * fp32 weight exactly, and the logits come from the bf16 matrix cores with exact products.  The
 * logits of the forms can differ in the last bit (the fp64 partial sums are grouped
 * differently); each form is deterministic.
 */
int mohge_route(const mohge_config* cfg, const void* x, const float* w_group,
                const float* w_expert, const float* expert_logit_bias, int32_t* group_idx,
                int32_t* expert_idx, float* gates, float* gs_out, float* es1_out,
                void* workspace, size_t workspace_bytes, void* stream);

/*
 * Token permutation: buckets the P pairs by expert in stable order (expert id, then
 * pair id).  The paper implies dispatch without describing it; this is a stable
 * counting sort, deterministic (bit-identical from run to run).
 * In:  expert_idx DEVICE [T,K_e], values in [0, N_e).
 * Out: counts DEVICE [N_e]; offsets DEVICE [N_e+1] (exclusive prefix sum, last = P);
 *      perm DEVICE [P], perm[r] = p; inv_perm DEVICE [P], inv_perm[p] = r.
 *      If x_perm != NULL (then x must be given): x_perm DEVICE [P,d] (dtype),
 *      x_perm[r,:] = x[perm[r] / K_e, :].
 * workspace DEVICE, at least mohge_workspace_size(cfg, MOHGE_CALL_PERMUTE) bytes.
 */
int mohge_permute(const mohge_config* cfg, const int32_t* expert_idx, int32_t* counts,
                  int32_t* offsets, int32_t* perm, int32_t* inv_perm, const void* x,
                  void* x_perm, void* workspace, size_t workspace_bytes, void* stream);

/*
 * mohge_permute for callers that cannot allocate device memory or hand over a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same
 * arguments, kernels and results as mohge_permute, with the segment histograms (the call's only
 * scratch memory) in a static device array of MOHGE_PERMUTE_STATIC_BYTES inside the library,
 * which every GPU the library runs on holds until the process ends.  The call allocates and
 * frees nothing.  MOHGE_EWORKSPACE when mohge_workspace_size(cfg, MOHGE_CALL_PERMUTE) exceeds
 * MOHGE_PERMUTE_STATIC_BYTES (at N_e = 64 that is beyond 2^21 pairs); nothing is enqueued then.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 * streams, two threads) race on it and must be serialised by the caller; calls in stream order
 * need no clearing in between (every cell that is read is overwritten first).
 */
#define MOHGE_PERMUTE_STATIC_BYTES (1u << 20)
int mohge_permute_static(const mohge_config* cfg, const int32_t* expert_idx, int32_t* counts,
                         int32_t* offsets, int32_t* perm, int32_t* inv_perm, const void* x,
                         void* x_perm, void* stream);

/*
 * Expert networks on the bucketed tokens (section 3.1: every expert of group g has
 * width F_g; the form is a SwiGLU feed-forward network without bias):
 *   for sorted position r in [offsets[e], offsets[e+1]), expert e = g*N + i:
 *     a = W_gate x_r, b = W_up x_r, h = a*sigmoid(a)*b, y_perm[r,:] = W_down h.
 * In:  x DEVICE (dtype): if perm != NULL, [T,d] and row r reads x[perm[r]/K_e,:]
 *      (gather fused into the operand load); if perm == NULL, [P,d] already permuted.
 *      offsets DEVICE [N_e+1] as written by mohge_permute.
 *      w13 HOST array [N_g] of DEVICE pointers; w13[g] is [N, 2*F_g, d]: for expert i
 *      rows 0..F_g-1 are W_gate, rows F_g..2F_g-1 are W_up.
 *      w2 HOST array [N_g] of DEVICE pointers; w2[g] is [N, d, F_g] (W_down).
 * Out: y_perm DEVICE [P,d] (dtype).
 * workspace DEVICE, at least mohge_workspace_size(cfg, MOHGE_CALL_EXPERT_FFN) bytes;
 * it holds h between the two projections.
 * bf16: products on the matrix cores with fp32 accumulation; h and y_perm are
 * rounded to bf16 once each.  fp32: plain fp32 arithmetic.
 * Residency: for bf16 and T > 32 both projections run as ONE persistent launch of one workgroup
 * per compute unit, in which the down-projection tiles of a row block wait until its
 * up-projection tiles are complete.  The tiles waited for are always in the hands of workgroups
 * that never wait themselves, so the launch finishes on a GPU of its own and also when another
 * process delays some of its workgroups; the wait is bounded all the same (about a second of
 * polling).  A tile whose wait expires writes NaN to its part of y_perm instead of a result and
 * leaves a flag that mohge_fused_status reports: a wrong number can never pass for a result.
 */
int mohge_expert_ffn(const mohge_config* cfg, const void* x, const int32_t* perm,
                     const int32_t* offsets, const void* const* w13, const void* const* w2,
                     void* y_perm, void* workspace, size_t workspace_bytes, void* stream);

/*
 * The two halves of mohge_expert_ffn as separate calls (same arguments, same kernels):
 * mohge_expert_ffn_up writes h = SiLU(W_gate x) * (W_up x) for every sorted position
 * into `h` (DEVICE, mohge_workspace_size(cfg, MOHGE_CALL_EXPERT_FFN) bytes; the layout
 * inside is the library's; MOHGE_EWORKSPACE if h_bytes is smaller, in either call);
 * mohge_expert_ffn_down reads it and writes y_perm.
 * mohge_expert_ffn(…, workspace) computes exactly up(…, workspace) followed by down(workspace, …)
 * (on the matrix-core path as one launch instead of two, with the same bits).
 */
int mohge_expert_ffn_up(const mohge_config* cfg, const void* x, const int32_t* perm,
                        const int32_t* offsets, const void* const* w13, void* h, size_t h_bytes,
                        void* stream);
int mohge_expert_ffn_down(const mohge_config* cfg, const void* h, size_t h_bytes, const int32_t* offsets,
                          const void* const* w2, void* y_perm, void* stream);

/*
 * Gated un-permute and combine (appendix, background: y = sum_i G_i(x) E_i(x)):
 *   y[t,:] = sum_{slot<K_e} gates[t,slot] * y_perm[inv_perm[t*K_e+slot], :]
 * accumulated in fp32 in slot order.
 * In:  y_perm DEVICE [P,d] (dtype), inv_perm DEVICE [P], gates DEVICE [T,K_e].
 * Out: y DEVICE [T,d] (dtype).
 */
int mohge_combine(const mohge_config* cfg, const void* y_perm, const int32_t* inv_perm,
                  const float* gates, void* y, void* stream);

/*
 * Shared experts.  The paper's architecture table lists N_s = 2 shared experts next to the
 * routed ones and its method text never mentions them; the reading taken here is the usual
 * one: experts every token goes through with weight 1, added to the routed output,
 *   y[t,:] = sum_{s<N_s} E^shared_s(x[t,:]) + sum_{kept e} gate * E_e(x[t,:]).
 * They are run with the calls above on a second configuration (n_groups = k_groups = 1,
 * experts_per_group = k_experts = N_s, d_ff = their width): mohge_shared_routing fills the
 * constant routing of that configuration once (expert_idx[t,s] = s, gates = 1, and the
 * permutation in which sorted position s*T + t is pair t*N_s + s), mohge_expert_ffn and
 * mohge_combine then give the shared term, and mohge_combine_add adds it to the gated sum:
 *   y[t,:] = y_add[t,:] + sum_slot gates[t,slot] * y_perm[inv_perm[t*K_e+slot], :]
 * (y_add DEVICE [T,d] (dtype); y_add == y is allowed).
 * Their backward pass needs no call of its own either: on the shared configuration,
 * mohge_combine_bwd with the constant gates turns dy into dy_perm, mohge_expert_ffn_bwd gives
 * dx_perm and the weight gradients, and mohge_combine_add adds the N_s rows of dx_perm of a
 * token to the routed part of dx.
 */
int mohge_shared_routing(const mohge_config* cfg, int32_t* expert_idx, float* gates, int32_t* counts,
                         int32_t* offsets, int32_t* perm, int32_t* inv_perm, void* stream);
int mohge_combine_add(const mohge_config* cfg, const void* y_perm, const int32_t* inv_perm,
                      const float* gates, const void* y_add, void* y, void* stream);

/*
 * Group-Wise Auxiliary Loss L_G (section 3.3) and Intra-Group Experts Auxiliary
 * Loss L_E (section 3.4.2) over the T tokens of the call:
 *   f^G_g = (N_g/K_g) * [1/T] * #{t : g kept},  p^G_g = (1/T) sum_t GS_{g,t}/sum_j GS_{j,t}
 *   L_G = alpha_g * sum_g (F_g / max F) f^G_g p^G_g
 *   f^E_e = (N/K_e) * [1/T] * #{t : e kept},
 *   p^E_e = (1/T) sum_t ES'_{e,t} / (sum_{j in group} ES'_{j,t} + eps)
 *   L_E = alpha_e * sum_e f^E_e p^E_e
 * ([1/T] present when aux_freq_norm != 0.)
 * In:  gs DEVICE [T,N_g], es1 DEVICE [T,N_e] (as written by mohge_route),
 *      group_idx DEVICE [T,K_g], expert_idx DEVICE [T,K_e].
 * Out: losses DEVICE [2] = (L_G, L_E); stats DEVICE [2*N_g + 2*N_e] = f^G, p^G, f^E,
 *      p^E, or NULL.
 * workspace DEVICE, at least mohge_workspace_size(cfg, MOHGE_CALL_AUX_LOSS) bytes.
 * Sums over tokens are taken in fp64 in a fixed order (deterministic).
 */
int mohge_aux_loss(const mohge_config* cfg, const float* gs, const float* es1,
                   const int32_t* group_idx, const int32_t* expert_idx, float* losses,
                   float* stats, void* workspace, size_t workspace_bytes, void* stream);

/*
 * mohge_expert_ffn for decode with quantised expert weights (not in the paper: halves the bytes
 * the memory-bound decode step streams).  w13q[g] DEVICE [N, 2*F_g, d] and w2q[g] DEVICE
 * [N, d, F_g] hold FP8 E4M3 codes (the OCP 8-bit format: 1 sign, 4 exponent bits with bias 7,
 * 3 mantissa bits, no infinities, S.1111.111 = NaN), one byte per element in the layout of
 * w13 / w2; w13_scale[g] DEVICE [N, 2*F_g] f32 and w2_scale[g] DEVICE [N, d] f32 hold one scale per
 * weight row: the weight is scale[row] * value(code).  x, H and y_perm stay bf16; the codes are
 * converted exactly to bf16 matrix-core operands, sums are fp32, the scale multiplies the sum.
 * Only for cfg->dtype == MOHGE_BF16 and T <= 32 (MOHGE_EINVAL otherwise).  workspace as for
 * mohge_expert_ffn.  mohge_fp8_decode converts n codes to f32 with the same hardware conversion
 * (DEVICE pointers), for checks and tools.
 */
int mohge_expert_ffn_w8(const mohge_config* cfg, const void* x, const int32_t* perm,
                        const int32_t* offsets, const void* const* w13q, const float* const* w13_scale,
                        const void* const* w2q, const float* const* w2_scale, void* y_perm,
                        void* workspace, size_t workspace_bytes, void* stream);
int mohge_fp8_decode(const void* codes, float* out, size_t n, void* stream);

/*
 * The same for weights in the MXFP4 microscaling format (OCP MX: elements are FP4 E2M1 codes,
 * 1 sign, 2 exponent bits with bias 1, 1 mantissa bit, magnitudes 0, 0.5, 1, 1.5, 2, 3, 4, 6;
 * every block of 32 consecutive elements of a weight row shares one E8M0 scale 2^(code - 127)).
 * w13q[g] DEVICE [N, 2*F_g, d/2] and w2q[g] DEVICE [N, d, F_g/2] bytes: two codes per byte, the
 * element with the even index in the low four bits; 16-byte aligned.  w13_scale[g] DEVICE
 * [N, 2*F_g, d/32] and w2_scale[g] DEVICE [N, d, F_g/32] bytes (16-byte aligned like every
 * device pointer): the scale codes.  The weight is scale(block) * value(code), formed as a bf16 matrix-core operand: exact
 * whenever the product lies in bf16's normal range, which scale codes 2..252 guarantee (beyond
 * them small products may lose their value and large ones overflow; code 255 is NaN); sums are
 * fp32.  Same restrictions, workspace and error behaviour as mohge_expert_ffn_w8.
 * mohge_mxfp4_decode converts n elements (n a multiple of 32, else MOHGE_EINVAL; packed = n/2
 * bytes, 16-byte aligned; scales = n/32 bytes; DEVICE pointers) to f32 with the same conversion.
 */
int mohge_expert_ffn_w4(const mohge_config* cfg, const void* x, const int32_t* perm,
                        const int32_t* offsets, const void* const* w13q, const void* const* w13_scale,
                        const void* const* w2q, const void* const* w2_scale, void* y_perm,
                        void* workspace, size_t workspace_bytes, void* stream);
int mohge_mxfp4_decode(const void* packed, const void* scales, float* out, size_t n, void* stream);

/*
 * The whole layer for a decode-sized call as ONE launch (not in the paper, which gives no kernel
 * design: at a handful of tokens the layer is bound by streaming the touched experts' weights, and
 * the gaps between five dependent launches are a measurable share of the step):
 *     y = mohge_combine(mohge_expert_ffn(x, mohge_permute(mohge_route(x))))
 * with the definitions of those calls (sections 3.2.1, 3.2.2 and 3.1 of the paper; appendix,
 * first equation).  The pieces of work (partial logits, selection + permutation, units of the up
 * and of the down projection, the gated sums) are workgroups of one grid that wait for each other
 * through counters in the workspace; every wait is bounded.
 * Only for cfg->dtype == MOHGE_BF16, T <= 32 and T*K_e <= 2048 (MOHGE_EINVAL otherwise).
 * In:  x DEVICE [T,d] bf16; w_group DEVICE [N_g,d] f32; w_expert DEVICE [N_e,d] f32;
 *      expert_logit_bias DEVICE [N_e] f32 or NULL; w13 / w2 HOST [N_g] of DEVICE pointers as for
 *      mohge_expert_ffn.
 * Out: y DEVICE [T,d] bf16; group_idx DEVICE [T,K_g], expert_idx DEVICE [T,K_e], gates DEVICE
 *      [T,K_e] as mohge_route writes them.  The logits are those of the router's split form up to
 *      the grouping of the fp64 partial sums; given equal routing, y is bit-identical to the four
 *      separate calls.
 * workspace DEVICE, mohge_workspace_size(cfg, MOHGE_CALL_DECODE_LAYER) bytes.  Its first
 * mohge_decode_layer_ctl_bytes(cfg) bytes hold the counters: they MUST BE ZERO when the call
 * starts and the call leaves them zero, so a workspace cleared once (hipMemset) serves any number
 * of calls issued in stream order; calls that overlap on one workspace race.  If the counters
 * are not zero at the start, or a wait expires, nothing hangs: y is overwritten with NaN and
 * mohge_fused_status(cfg, MOHGE_CALL_DECODE_LAYER, workspace, ...) reports MOHGE_EINVAL or
 * MOHGE_ETIMEOUT.
 */
int mohge_decode_layer(const mohge_config* cfg, const void* x, const float* w_group,
                       const float* w_expert, const float* expert_logit_bias,
                       const void* const* w13, const void* const* w2, int32_t* group_idx,
                       int32_t* expert_idx, float* gates, void* y, void* workspace,
                       size_t workspace_bytes, void* stream);
size_t mohge_decode_layer_ctl_bytes(const mohge_config* cfg);

/*
 * ---- Training: backward pass of the layer (dtype MOHGE_BF16 only; MOHGE_EINVAL otherwise) ----
 *
 * The paper trains the layer with  L_task + L_G + L_E  (sections 3.3, 3.4.2) and prints no
 * backward formulas; these calls apply the chain rule to the forward definitions of section
 * 3.2 and of the two losses.  The routing decisions and the routing frequencies f are
 * constants.  Given dy = dL_task/dy, one backward pass is
 *     mohge_combine_bwd -> mohge_expert_ffn_bwd -> mohge_route_bwd
 * after a forward pass that used mohge_expert_ffn_train in place of mohge_expert_ffn and kept
 * gs, es1, gates, the indices and the permutation.  Gradients of bf16 tensors are bf16 (one
 * rounding of an fp32 accumulator); router gradients are fp32.
 */

/*
 * mohge_expert_ffn with the same results, which additionally keeps, in `saved` (DEVICE,
 * mohge_workspace_size(cfg, MOHGE_CALL_FFN_SAVED) bytes, layout the library's), the hidden
 * activations h and, with a = W_gate x, b = W_up x, the two factors b*SiLU'(a) and SiLU(a) that turn
 * dh into (da, db) (all bf16) of every routed row.
 * Uses the matrix-core tile path for every T.
 */
int mohge_expert_ffn_train(const mohge_config* cfg, const void* x, const int32_t* perm,
                           const int32_t* offsets, const void* const* w13, const void* const* w2,
                           void* y_perm, void* saved, size_t saved_bytes, void* stream);

/*
 * Backward of mohge_combine:
 *   dgates[t,slot] = <dy[t,:], y_perm[inv_perm[t*K_e+slot],:]>   (fp32, fixed summation order)
 *   dy_perm[inv_perm[t*K_e+slot],:] = gates[t,slot] * dy[t,:]
 * In:  dy DEVICE [T,d], y_perm DEVICE [P,d] (the forward's), inv_perm DEVICE [P], gates DEVICE [T,K_e].
 * Out: dgates DEVICE [T,K_e] f32, dy_perm DEVICE [P,d].
 */
int mohge_combine_bwd(const mohge_config* cfg, const void* dy, const void* y_perm,
                      const int32_t* inv_perm, const float* gates, float* dgates, void* dy_perm,
                      void* stream);

/*
 * Backward of the expert networks.  For every routed row r of expert e, with s = sigmoid(a):
 *   dh = W_down^T dy_perm[r],  da = dh*b*s*(1 + a*(1-s)),  db = dh*a*s,
 *   dx_perm[r] = W_gate^T da + W_up^T db,
 *   dw2[e] = sum_r dy_perm[r] h_r^T,  dw13[e] = sum_r [da; db] x_r^T   (zero for an expert without rows).
 * In:  x, perm, offsets, w13, w2 as for mohge_expert_ffn (the weights are read in
 *      that layout, no transposed copies are needed); saved as written by
 *      mohge_expert_ffn_train for the same x / perm / offsets / weights; dy_perm DEVICE [P,d].
 * Out: dx_perm DEVICE [P,d]; dw13 HOST array [N_g] of DEVICE pointers, dw13[g] [N, 2*F_g, d]
 *      (gate rows, then up rows, as w13); dw2[g] DEVICE [N, d, F_g].  Overwritten, not accumulated.
 * workspace DEVICE, at least mohge_workspace_size(cfg, MOHGE_CALL_EXPERT_FFN_BWD) bytes.
 * h, the two stored factors, dh and [da|db] pass through bf16 once each; products accumulate in fp32.
 */
int mohge_expert_ffn_bwd(const mohge_config* cfg, const void* x, const int32_t* perm,
                         const int32_t* offsets, const void* const* w13, const void* const* w2,
                         const void* saved, const void* dy_perm, void* dx_perm, void* const* dw13,
                         void* const* dw2, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Backward of mohge_route plus the router gradients of L_G and L_E, and the assembly of dx.
 * Per token, with u_g = alpha_g (F_g/max F) f^G_g / T, v_e = alpha_e f^E_e / T,
 * S = sum_g GS_g, sigma_g = sum_i ES'_{g,i}, D = sum_kept ES'':
 *   dES''_e = (dgate_e - sum_kept dgate*gate) / D                        kept experts, else 0
 *   dES'_e  = dES''_e GS_g + v_e/(sigma_g+eps) - sum_i v_i ES'_i/(sigma_g+eps)^2     kept groups
 *   dGS_g   = sum_i dES''_{g,i} ES'_{g,i} + (u_g - sum_j u_j GS_j/S)/S               all groups
 *   dzE_e = ES'_e (dES'_e - sum_i dES'_i ES'_i),  dzG_g = dGS_g GS_g (1-GS_g)
 *   dw_group = dzG^T x,  dw_expert = dzE^T x,
 *   dx[t] = sum_slot dx_perm[inv_perm[t*K_e+slot]] + dzG_t w_group + dzE_t w_expert.
 * In:  x DEVICE [T,d]; w_group, w_expert; gs, es1, group_idx, expert_idx, gates as written by
 *      mohge_route; dgates DEVICE [T,K_e]; stats DEVICE as written by mohge_aux_loss (f^G and
 *      f^E are read), or NULL to leave the auxiliary losses out; dx_perm DEVICE [P,d] and
 *      inv_perm DEVICE [P], or both NULL to get the router's part of dx alone.
 * Out: dx DEVICE [T,d] (bf16); dw_group DEVICE [N_g,d] f32; dw_expert DEVICE [N_e,d] f32;
 *      dz_out DEVICE [T, N_g+N_e] f32 (dzG then dzE per token; dzE is also the gradient of the
 *      expert logit bias per token) or NULL.
 * workspace DEVICE, at least mohge_workspace_size(cfg, MOHGE_CALL_ROUTE_BWD) bytes.
 * Sums over tokens use a fixed order (deterministic).
 */
int mohge_route_bwd(const mohge_config* cfg, const void* x, const float* w_group,
                    const float* w_expert, const float* gs, const float* es1,
                    const int32_t* group_idx, const int32_t* expert_idx, const float* gates,
                    const float* dgates, const float* stats, const void* dx_perm,
                    const int32_t* inv_perm, void* dx, float* dw_group, float* dw_expert,
                    float* dz_out, void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of DEVICE workspace that call `which_call` (MOHGE_CALL_*) needs for `cfg`;
 * 0 for an invalid configuration or call id. */
size_t mohge_workspace_size(const mohge_config* cfg, int which_call);

/*
 * Diagnostic for the launches that run two dependent tile lists at once (the fused forms of
 * mohge_expert_ffn, mohge_expert_ffn_train and mohge_expert_ffn_bwd): a tile of the second list
 * waits, for a bounded number of polls, until the tiles it depends on are complete; the design
 * guarantees they are already running, and a tile that gives up all the same writes NaN to its
 * output region and leaves a flag in the workspace.  This call SYNCHRONISES `stream`, reads the flag left by the
 * last call of `which_call` (MOHGE_CALL_EXPERT_FFN, MOHGE_CALL_FFN_SAVED,
 * MOHGE_CALL_EXPERT_FFN_BWD or MOHGE_CALL_DECODE_LAYER) on `workspace` (DEVICE; for
 * MOHGE_CALL_FFN_SAVED the `saved` buffer) and returns MOHGE_OK, or MOHGE_ETIMEOUT when that
 * call's output holds NaN (MOHGE_CALL_DECODE_LAYER: also MOHGE_EINVAL when the counters in the
 * workspace were not zero at the start).
 * MOHGE_OK at once where the call has no such launch for cfg (fp32, decode sizes).
 */
int mohge_fused_status(const mohge_config* cfg, int which_call, const void* workspace,
                       size_t workspace_bytes, void* stream);

/* Message of the last error on this thread ("" if none); valid until the next call. */
const char* mohge_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* MOHGE_H */
