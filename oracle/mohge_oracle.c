/*
 * CPU oracle for the forward pass of one MoHGE layer (Mixture of Heterogeneous
 * Grouped Experts) and its two auxiliary losses.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It exists so that the HIP
 * library can be checked against the paper's definitions.  Only tests, the smoke
 * check and the benchmark's "cpu_baseline" leg may call it.  It shares no code,
 * header, table or helper with the HIP library and must never be used as a
 * fallback for it.
 *
 * Every function is the paper's definition written out: plain loops, one token
 * (or one token/expert pair) at a time, all arithmetic in double.  Inputs are
 * float arrays holding exactly the values the GPU sees (bf16 storage is widened
 * to float by the caller, which is exact).  No blocking, fusion or reordering.
 * OpenMP, when enabled, only distributes independent tokens / pairs over threads.
 *
 * Notation (paper, section 3): T tokens, hidden size d, N_g groups of N experts,
 * expert e = g*N + i, per-group expert width F_g, K_g groups and K_e experts kept
 * per token.
 *
 * Readings taken where the paper leaves a choice (each is listed with its reason
 * in the design notes of this repository):
 *  - the group "centroid embedding" e_g is its own parameter W_G[N_g, d];
 *  - top-K_g is taken on the logit x.e_g: sigmoid is increasing, so this is the
 *    set section 3.2.1 defines, without sigmoid rounding deciding near-ties;
 *  - select_mode 0 keeps the K_e largest ES'' over all selected groups (the
 *    "Experts for Global Selection" step); select_mode 1 keeps K_e/K_g experts in
 *    every selected group (inside one group ES'' is increasing in the logit, so
 *    the key is the logit).  Gates are always ES'' over the sum of kept ES'';
 *  - ties go to the lowest index; kept ids are reported in ascending order;
 *  - experts are SwiGLU feed-forward networks without bias:
 *        E(x) = W_down ( SiLU(W_gate x) * (W_up x) ),  SiLU(z) = z / (1 + exp(-z));
 *  - the layer output is y_t = sum over kept experts of gate * E(x_t)
 *    (appendix, background, first equation);
 *  - in both auxiliary losses the frequency f counts actual routing decisions and
 *    carries 1/T when aux_freq_norm != 0 (the printed formulas omit it while
 *    calling f a frequency; aux_freq_norm == 0 is the printed form, T times larger);
 *  - W_i / W_max in the group-wise loss is F_i / max_j F_j.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct oracle_config {
  int32_t T, d;
  int32_t n_groups;        /* N_g */
  int32_t n_per_group;     /* N   */
  const int32_t* d_ff;     /* [N_g] F_g */
  int32_t k_groups;        /* K_g */
  int32_t k_experts;       /* K_e */
  int32_t select_mode;     /* 0 global, 1 per group */
  int32_t aux_freq_norm;   /* 1: f carries 1/T */
  double alpha_g, alpha_e, eps;
} oracle_config;

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

static int config_ok(const oracle_config* c) {
  if (!c || !c->d_ff) return 0;
  if (c->T < 0 || c->d < 1 || c->n_groups < 1 || c->n_per_group < 1) return 0;
  if (c->k_groups < 1 || c->k_groups > c->n_groups) return 0;
  if (c->k_experts < 1 || c->k_experts > c->k_groups * c->n_per_group) return 0;
  if (c->select_mode == 1) {
    if (c->k_experts % c->k_groups) return 0;
    if (c->k_experts / c->k_groups > c->n_per_group) return 0;
  } else if (c->select_mode != 0) {
    return 0;
  }
  return 1;
}

static double dot_fd(const float* a, const float* b, int n) {
  double s = 0.0;
  for (int k = 0; k < n; ++k) s += (double)a[k] * (double)b[k];
  return s;
}

/* Pick the `k` largest of key[idx] over the candidates with cand[idx] != 0,
 * largest first, strict comparison so that the lowest index wins a tie.
 * Sets sel[idx] = 1 for the picks.  Returns (smallest kept key) - (largest
 * rejected key), or +inf when nothing is rejected. */
static double pick_top(const double* key, const char* cand, int n, int k, char* sel) {
  double kept_min = INFINITY;
  for (int r = 0; r < k; ++r) {
    int best = -1;
    for (int j = 0; j < n; ++j) {
      if (!cand[j] || sel[j]) continue;
      if (best < 0 || key[j] > key[best]) best = j;
    }
    sel[best] = 1;
    kept_min = key[best];
  }
  double rej_max = -INFINITY;
  for (int j = 0; j < n; ++j)
    if (cand[j] && !sel[j] && key[j] > rej_max) rej_max = key[j];
  return (rej_max == -INFINITY) ? INFINITY : kept_min - rej_max;
}

/* Section 3.2 for one token.  Scratch arrays are sized by the caller. */
static void route_token(const oracle_config* c, const float* x_t, const float* w_group,
                        const float* w_expert, const float* bias, int32_t* gidx,
                        int32_t* eidx, double* gate, double* gs_row, double* es1_row,
                        double* margin, double* zG, double* GS, double* zE, double* ES1,
                        double* ES2, char* gsel, char* cand, char* esel) {
  const int Ng = c->n_groups, N = c->n_per_group, Ne = Ng * N, d = c->d;
  double m = INFINITY;

  /* Group gating model: GS_g = Sigmoid(x . e_g); keep the K_g best groups. */
  for (int g = 0; g < Ng; ++g) {
    zG[g] = dot_fd(x_t, w_group + (size_t)g * d, d);
    GS[g] = 1.0 / (1.0 + exp(-zG[g]));
    gsel[g] = 0;
    cand[g] = 1;
  }
  double mg = pick_top(zG, cand, Ng, c->k_groups, gsel);
  if (mg < m) m = mg;

  /* Step 1: softmax over the experts of each kept group, zero elsewhere.
   * Step 2 (first half): scale by the group score. */
  for (int e = 0; e < Ne; ++e) { zE[e] = 0.0; ES1[e] = 0.0; ES2[e] = 0.0; esel[e] = 0; cand[e] = 0; }
  for (int g = 0; g < Ng; ++g) {
    if (!gsel[g]) continue;
    double mx = -INFINITY, sum = 0.0;
    for (int i = 0; i < N; ++i) {
      int e = g * N + i;
      zE[e] = dot_fd(x_t, w_expert + (size_t)e * d, d) + (bias ? (double)bias[e] : 0.0);
      if (zE[e] > mx) mx = zE[e];
      cand[e] = 1;
    }
    for (int i = 0; i < N; ++i) sum += exp(zE[g * N + i] - mx);
    for (int i = 0; i < N; ++i) {
      int e = g * N + i;
      ES1[e] = exp(zE[e] - mx) / sum;
      ES2[e] = ES1[e] * GS[g];
    }
  }

  /* Step 2 (second half): which experts are kept. */
  if (c->select_mode == 0) {
    double me = pick_top(ES2, cand, Ne, c->k_experts, esel);
    if (me < m) m = me;
  } else {
    const int k = c->k_experts / c->k_groups;
    for (int g = 0; g < Ng; ++g) {
      if (!gsel[g]) continue;
      double me = pick_top(zE + g * N, cand + g * N, N, k, esel + g * N);
      if (me < m) m = me;
    }
  }

  /* Step 3: divide the kept scores by their sum. */
  double D = 0.0;
  for (int e = 0; e < Ne; ++e) if (esel[e]) D += ES2[e];
  int s = 0;
  for (int g = 0; g < Ng; ++g) if (gsel[g]) gidx[s++] = g;
  s = 0;
  for (int e = 0; e < Ne; ++e) if (esel[e]) { eidx[s] = e; gate[s] = ES2[e] / D; ++s; }

  if (gs_row) for (int g = 0; g < Ng; ++g) gs_row[g] = GS[g];
  if (es1_row) for (int e = 0; e < Ne; ++e) es1_row[e] = ES1[e];
  if (margin) *margin = m;
}

/*
 * Two-level routing for all T tokens.
 *   x[T,d], w_group[N_g,d], w_expert[N_e,d], bias[N_e] or NULL (added to the
 *   expert logits before the softmax).
 *   group_idx[T,K_g], expert_idx[T,K_e] ascending ids; gates[T,K_e] aligned with
 *   expert_idx.  gs[T,N_g] (GS), es1[T,N_e] (ES', zero for unselected groups) and
 *   margin[T] may be NULL.  margin is the smallest (kept - rejected) key gap of
 *   any top-k decision the token went through: logit units for groups and for
 *   per-group expert choice, ES'' units for global expert choice.
 * Returns 0, or -1 for an invalid configuration.
 */
int oracle_route(const oracle_config* c, const float* x, const float* w_group,
                 const float* w_expert, const float* bias, int32_t* group_idx,
                 int32_t* expert_idx, double* gates, double* gs, double* es1,
                 double* margin) {
  if (!config_ok(c)) return -1;
  const int Ng = c->n_groups, Ne = Ng * c->n_per_group;
#pragma omp parallel
  {
    double* buf = (double*)malloc(sizeof(double) * (size_t)(2 * Ng + 3 * Ne));
    char* cbuf = (char*)malloc((size_t)(Ng + 2 * Ne) + (size_t)(Ng > Ne ? Ng : Ne));
    double *zG = buf, *GS = buf + Ng, *zE = buf + 2 * Ng, *ES1 = zE + Ne, *ES2 = ES1 + Ne;
    char *gsel = cbuf, *esel = cbuf + Ng, *cand = esel + Ne;
#pragma omp for schedule(static)
    for (int t = 0; t < c->T; ++t) {
      route_token(c, x + (size_t)t * c->d, w_group, w_expert, bias,
                  group_idx + (size_t)t * c->k_groups, expert_idx + (size_t)t * c->k_experts,
                  gates + (size_t)t * c->k_experts, gs ? gs + (size_t)t * Ng : NULL,
                  es1 ? es1 + (size_t)t * Ne : NULL, margin ? margin + t : NULL, zG, GS, zE,
                  ES1, ES2, gsel, cand, esel);
    }
    free(buf);
    free(cbuf);
  }
  return 0;
}

/*
 * Token permutation: the P = T*K_e (token, slot) pairs p = t*K_e + slot bucketed
 * by expert, in stable order (expert id, then p).
 *   counts[N_e], offsets[N_e+1] (exclusive prefix sum), perm[r] = p, inv_perm[p] = r.
 * The paper does not describe dispatch; this is the plain definition of a stable
 * bucket sort.
 */
int oracle_permute(const oracle_config* c, const int32_t* expert_idx, int32_t* counts,
                   int32_t* offsets, int32_t* perm, int32_t* inv_perm) {
  if (!config_ok(c)) return -1;
  const int Ne = c->n_groups * c->n_per_group;
  const int64_t P = (int64_t)c->T * c->k_experts;
  int32_t r = 0;
  for (int e = 0; e < Ne; ++e) {
    offsets[e] = r;
    for (int64_t p = 0; p < P; ++p)
      if (expert_idx[p] == e) { perm[r] = (int32_t)p; inv_perm[p] = r; ++r; }
    counts[e] = r - offsets[e];
  }
  offsets[Ne] = r;
  return (r == P) ? 0 : -2;
}

/*
 * Expert networks applied to a list of (token, expert) pairs.
 *   pair_token[n], pair_expert[n]; w_gate[g] / w_up[g] point to [N, F_g, d],
 *   w_down[g] to [N, d, F_g], all row-major.  y_pairs[n, d] = E_e(x_t).
 *   h_pairs (may be NULL) receives the hidden activation SiLU(a)*b, row stride
 *   h_stride >= max F_g.
 */
int oracle_expert_ffn(const oracle_config* c, const float* x, const float* const* w_gate,
                      const float* const* w_up, const float* const* w_down, int64_t n,
                      const int32_t* pair_token, const int32_t* pair_expert, double* y_pairs,
                      double* h_pairs, int64_t h_stride) {
  if (!config_ok(c)) return -1;
  const int d = c->d, N = c->n_per_group;
  int Fmax = 0;
  for (int g = 0; g < c->n_groups; ++g) if (c->d_ff[g] > Fmax) Fmax = c->d_ff[g];
#pragma omp parallel
  {
    double* h = (double*)malloc(sizeof(double) * (size_t)Fmax);
#pragma omp for schedule(dynamic, 1)
    for (int64_t q = 0; q < n; ++q) {
      const int e = pair_expert[q], g = e / N, i = e % N, F = c->d_ff[g];
      const float* x_t = x + (size_t)pair_token[q] * d;
      const float* Wg = w_gate[g] + (size_t)i * F * d;
      const float* Wu = w_up[g] + (size_t)i * F * d;
      const float* Wd = w_down[g] + (size_t)i * d * F;
      for (int j = 0; j < F; ++j) {
        double a = dot_fd(x_t, Wg + (size_t)j * d, d);
        double b = dot_fd(x_t, Wu + (size_t)j * d, d);
        h[j] = a / (1.0 + exp(-a)) * b;
      }
      if (h_pairs) for (int j = 0; j < F; ++j) h_pairs[q * h_stride + j] = h[j];
      double* y = y_pairs + (size_t)q * d;
      for (int k = 0; k < d; ++k) {
        const float* row = Wd + (size_t)k * F;
        double s = 0.0;
        for (int j = 0; j < F; ++j) s += (double)row[j] * h[j];
        y[k] = s;
      }
    }
    free(h);
  }
  return 0;
}

/*
 * Gated combine for n_tok tokens: y[q,:] = sum_slot gates[q,slot] * y_pairs[q*K_e+slot,:].
 */
int oracle_combine(const oracle_config* c, int64_t n_tok, const double* y_pairs,
                   const double* gates, double* y) {
  if (!config_ok(c)) return -1;
  const int d = c->d, Ke = c->k_experts;
  for (int64_t q = 0; q < n_tok; ++q)
    for (int k = 0; k < d; ++k) {
      double s = 0.0;
      for (int slot = 0; slot < Ke; ++slot)
        s += gates[q * Ke + slot] * y_pairs[((size_t)q * Ke + slot) * d + k];
      y[(size_t)q * d + k] = s;
    }
  return 0;
}

/*
 * Group-Wise Auxiliary Loss L_G (section 3.3) and Intra-Group Experts Auxiliary
 * Loss L_E (section 3.4.2) over the T tokens of the call.
 *   gs[T,N_g] = GS, es1[T,N_e] = ES' (zero rows for unselected groups).
 *   losses[0] = L_G, losses[1] = L_E.
 *   stats (may be NULL): f^G[N_g], p^G[N_g], f^E[N_e], p^E[N_e] in this order.
 */
int oracle_aux_loss(const oracle_config* c, const double* gs, const double* es1,
                    const int32_t* group_idx, const int32_t* expert_idx, double* losses,
                    double* stats) {
  if (!config_ok(c)) return -1;
  const int Ng = c->n_groups, N = c->n_per_group, Ne = Ng * N, T = c->T;
  double* fG = (double*)calloc((size_t)(2 * Ng + 2 * Ne), sizeof(double));
  double *pG = fG + Ng, *fE = pG + Ng, *pE = fE + Ne;
  double Fmax = 0.0;
  for (int g = 0; g < Ng; ++g) if (c->d_ff[g] > Fmax) Fmax = c->d_ff[g];
  const double fscale = c->aux_freq_norm ? 1.0 / (double)T : 1.0;

  for (int t = 0; t < T; ++t) {
    /* how often each group / expert was routed to */
    for (int s = 0; s < c->k_groups; ++s) fG[group_idx[(size_t)t * c->k_groups + s]] += 1.0;
    for (int s = 0; s < c->k_experts; ++s) fE[expert_idx[(size_t)t * c->k_experts + s]] += 1.0;
    /* s'_{g,t} = GS_{g,t} / sum_j GS_{j,t}, over all groups */
    double sg = 0.0;
    for (int g = 0; g < Ng; ++g) sg += gs[(size_t)t * Ng + g];
    for (int g = 0; g < Ng; ++g) pG[g] += gs[(size_t)t * Ng + g] / sg;
    /* S^E_{g,i,t} = ES'_{g,i,t} / (sum_j ES'_{g,j,t} + eps), inside each group */
    for (int g = 0; g < Ng; ++g) {
      double se = 0.0;
      for (int i = 0; i < N; ++i) se += es1[(size_t)t * Ne + g * N + i];
      for (int i = 0; i < N; ++i)
        pE[g * N + i] += es1[(size_t)t * Ne + g * N + i] / (se + c->eps);
    }
  }
  double LG = 0.0, LE = 0.0;
  for (int g = 0; g < Ng; ++g) {
    fG[g] *= (double)Ng / (double)c->k_groups * fscale;
    pG[g] /= (double)T;
    LG += (double)c->d_ff[g] / Fmax * fG[g] * pG[g];
  }
  for (int e = 0; e < Ne; ++e) {
    fE[e] *= (double)N / (double)c->k_experts * fscale;
    pE[e] /= (double)T;
    LE += fE[e] * pE[e];
  }
  losses[0] = c->alpha_g * LG;
  losses[1] = c->alpha_e * LE;
  if (stats) memcpy(stats, fG, sizeof(double) * (size_t)(2 * Ng + 2 * Ne));
  free(fG);
  return 0;
}
