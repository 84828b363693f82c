/*
 * CPU oracle for the backward pass of one MoHGE layer.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT (see mohge_oracle.c): only tests, the
 * smoke check and the benchmark's cpu_baseline leg may call it, and it shares nothing
 * with the HIP library.
 *
 * The paper trains the layer with the objective  L_task + L_G + L_E  (sections 3.3 and
 * 3.4.2) and gives no backward formulas; what is written out here is the chain rule
 * applied, step by step and in reverse order, to the forward definitions of section 3.2
 * and of the two auxiliary losses, all in double.  The function differentiated is
 *
 *     L = sum_{t,k} dy[t,k] * y[t,k]  +  L_G  +  L_E
 *
 * where dy is the incoming gradient of the layer output.  The routing decisions (which
 * groups and experts a token keeps) and the routing frequencies f^G, f^E are counts and
 * are held constant; the gradient flows through GS, ES', ES'', the gates, the
 * probabilities p^G, p^E and the experts.
 *
 * Forward recap for one token (masks fixed): GS_g = sigmoid(zG_g), zG = W_G x;
 * ES'_{g,i} = softmax_i(zE_{g,.}) in kept groups, zE = W_E x + bias; ES'' = ES' * GS_g;
 * D = sum of kept ES''; gate_e = ES''_e / D; y = sum_kept gate_e * E_e(x);
 * E_e(x) = W_down h, h = SiLU(a) * b, a = W_gate x, b = W_up x.
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
  int32_t n_groups;
  int32_t n_per_group;
  const int32_t* d_ff;
  int32_t k_groups;
  int32_t k_experts;
  int32_t select_mode;
  int32_t aux_freq_norm;
  double alpha_g, alpha_e, eps;
} oracle_config;

static double dotd(const float* a, const float* b, int n) {
  double s = 0.0;
  for (int k = 0; k < n; ++k) s += (double)a[k] * (double)b[k];
  return s;
}

/*
 * Backward of the gated combine  y_q = sum_slot gate[q,slot] * y_pairs[q*K_e+slot].
 *   dy[n_tok, d] (float, the values the GPU sees), y_pairs[n_tok*K_e, d] = E_e(x_t).
 *   dgates[q,slot] = <dy_q, y_pairs[q*K_e+slot]>;  dy_pairs[q*K_e+slot] = gate * dy_q.
 */
int oracle_combine_bwd(const oracle_config* c, int64_t n_tok, const double* y_pairs,
                       const double* gates, const float* dy, double* dgates, double* dy_pairs) {
  const int d = c->d, Ke = c->k_experts;
  for (int64_t q = 0; q < n_tok; ++q)
    for (int slot = 0; slot < Ke; ++slot) {
      const double* yp = y_pairs + ((size_t)q * Ke + slot) * d;
      double* dyp = dy_pairs + ((size_t)q * Ke + slot) * d;
      double s = 0.0;
      for (int k = 0; k < d; ++k) {
        s += (double)dy[(size_t)q * d + k] * yp[k];
        dyp[k] = gates[q * Ke + slot] * (double)dy[(size_t)q * d + k];
      }
      dgates[q * Ke + slot] = s;
    }
  return 0;
}

/*
 * Backward of the expert networks for a list of (token, expert) pairs.
 *   dy_pairs[n, d]: gradient of E_e(x_t) for pair q.
 *   dx_pairs[n, d]: gradient of x_t through pair q (the caller sums a token's pairs).
 *   dw_gate[g] / dw_up[g] -> [N, F_g, d], dw_down[g] -> [N, d, F_g]: sums over the pairs
 *   of each expert; the three tables may be NULL (then only dx_pairs is produced).
 *   With  dh = W_down^T dyp,  s = 1/(1+exp(-a)):
 *     da = dh * b * s * (1 + a*(1-s)),   db = dh * a * s,
 *     dW_down += dyp h^T,  dW_gate += da x^T,  dW_up += db x^T,
 *     dx_pair = W_gate^T da + W_up^T db.
 */
int oracle_expert_ffn_bwd(const oracle_config* c, const float* x, const float* const* w_gate,
                          const float* const* w_up, const float* const* w_down, int64_t n,
                          const int32_t* pair_token, const int32_t* pair_expert,
                          const double* dy_pairs, double* dx_pairs, double* const* dw_gate,
                          double* const* dw_up, double* const* dw_down) {
  const int d = c->d, N = c->n_per_group, Ne = c->n_groups * N;
  const int want_w = dw_gate && dw_up && dw_down;
  int Fmax = 0;
  for (int g = 0; g < c->n_groups; ++g) if (c->d_ff[g] > Fmax) Fmax = c->d_ff[g];
#pragma omp parallel
  {
    double* buf = (double*)malloc(sizeof(double) * (size_t)Fmax * 5);
    double *a = buf, *b = a + Fmax, *h = b + Fmax, *da = h + Fmax, *db = da + Fmax;
    /* one expert per thread at a time: its weight gradients are touched by no other */
#pragma omp for schedule(dynamic, 1)
    for (int e = 0; e < Ne; ++e) {
      const int g = e / N, i = e % N, F = c->d_ff[g];
      const float* Wg = w_gate[g] + (size_t)i * F * d;
      const float* Wu = w_up[g] + (size_t)i * F * d;
      const float* Wd = w_down[g] + (size_t)i * d * F;
      double *dWg = NULL, *dWu = NULL, *dWd = NULL;
      if (want_w) {
        dWg = dw_gate[g] + (size_t)i * F * d;
        dWu = dw_up[g] + (size_t)i * F * d;
        dWd = dw_down[g] + (size_t)i * d * F;
        memset(dWg, 0, sizeof(double) * (size_t)F * d);
        memset(dWu, 0, sizeof(double) * (size_t)F * d);
        memset(dWd, 0, sizeof(double) * (size_t)F * d);
      }
      for (int64_t q = 0; q < n; ++q) {
        if (pair_expert[q] != e) continue;
        const float* x_t = x + (size_t)pair_token[q] * d;
        const double* dyp = dy_pairs + (size_t)q * d;
        double* dxp = dx_pairs + (size_t)q * d;
        for (int j = 0; j < F; ++j) {
          a[j] = dotd(x_t, Wg + (size_t)j * d, d);
          b[j] = dotd(x_t, Wu + (size_t)j * d, d);
          const double s = 1.0 / (1.0 + exp(-a[j]));
          h[j] = a[j] * s * b[j];
          double dh = 0.0;
          for (int k = 0; k < d; ++k) dh += (double)Wd[(size_t)k * F + j] * dyp[k];
          da[j] = dh * b[j] * s * (1.0 + a[j] * (1.0 - s));
          db[j] = dh * a[j] * s;
        }
        for (int k = 0; k < d; ++k) dxp[k] = 0.0;
        for (int j = 0; j < F; ++j)
          for (int k = 0; k < d; ++k)
            dxp[k] += (double)Wg[(size_t)j * d + k] * da[j] + (double)Wu[(size_t)j * d + k] * db[j];
        if (want_w) {
          for (int k = 0; k < d; ++k)
            for (int j = 0; j < F; ++j) dWd[(size_t)k * F + j] += dyp[k] * h[j];
          for (int j = 0; j < F; ++j)
            for (int k = 0; k < d; ++k) {
              dWg[(size_t)j * d + k] += da[j] * (double)x_t[k];
              dWu[(size_t)j * d + k] += db[j] * (double)x_t[k];
            }
        }
      }
    }
    free(buf);
  }
  return 0;
}

/*
 * Backward of the two-level router (section 3.2) together with the gradients of the two
 * auxiliary losses (sections 3.3, 3.4.2) with respect to the router.
 *   group_idx[T,K_g], expert_idx[T,K_e]: the forward's decisions (held fixed).
 *   dgates[T,K_e]: gradient of the gates, aligned with expert_idx.
 *   f_G[N_g], f_E[N_e]: the scaled routing frequencies of the two losses (constants).
 *   dx[T,d]: gradient of x through the router only.  dw_group[N_g,d], dw_expert[N_e,d].
 *   dz (may be NULL) [T, N_g+N_e]: gradients of the group logits, then the expert logits
 *   (the latter is also the per-token gradient of the expert logit bias).
 * Per token, with s'_g = GS_g / S, S = sum_g GS_g, u_g = alpha_G (F_g/F_max) f_G[g] / T,
 * v_e = alpha_E f_E[e] / T and sigma_g = sum_i ES'_{g,i}:
 *   dES''_e = (dgate_e - sum_kept dgate*gate) / D            for kept e, else 0
 *   dES'_e  = dES''_e GS_g + v_e/(sigma_g+eps) - sum_i v_i ES'_i / (sigma_g+eps)^2   (kept groups)
 *   dGS_g   = sum_i dES''_{g,i} ES'_{g,i}  +  (u_g - sum_j u_j s'_j) / S             (all groups)
 *   dzE_e   = ES'_e (dES'_e - sum_i dES'_i ES'_i)   (softmax inside the group)
 *   dzG_g   = dGS_g GS_g (1 - GS_g)
 */
int oracle_route_bwd(const oracle_config* c, const float* x, const float* w_group,
                     const float* w_expert, const float* bias, const int32_t* group_idx,
                     const int32_t* expert_idx, const double* dgates, const double* f_G,
                     const double* f_E, double* dx, double* dw_group, double* dw_expert,
                     double* dz_out) {
  const int Ng = c->n_groups, N = c->n_per_group, Ne = Ng * N, d = c->d, T = c->T;
  const int Z = Ng + Ne;
  double Fmax = 0.0;
  for (int g = 0; g < Ng; ++g) if (c->d_ff[g] > Fmax) Fmax = c->d_ff[g];
  double* dz = dz_out ? dz_out : (double*)malloc(sizeof(double) * (size_t)T * Z);
#pragma omp parallel
  {
    double* buf = (double*)calloc((size_t)(4 * Ng + 6 * Ne), sizeof(double));
    double *zG = buf, *GS = zG + Ng, *dGS = GS + Ng, *u = dGS + Ng;
    double *zE = u + Ng, *ES1 = zE + Ne, *ES2 = ES1 + Ne, *dES2 = ES2 + Ne, *dES1 = dES2 + Ne,
           *v = dES1 + Ne;
    char* gsel = (char*)malloc((size_t)Ng);
    for (int g = 0; g < Ng; ++g) u[g] = c->alpha_g * ((double)c->d_ff[g] / Fmax) * f_G[g] / (double)T;
    for (int e = 0; e < Ne; ++e) v[e] = c->alpha_e * f_E[e] / (double)T;
#pragma omp for schedule(static)
    for (int t = 0; t < T; ++t) {
      const float* x_t = x + (size_t)t * d;
      double* dzr = dz + (size_t)t * Z;
      /* forward values, recomputed */
      double S = 0.0;
      for (int g = 0; g < Ng; ++g) {
        zG[g] = dotd(x_t, w_group + (size_t)g * d, d);
        GS[g] = 1.0 / (1.0 + exp(-zG[g]));
        S += GS[g];
        gsel[g] = 0;
        dGS[g] = 0.0;
      }
      for (int s = 0; s < c->k_groups; ++s) gsel[group_idx[(size_t)t * c->k_groups + s]] = 1;
      for (int e = 0; e < Ne; ++e) { ES1[e] = 0.0; ES2[e] = 0.0; dES2[e] = 0.0; dES1[e] = 0.0; }
      for (int g = 0; g < Ng; ++g) {
        if (!gsel[g]) continue;
        double mx = -INFINITY, sum = 0.0;
        for (int i = 0; i < N; ++i) {
          const int e = g * N + i;
          zE[e] = dotd(x_t, w_expert + (size_t)e * d, d) + (bias ? (double)bias[e] : 0.0);
          if (zE[e] > mx) mx = zE[e];
        }
        for (int i = 0; i < N; ++i) sum += exp(zE[g * N + i] - mx);
        for (int i = 0; i < N; ++i) {
          const int e = g * N + i;
          ES1[e] = exp(zE[e] - mx) / sum;
          ES2[e] = ES1[e] * GS[g];
        }
      }
      double D = 0.0;
      for (int s = 0; s < c->k_experts; ++s) D += ES2[expert_idx[(size_t)t * c->k_experts + s]];
      /* gates -> ES'' */
      double gd = 0.0;
      for (int s = 0; s < c->k_experts; ++s) {
        const int e = expert_idx[(size_t)t * c->k_experts + s];
        gd += dgates[(size_t)t * c->k_experts + s] * (ES2[e] / D);
      }
      for (int s = 0; s < c->k_experts; ++s) {
        const int e = expert_idx[(size_t)t * c->k_experts + s];
        dES2[e] = (dgates[(size_t)t * c->k_experts + s] - gd) / D;
      }
      /* ES'' = ES' * GS, plus the intra-group loss acting on ES' of the kept groups */
      for (int g = 0; g < Ng; ++g) {
        if (!gsel[g]) continue;
        double sigma = 0.0, vs = 0.0;
        for (int i = 0; i < N; ++i) { sigma += ES1[g * N + i]; vs += v[g * N + i] * ES1[g * N + i]; }
        for (int i = 0; i < N; ++i) {
          const int e = g * N + i;
          dES1[e] = dES2[e] * GS[g] + v[e] / (sigma + c->eps) - vs / ((sigma + c->eps) * (sigma + c->eps));
          dGS[g] += dES2[e] * ES1[e];
        }
      }
      /* the group-wise loss acts on every GS through s' = GS / S */
      double us = 0.0;
      for (int g = 0; g < Ng; ++g) us += u[g] * GS[g] / S;
      for (int g = 0; g < Ng; ++g) dGS[g] += (u[g] - us) / S;
      /* logits */
      for (int g = 0; g < Ng; ++g) dzr[g] = dGS[g] * GS[g] * (1.0 - GS[g]);
      for (int g = 0; g < Ng; ++g) {
        double w = 0.0;
        if (gsel[g]) for (int i = 0; i < N; ++i) w += dES1[g * N + i] * ES1[g * N + i];
        for (int i = 0; i < N; ++i) {
          const int e = g * N + i;
          dzr[Ng + e] = gsel[g] ? ES1[e] * (dES1[e] - w) : 0.0;
        }
      }
      /* x through both logit products */
      double* dxr = dx + (size_t)t * d;
      for (int k = 0; k < d; ++k) dxr[k] = 0.0;
      for (int g = 0; g < Ng; ++g)
        for (int k = 0; k < d; ++k) dxr[k] += dzr[g] * (double)w_group[(size_t)g * d + k];
      for (int e = 0; e < Ne; ++e) {
        if (dzr[Ng + e] == 0.0) continue;
        for (int k = 0; k < d; ++k) dxr[k] += dzr[Ng + e] * (double)w_expert[(size_t)e * d + k];
      }
    }
    /* router weights: dW[r,:] = sum_t dz[t,r] x_t, one row per thread at a time */
#pragma omp for schedule(dynamic, 1)
    for (int r = 0; r < Z; ++r) {
      double* row = r < Ng ? dw_group + (size_t)r * d : dw_expert + (size_t)(r - Ng) * d;
      for (int k = 0; k < d; ++k) row[k] = 0.0;
      for (int t = 0; t < T; ++t) {
        const double z = dz[(size_t)t * Z + r];
        if (z == 0.0) continue;
        for (int k = 0; k < d; ++k) row[k] += z * (double)x[(size_t)t * d + k];
      }
    }
    free(buf);
    free(gsel);
  }
  if (!dz_out) free(dz);
  return 0;
}
