/*
 * CPU oracle for one GPU's share of an expert-parallel MoE layer (PROBE, arxiv 2602.00509).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the HIP library
 * is checked against.  It shares no code, header, table or helper with the HIP path and
 * must never be called from the product path: only the tests, the smoke check and the
 * benchmark's cpu_baseline leg load it.
 *
 * Everything floating point is computed in fp64.  bf16 inputs are widened exactly.
 * No blocking, no fusion, no reordering beyond what each definition states; the only
 * concession to speed is an OpenMP "parallel for" over independent tokens / rows.
 *
 * What each function follows:
 *   oracle_route_topk   - router of Sec. 4.2: logits W_L h + b_L, softmax over all experts,
 *                         k largest; Table 1: n_e with sum_e n_e = B*k.
 *   oracle_predict_topk - Eq. 7 (gate-initialised lookahead predictor) with the residual at
 *                         its zero initialisation: the cloned router applied to h_{L-1}.
 *   oracle_predict_topk_residual - Eq. 7 in full: frozen prior + W2_hat silu(W1_hat h).  The
 *                         paper gives neither the hidden width nor the storage types of the
 *                         residual; here W1_hat is bf16 [D,H], W2_hat fp32 [E,D], no biases.
 *   oracle_permute      - token assignment A of Sec. 3.1 / Sec. 4.3: sum_r n_{e,r} = n_e and
 *                         n_{e,r} > 0 => P_{r,e} = 1, applied by weighted round-robin in
 *                         arrival order (a reading; the paper does not fix the rule).
 *   oracle_grouped_ffn  - the grouped GEMM over E_r U Delta_r of Sec. 3.2, with a SwiGLU
 *                         expert (silu(W1 x) * (W3 x), then W2).
 *   oracle_combine      - gate-weighted sum of the expert outputs of a token (the local part
 *                         of the combine step of the main track, Sec. 4.1).
 *   oracle_combine_shared - the same plus a shared expert's output per token.
 *   oracle_imbalance_ratio - Eq. 1.
 *
 * Pins (tests/test_oracle_*.py): brute-force stable sort top-k, the Zipf closed form of a
 * bias-only softmax, uniform case and tie-break, torch fp64 library cross-checks, permutation
 * invariants and a hand-worked 6-token example, the closed-form per-replica counts,
 * identity-expert combine (with a shared expert: (sum of weights + scale) x), plan invariance of the
 * whole layer; for the residual: W2_hat = 0
 * gives the router bit for bit, a one-hot construction with a closed form, additivity in
 * W2_hat of the logits, and a torch fp64 cross-check.
 */
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static double bf16_to_double(uint16_t v) {
  uint32_t u = ((uint32_t)v) << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

/* ---------------------------------------------------------------- router ---- */

/*
 * x        [T,H]  bf16 bit patterns
 * w_gate   [E,H]  fp32
 * bias     [G,E]  fp32 or NULL; token t uses row min(t / tokens_per_group, G-1)
 * outputs: logits [T,E] f64, probs [T,E] f64, idx [T,k] i32, w [T,k] f64,
 *          counts [E] i32.  Any output pointer may be NULL.
 */
/*
 * Shared body of the router and of the predictor.  With w1_hat == NULL the logits are
 * W h + b; otherwise the residual of Eq. 7 is added:
 *     l = W h + b + W2_hat silu(W1_hat h),   silu(u) = u / (1 + exp(-u))
 *   w1_hat  [D,H] bf16 bit patterns,  w2_hat  [E,D] fp32.
 */
static int route_body(const uint16_t* x, const float* w_gate, const float* bias,
                      int G, int tokens_per_group, const uint16_t* w1_hat, const float* w2_hat,
                      int D, int T, int H, int E, int k,
                      int renormalize, double* logits_out, double* probs_out,
                      int32_t* idx_out, double* w_out, int32_t* counts_out) {
  if (T < 0 || H <= 0 || E <= 0 || k <= 0 || k > E) return -1;
  if (bias && (G < 1 || tokens_per_group < 1)) return -1;
  if (w1_hat && (!w2_hat || D <= 0)) return -1;
  int32_t* idx_tmp = (int32_t*)malloc(sizeof(int32_t) * (size_t)(T > 0 ? T : 1) * k);
  if (!idx_tmp) return -2;

#pragma omp parallel for schedule(static)
  for (int t = 0; t < T; ++t) {
    double* l = (double*)malloc(sizeof(double) * E);
    double* p = (double*)malloc(sizeof(double) * E);
    char* taken = (char*)calloc(E, 1);
    int g = 0;
    if (bias) {
      g = t / tokens_per_group;
      if (g > G - 1) g = G - 1;
    }
    /* logits: l_e = sum_h W[e,h] x[t,h] + b[g,e] */
    for (int e = 0; e < E; ++e) {
      double acc = 0.0;
      for (int h = 0; h < H; ++h)
        acc += (double)w_gate[(size_t)e * H + h] * bf16_to_double(x[(size_t)t * H + h]);
      if (bias) acc += (double)bias[(size_t)g * E + e];
      l[e] = acc;
    }
    if (w1_hat) {
      /* trainable residual: s = silu(W1_hat h), l_e += sum_d W2_hat[e,d] s_d */
      double* sv = (double*)malloc(sizeof(double) * D);
      for (int d = 0; d < D; ++d) {
        double u = 0.0;
        for (int h = 0; h < H; ++h)
          u += bf16_to_double(w1_hat[(size_t)d * H + h]) * bf16_to_double(x[(size_t)t * H + h]);
        sv[d] = u / (1.0 + exp(-u));
      }
      for (int e = 0; e < E; ++e) {
        double r = 0.0;
        for (int d = 0; d < D; ++d) r += (double)w2_hat[(size_t)e * D + d] * sv[d];
        l[e] += r;
      }
      free(sv);
    }
    /* softmax over all E experts */
    double m = l[0];
    for (int e = 1; e < E; ++e)
      if (l[e] > m) m = l[e];
    double z = 0.0;
    for (int e = 0; e < E; ++e) {
      p[e] = exp(l[e] - m);
      z += p[e];
    }
    for (int e = 0; e < E; ++e) p[e] /= z;
    /* k largest logits, descending; exact ties go to the lower expert index */
    double wsum = 0.0;
    for (int s = 0; s < k; ++s) {
      int best = -1;
      for (int e = 0; e < E; ++e) {
        if (taken[e]) continue;
        if (best < 0 || l[e] > l[best]) best = e;
      }
      taken[best] = 1;
      idx_tmp[(size_t)t * k + s] = best;
      wsum += p[best];
    }
    for (int s = 0; s < k; ++s) {
      int e = idx_tmp[(size_t)t * k + s];
      double w = p[e];
      if (renormalize) w /= wsum;
      if (w_out) w_out[(size_t)t * k + s] = w;
      if (idx_out) idx_out[(size_t)t * k + s] = e;
    }
    if (logits_out) memcpy(logits_out + (size_t)t * E, l, sizeof(double) * E);
    if (probs_out) memcpy(probs_out + (size_t)t * E, p, sizeof(double) * E);
    free(l);
    free(p);
    free(taken);
  }
  if (counts_out) {
    for (int e = 0; e < E; ++e) counts_out[e] = 0;
    for (size_t i = 0; i < (size_t)T * k; ++i) counts_out[idx_tmp[i]] += 1;
  }
  free(idx_tmp);
  return 0;
}

int oracle_route_topk(const uint16_t* x, const float* w_gate, const float* bias,
                      int G, int tokens_per_group, int T, int H, int E, int k,
                      int renormalize, double* logits_out, double* probs_out,
                      int32_t* idx_out, double* w_out, int32_t* counts_out) {
  return route_body(x, w_gate, bias, G, tokens_per_group, NULL, NULL, 0, T, H, E, k, renormalize,
                    logits_out, probs_out, idx_out, w_out, counts_out);
}

/* Eq. 7 with the trainable residual at its zero initialisation: the frozen prior only. */
int oracle_predict_topk(const uint16_t* h_prev, const float* w_gate_next,
                        const float* bias_next, int G, int tokens_per_group, int T, int H,
                        int E, int k, int renormalize, double* logits_out,
                        double* probs_out, int32_t* idx_out, double* w_out,
                        int32_t* nhat_out) {
  return route_body(h_prev, w_gate_next, bias_next, G, tokens_per_group, NULL, NULL, 0, T, H, E, k,
                    renormalize, logits_out, probs_out, idx_out, w_out, nhat_out);
}

/* Eq. 7 in full: frozen prior plus the residual MLP (hidden width D, SiLU, no biases). */
int oracle_predict_topk_residual(const uint16_t* h_prev, const float* w_gate_next,
                                 const float* bias_next, int G, int tokens_per_group,
                                 const uint16_t* w1_hat, const float* w2_hat, int D, int T, int H,
                                 int E, int k, int renormalize, double* logits_out,
                                 double* probs_out, int32_t* idx_out, double* w_out,
                                 int32_t* nhat_out) {
  if (!w1_hat || !w2_hat || D <= 0) return -1;
  return route_body(h_prev, w_gate_next, bias_next, G, tokens_per_group, w1_hat, w2_hat, D, T, H,
                    E, k, renormalize, logits_out, probs_out, idx_out, w_out, nhat_out);
}

/* --------------------------------------------------------------- permute ---- */

/*
 * Plan: expert e owns replicas rep_off[e] .. rep_off[e+1]-1; replica i lives in local weight
 * slot rep_slot[i] (0..S-1) or on another GPU (-1) and takes rep_weight[i] out of every
 * P_e = sum of the expert's weights consecutive arrivals.
 *
 * Sequential definition: walk the pairs p = t*k + s in ascending order; the j-th arrival of
 * expert e (j counted from 0) goes to the first replica whose cumulative weight exceeds
 * j mod P_e.  A pair sent to a local slot is appended to that slot's list.  Rows are the
 * lists concatenated in slot order.
 *
 * outputs: slot_counts [S], slot_offsets [S+1], row_pair [T*k] (entries >= n_local are -1),
 *          pair_row [T*k] (-1 = not computed on this GPU), xp [T*k,H] bf16 bits (rows >=
 *          n_local zero; may be NULL together with x), n_local [1].
 */
int oracle_permute(const int32_t* topk_idx, const int32_t* rep_off, const int32_t* rep_slot,
                   const int32_t* rep_weight, int S, const uint16_t* x, int T, int H, int E,
                   int k, int32_t* slot_counts, int32_t* slot_offsets, int32_t* row_pair,
                   int32_t* pair_row, uint16_t* xp, int32_t* n_local) {
  if (T < 0 || E <= 0 || k <= 0 || S < 0) return -1;
  size_t N = (size_t)T * k;
  int32_t* cnt = (int32_t*)calloc(E, sizeof(int32_t));
  int32_t* pair_slot = (int32_t*)malloc(sizeof(int32_t) * (N ? N : 1));
  if (!cnt || !pair_slot) return -2;

  for (int s = 0; s < S; ++s) slot_counts[s] = 0;
  for (size_t p = 0; p < N; ++p) {
    int e = topk_idx[p];
    if (e < 0 || e >= E) return -3;
    int j = cnt[e]++;
    int lo = rep_off[e], hi = rep_off[e + 1];
    long P = 0;
    for (int i = lo; i < hi; ++i) {
      if (rep_weight[i] < 0) return -3;
      P += rep_weight[i];
    }
    if (P < 1) return -3;
    long u = (long)j % P;
    long cum = 0;
    int slot = -1;
    for (int i = lo; i < hi; ++i) {
      cum += rep_weight[i];
      if (cum > u) {
        slot = rep_slot[i];
        break;
      }
    }
    if (slot >= S) return -3;
    pair_slot[p] = slot;
    if (slot >= 0) slot_counts[slot] += 1;
  }
  slot_offsets[0] = 0;
  for (int s = 0; s < S; ++s) slot_offsets[s + 1] = slot_offsets[s] + slot_counts[s];
  *n_local = slot_offsets[S];

  /* append in ascending pair order: next free row of each slot */
  int32_t* next = (int32_t*)malloc(sizeof(int32_t) * (S ? S : 1));
  for (int s = 0; s < S; ++s) next[s] = slot_offsets[s];
  for (size_t r = 0; r < N; ++r) row_pair[r] = -1;
  for (size_t p = 0; p < N; ++p) {
    int slot = pair_slot[p];
    if (slot < 0) {
      pair_row[p] = -1;
      continue;
    }
    int row = next[slot]++;
    pair_row[p] = row;
    row_pair[row] = (int32_t)p;
  }
  if (xp && x) {
    memset(xp, 0, sizeof(uint16_t) * N * H);
    for (size_t r = 0; r < (size_t)*n_local; ++r) {
      size_t t = (size_t)row_pair[r] / k;
      memcpy(xp + r * H, x + t * H, sizeof(uint16_t) * H);
    }
  }
  free(next);
  free(pair_slot);
  free(cnt);
  return 0;
}

/* ------------------------------------------------------------ grouped FFN ---- */

/*
 * For every requested row r (rows[i], or i itself when rows == NULL) that falls inside a
 * slot sigma (slot_offsets[sigma] <= r < slot_offsets[sigma+1]):
 *     a = W1_sigma xp[r],  c = W3_sigma xp[r]            (length F)
 *     h = a / (1 + exp(-a)) * c
 *     y[i] = W2_sigma h                                    (length H)
 * w13[sigma] is bf16 [2F,H] (rows 0..F-1 = W1 gate projection, F..2F-1 = W3 up projection),
 * w2[sigma] is bf16 [H,F].  Nothing is rounded on the way.  y is fp64 [n_rows,H]; rows that
 * fall in no slot are left untouched.
 */
int oracle_grouped_ffn(const uint16_t* xp, const int32_t* slot_offsets,
                       const uint16_t* const* w13, const uint16_t* const* w2, int S, int H,
                       int F, const int32_t* rows, int n_rows, double* y) {
  if (S < 0 || H <= 0 || F <= 0 || n_rows < 0) return -1;
#pragma omp parallel for schedule(dynamic, 1)
  for (int i = 0; i < n_rows; ++i) {
    int r = rows ? rows[i] : i;
    int sigma = -1;
    for (int s = 0; s < S; ++s)
      if (r >= slot_offsets[s] && r < slot_offsets[s + 1]) sigma = s;
    if (sigma < 0) continue;
    const uint16_t* W13 = w13[sigma];
    const uint16_t* W2 = w2[sigma];
    const uint16_t* xr = xp + (size_t)r * H;
    double* hbuf = (double*)malloc(sizeof(double) * F);
    for (int f = 0; f < F; ++f) {
      double a = 0.0, c = 0.0;
      const uint16_t* w1 = W13 + (size_t)f * H;
      const uint16_t* w3 = W13 + (size_t)(F + f) * H;
      for (int h = 0; h < H; ++h) {
        double xv = bf16_to_double(xr[h]);
        a += bf16_to_double(w1[h]) * xv;
        c += bf16_to_double(w3[h]) * xv;
      }
      hbuf[f] = a / (1.0 + exp(-a)) * c;
    }
    for (int h = 0; h < H; ++h) {
      double acc = 0.0;
      const uint16_t* w = W2 + (size_t)h * F;
      for (int f = 0; f < F; ++f) acc += bf16_to_double(w[f]) * hbuf[f];
      y[(size_t)i * H + h] = acc;
    }
    free(hbuf);
  }
  return 0;
}

/* --------------------------------------------------------------- combine ---- */

/*
 * out[t,:] = sum over s ascending with pair_row[t,s] >= 0 of w[t,s] * y[pair_row[t,s],:]
 * y fp64 [n_rows,H]; w fp64 [T,k]; out fp64 [T,H].  A token with no local pair gives zeros.
 */
int oracle_combine(const double* y, const int32_t* pair_row, const double* w, int T, int H,
                   int k, double* out) {
  if (T < 0 || H <= 0 || k <= 0) return -1;
#pragma omp parallel for schedule(static)
  for (int t = 0; t < T; ++t) {
    double* o = out + (size_t)t * H;
    for (int h = 0; h < H; ++h) o[h] = 0.0;
    for (int s = 0; s < k; ++s) {
      int row = pair_row[(size_t)t * k + s];
      if (row < 0) continue;
      double ws = w[(size_t)t * k + s];
      const double* yr = y + (size_t)row * H;
      for (int h = 0; h < H; ++h) o[h] += ws * yr[h];
    }
  }
  return 0;
}

/*
 * Combine for a model with a shared expert (an expert every token uses, outside the gate; the
 * output of the MoE block is the routed sum plus the shared expert's output, as in Eq. 12 of the
 * DeepSeek-V3 technical report, without the residual connection, which lies outside the block):
 *   out[t,:] = sum_s w[t,s] * y[pair_row[t,s],:]  +  shared_scale * shared[t,:]
 * shared fp64 [T,H] is the shared expert's FFN output for every token (the grouped FFN run on x
 * itself with one slot of T rows).
 */
int oracle_combine_shared(const double* y, const int32_t* pair_row, const double* w,
                          const double* shared, double shared_scale, int T, int H, int k,
                          double* out) {
  if (!shared) return -1;
  int rc = oracle_combine(y, pair_row, w, T, H, k, out);
  if (rc != 0) return rc;
  for (int t = 0; t < T; ++t)
    for (int h = 0; h < H; ++h)
      out[(size_t)t * H + h] += shared_scale * shared[(size_t)t * H + h];
  return 0;
}

/* ------------------------------------------------------------- metrics ---- */

/* Eq. 1: IR = max_r L_r / mean_r L_r for rank loads L_r (returns 1 for an all-zero load). */
double oracle_imbalance_ratio(const double* rank_load, int ep) {
  double mx = 0.0, sum = 0.0;
  for (int r = 0; r < ep; ++r) {
    if (rank_load[r] > mx) mx = rank_load[r];
    sum += rank_load[r];
  }
  if (sum <= 0.0) return 1.0;
  return mx / (sum / ep);
}

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
