/*
 * CPU oracle for the group-limited gate (model-faithful gating variant of the router).
 *
 * TEST INFRASTRUCTURE ONLY: loaded by the tests, the smoke check and nothing else; shares no
 * code with the HIP library.  Everything floating point is fp64; bf16 inputs are widened exactly.
 *
 * The PROBE paper names DeepSeek-V3 among the models it targets (Sec. 1) and leaves the gate of
 * each model as published.  This file restates the gate of the DeepSeek-V3 technical report,
 * Sec. 2.1.2 (sigmoid affinities, gating values normalised over the selected experts), its
 * auxiliary-loss-free balancing (a per-expert bias that takes part in the selection only) and
 * its node-limited routing as the released model configures it (experts in n_group consecutive
 * groups; a group is scored by the sum of its largest selection scores; a token may only use the
 * topk_group best groups).  Steps, per token t:
 *
 *   1. l_e  = sum_h W[e,h] x[t,h] + b[g(t),e]                        logits (b optional)
 *   2. s_e  = sigmoid(l_e)            (scoring = 1)
 *           = softmax(l)_e            (scoring = 0)
 *   3. c_e  = s_e + select_bias[e]    (select_bias optional)          selection scores
 *   4. G_j  = sum of the group_top largest c_e of group j = { j*E/n_group .. (j+1)*E/n_group - 1 }
 *   5. the topk_group groups with the largest G_j (equal scores: lower group first) are allowed
 *   6. the k allowed experts with the largest c_e, descending (equal scores: lower expert first)
 *   7. w    = s_e of the chosen experts (not c_e), divided by their sum when renormalize != 0,
 *             times routed_scale
 *   8. counts[e] = number of (token, slot) pairs that chose e
 *
 * The report adds 1e-20 to the normalising sum of step 7; with sigmoid or softmax scores the sum is
 * positive and the term changes nothing at fp64 precision, so it is left out.
 *
 * Pins (tests/test_oracle_gating.py): a hand-worked token with exactly representable scores
 * (tests/golden/gating_example.txt), a sort-based brute force in numpy, the reductions to the
 * plain router (one group, softmax) and to its index order (sigmoid is monotone), invariants
 * (chosen experts lie in allowed groups, weights sum to routed_scale, the selection bias moves
 * the choice but not the weight), and planted-mistake checks on the example (group score from the
 * largest element only, bias leaking into the weight, groups not limited).
 */
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static double bf16_widen(uint16_t v) {
  uint32_t u = ((uint32_t)v) << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

/*
 * x [T,H] bf16 bits; w_gate [E,H] fp32; bias [G,E] fp32 or NULL (token t uses row
 * min(t / tokens_per_group, G-1)); select_bias [E] fp32 or NULL.
 * outputs (any may be NULL): logits, scores, choice [T,E] f64; group_scores [T,n_group] f64;
 * groups [T,topk_group] i32 in the order chosen; idx [T,k] i32; w [T,k] f64; counts [E] i32.
 * returns 0, -1 for bad arguments, -2 out of memory.
 */
int oracle_route_grouped(const uint16_t* x, const float* w_gate, const float* bias, int G,
                         int tokens_per_group, const float* select_bias, int scoring, int n_group,
                         int topk_group, int group_top, int renormalize, double routed_scale,
                         int T, int H, int E, int k, double* logits_out, double* scores_out,
                         double* choice_out, double* group_scores_out, int32_t* groups_out,
                         int32_t* idx_out, double* w_out, int32_t* counts_out) {
  if (T < 0 || H <= 0 || E <= 0 || k <= 0 || k > E) return -1;
  if (bias && (G < 1 || tokens_per_group < 1)) return -1;
  if (scoring != 0 && scoring != 1) return -1;
  if (n_group < 1 || E % n_group != 0) return -1;
  const int gs = E / n_group;
  if (topk_group < 1 || topk_group > n_group) return -1;
  if (group_top < 1 || group_top > gs) return -1;
  if (k > topk_group * gs) return -1;
  int32_t* idx_tmp = (int32_t*)malloc(sizeof(int32_t) * (size_t)(T > 0 ? T : 1) * k);
  if (!idx_tmp) return -2;

#pragma omp parallel for schedule(static)
  for (int t = 0; t < T; ++t) {
    double* l = (double*)malloc(sizeof(double) * E);
    double* s = (double*)malloc(sizeof(double) * E);
    double* c = (double*)malloc(sizeof(double) * E);
    double* gscore = (double*)malloc(sizeof(double) * n_group);
    char* used = (char*)malloc(E);
    char* allowed = (char*)calloc(n_group, 1);
    int g = 0;
    if (bias) {
      g = t / tokens_per_group;
      if (g > G - 1) g = G - 1;
    }
    /* 1. logits */
    for (int e = 0; e < E; ++e) {
      double acc = 0.0;
      for (int h = 0; h < H; ++h)
        acc += (double)w_gate[(size_t)e * H + h] * bf16_widen(x[(size_t)t * H + h]);
      if (bias) acc += (double)bias[(size_t)g * E + e];
      l[e] = acc;
    }
    /* 2. scores */
    if (scoring == 1) {
      for (int e = 0; e < E; ++e) s[e] = 1.0 / (1.0 + exp(-l[e]));
    } else {
      double m = l[0], z = 0.0;
      for (int e = 1; e < E; ++e)
        if (l[e] > m) m = l[e];
      for (int e = 0; e < E; ++e) {
        s[e] = exp(l[e] - m);
        z += s[e];
      }
      for (int e = 0; e < E; ++e) s[e] /= z;
    }
    /* 3. selection scores */
    for (int e = 0; e < E; ++e) c[e] = s[e] + (select_bias ? (double)select_bias[e] : 0.0);
    /* 4. group scores: add up the group_top largest selection scores of each group */
    for (int j = 0; j < n_group; ++j) {
      memset(used, 0, E);
      double sum = 0.0;
      for (int r = 0; r < group_top; ++r) {
        int best = -1;
        for (int e = j * gs; e < (j + 1) * gs; ++e) {
          if (used[e]) continue;
          if (best < 0 || c[e] > c[best]) best = e;
        }
        used[best] = 1;
        sum += c[best];
      }
      gscore[j] = sum;
    }
    /* 5. allowed groups */
    for (int r = 0; r < topk_group; ++r) {
      int best = -1;
      for (int j = 0; j < n_group; ++j) {
        if (allowed[j]) continue;
        if (best < 0 || gscore[j] > gscore[best]) best = j;
      }
      allowed[best] = 1;
      if (groups_out) groups_out[(size_t)t * topk_group + r] = best;
    }
    /* 6. k largest selection scores among the experts of allowed groups */
    memset(used, 0, E);
    double wsum = 0.0;
    for (int r = 0; r < k; ++r) {
      int best = -1;
      for (int e = 0; e < E; ++e) {
        if (used[e] || !allowed[e / gs]) continue;
        if (best < 0 || c[e] > c[best]) best = e;
      }
      used[best] = 1;
      idx_tmp[(size_t)t * k + r] = best;
      wsum += s[best];
    }
    /* 7. gating values from the scores without the selection bias */
    for (int r = 0; r < k; ++r) {
      int e = idx_tmp[(size_t)t * k + r];
      double w = s[e];
      if (renormalize) w /= wsum;
      w *= routed_scale;
      if (w_out) w_out[(size_t)t * k + r] = w;
      if (idx_out) idx_out[(size_t)t * k + r] = e;
    }
    if (logits_out) memcpy(logits_out + (size_t)t * E, l, sizeof(double) * E);
    if (scores_out) memcpy(scores_out + (size_t)t * E, s, sizeof(double) * E);
    if (choice_out) memcpy(choice_out + (size_t)t * E, c, sizeof(double) * E);
    if (group_scores_out) memcpy(group_scores_out + (size_t)t * n_group, gscore, sizeof(double) * n_group);
    free(l);
    free(s);
    free(c);
    free(gscore);
    free(used);
    free(allowed);
  }
  /* 8. counts */
  if (counts_out) {
    for (int e = 0; e < E; ++e) counts_out[e] = 0;
    for (size_t i = 0; i < (size_t)T * k; ++i) counts_out[idx_tmp[i]] += 1;
  }
  free(idx_tmp);
  return 0;
}
