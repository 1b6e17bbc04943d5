/*
 * planner_oracle.c - CPU oracle of the greedy balance-optimal planner of PROBE
 * (arxiv 2602.00509, Sec. 4.3, Algorithm 1), in plain sequential C with integer arithmetic.
 *
 * TEST INFRASTRUCTURE ONLY, like probe_oracle.c: independent of the HIP sources, shares no
 * code with them.
 *
 * The paper gives the loop (Algorithm 1) and describes its sub-routines in words; it prints
 * neither their formulas nor their constants.  The steps below are taken in the paper's order
 * and notation; every choice the paper leaves open is stated where it is made.
 *
 * State.  n[rs][e][rt] = tokens that originate on rank rs, are routed to expert e and are
 * processed on rank rt (the n^{r_s}_{e,r_t} of Table 1).  host[e][r] = 1 when rank r holds a
 * copy of expert e (baseline placement P': expert e lives on rank e / E_loc; Delta^in adds
 * replicas).
 *
 * ComputeLatencies (Sec. 3.2, 3.3).  Per rank r, in integer cost units:
 *     T_comp^r = sum over experts with n_{e,r} > 0 of (n_{e,r} + n0)
 *         - the paper's T_{e,r} = n F / (eta_g(n) F_peak) with the saturating efficiency
 *           eta_g(n) = n / (n + n0): n0 is the token count at which a grouped GEMM runs at half
 *           its peak rate (a parameter; the paper only says eta_g falls for small n);
 *     V_in^r  = tokens processed on r that originate elsewhere,
 *     V_out^r = tokens that originate on r and are processed elsewhere   (lambda = 1: no
 *           deduplication), V^r = max(V_in^r, V_out^r);
 *     L_r = g_den * T_comp^r + 2 * g_num * V^r
 *         - g_num / g_den is the time to move one token over the network relative to the time
 *           to compute it (T_MoE = compute + 2 * V / BW of Sec. 3.3).
 *
 * SelectHeavyExpert(r_src).  The expert held by r_src and not by r_dst with the largest
 * n_{e,r_src} among those with something to move (tokens processed on r_src that originate on
 * r_dst or on a rank holding no copy of e); ties go to the lower expert id.
 *
 * CheckDualBudget.  |Delta^out_{r_src}| < budget and |Delta^in_{r_dst}| < min(budget,
 * max_replicas): the paper's T_trans = max(|Delta^in|, |Delta^out|) W / BW <= T_window with
 * budget = floor(T_window BW / W) experts, and the replica-slot cap of Sec. 5.
 *
 * WaterFillingRebalance(e*, r_src, r_dst).  r_dst gets a copy of e*.  Locality first: tokens
 * of e* that originate on r_dst are now processed on r_dst, wherever they were processed
 * before.  The remote pool - tokens of e* processed on r_src whose origin holds no copy -
 * is then redirected to r_dst, origins in ascending rank order, until the token load of
 * r_src (sum_e n_{e,r_src}) has come down to the cluster average ceil(total / R) or the pool
 * is empty.  gain = max_r L_r before - max_r L_r after.
 *
 * Loop control as printed: a failed budget check (or no expert to move) marks the pair
 * (r_src, r_dst) invalid and continues with the next least-loaded valid helper; the loop ends
 * when gain <= eps, after k_max accepted moves, or when no valid helper is left.
 *
 * Pins (tests/test_oracle_planner.py): conservation sum_rt n = n-hat and validity
 * n_{e,r} > 0 => P_{r,e} = 1 (the constraints of the optimisation problem), the budgets, a
 * non-increasing bottleneck latency, locality, the fixed point on balanced input, and two
 * hand-worked three-rank examples whose every number is written out in the test.  The two views
 * of the result (oracle_plan_for_rank: what a rank receives; oracle_plan_dispatch: what a rank
 * sends) are pinned by the hand-worked example, by each other (same replica lists, the origins'
 * weights add up to the receiver's) and by locality (an origin that holds a copy keeps its tokens).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define IDX(rs, e, rt) (((size_t)(rs) * E + (e)) * R + (rt))

typedef struct {
  int R, E;
  int64_t n0, g_num, g_den;
} cost_model;

static void latencies(const cost_model* m, const int32_t* n, int64_t* L, int64_t* load) {
  const int R = m->R, E = m->E;
  for (int r = 0; r < R; ++r) {
    int64_t comp = 0, tok = 0, vin = 0, vout = 0;
    for (int e = 0; e < E; ++e) {
      int64_t ner = 0;
      for (int rs = 0; rs < R; ++rs) {
        ner += n[IDX(rs, e, r)];
        if (rs != r) vin += n[IDX(rs, e, r)];
      }
      if (ner > 0) comp += ner + m->n0;
      tok += ner;
      for (int rt = 0; rt < R; ++rt)
        if (rt != r) vout += n[IDX(r, e, rt)];
    }
    const int64_t v = vin > vout ? vin : vout;
    L[r] = m->g_den * comp + 2 * m->g_num * v;
    if (load) load[r] = tok;
  }
}

static int64_t max_of(const int64_t* L, int R) {
  int64_t mx = L[0];
  for (int r = 1; r < R; ++r)
    if (L[r] > mx) mx = L[r];
  return mx;
}

/*
 * n_hat      [R][E]  predicted tokens per (source rank, expert)
 * outputs:
 *   n_out      [R][E][R]  final assignment n[rs][e][rt]
 *   delta_in   [R][max_replicas]  experts replicated onto each rank, in the order they were
 *                                 added, -1 padded
 *   delta_out  [R][budget]        experts each rank sends, same convention (may be NULL)
 *   moves      [k_max][3]         (e*, r_src, r_dst) of every accepted move, -1 padded
 *   stats      [4]  L_max before, L_max after, max token load after, accepted moves
 */
int oracle_plan_greedy(const int32_t* n_hat, int R, int E, int E_loc, int max_replicas,
                       int budget, int k_max, int64_t eps, int64_t n0, int64_t g_num,
                       int64_t g_den, int32_t* n_out, int32_t* delta_in, int32_t* delta_out,
                       int32_t* moves, int64_t* stats) {
  if (R < 1 || E < 1 || E_loc < 1 || (long)E_loc * R < E || max_replicas < 0 || budget < 0 ||
      k_max < 0 || g_den < 1 || g_num < 0 || n0 < 0)
    return -1;
  cost_model m = {R, E, n0, g_num, g_den};
  int32_t* n = (int32_t*)calloc((size_t)R * E * R, sizeof(int32_t));
  int32_t* trial = (int32_t*)malloc((size_t)R * E * R * sizeof(int32_t));
  char* host = (char*)calloc((size_t)E * R, 1);
  char* invalid = (char*)calloc((size_t)R * R, 1);
  int* n_in = (int*)calloc(R, sizeof(int));
  int* n_outc = (int*)calloc(R, sizeof(int));
  int64_t* L = (int64_t*)malloc(sizeof(int64_t) * R);
  int64_t* L2 = (int64_t*)malloc(sizeof(int64_t) * R);
  int64_t* load = (int64_t*)malloc(sizeof(int64_t) * R);
  if (!n || !trial || !host || !invalid || !n_in || !n_outc || !L || !L2 || !load) return -2;

  for (int i = 0; i < R * max_replicas; ++i) delta_in[i] = -1;
  if (delta_out)
    for (int i = 0; i < R * budget; ++i) delta_out[i] = -1;
  for (int i = 0; i < k_max * 3; ++i) moves[i] = -1;

  /* initial A from n-hat and the baseline placement: every token to the expert's home rank */
  for (int e = 0; e < E; ++e) host[(size_t)e * R + e / E_loc] = 1;
  for (int rs = 0; rs < R; ++rs)
    for (int e = 0; e < E; ++e) {
      if (n_hat[(size_t)rs * E + e] < 0) return -3;
      n[IDX(rs, e, e / E_loc)] = n_hat[(size_t)rs * E + e];
    }
  /* initial latencies */
  latencies(&m, n, L, load);
  const int64_t L_before = max_of(L, R);
  int64_t total = 0;
  for (int r = 0; r < R; ++r) total += load[r];
  const int64_t avg = (total + R - 1) / R;

  int k = 0;
  for (;;) {
    /* bottleneck rank, and the least-loaded helper whose pair with it is still valid */
    int src = 0;
    for (int r = 1; r < R; ++r)
      if (L[r] > L[src]) src = r;
    int dst = -1;
    for (int r = 0; r < R; ++r) {
      if (r == src || invalid[(size_t)src * R + r]) continue;
      if (dst < 0 || L[r] < L[dst]) dst = r;
    }
    if (dst < 0) break;

    /* SelectHeavyExpert */
    int best = -1;
    int64_t best_n = -1;
    for (int e = 0; e < E; ++e) {
      if (!host[(size_t)e * R + src] || host[(size_t)e * R + dst]) continue;
      int64_t ner = 0, movable = 0;
      for (int rs = 0; rs < R; ++rs) {
        const int64_t v = n[IDX(rs, e, src)];
        ner += v;
        if (rs == dst || !host[(size_t)e * R + rs]) movable += v;
      }
      if (movable > 0 && ner > best_n) {
        best_n = ner;
        best = e;
      }
    }
    /* dual-side budget check (an empty selection is treated the same way) */
    const int cap_in = budget < max_replicas ? budget : max_replicas;
    if (best < 0 || n_outc[src] >= budget || n_in[dst] >= cap_in) {
      invalid[(size_t)src * R + dst] = 1;
      continue;
    }

    /* WaterFillingRebalance on a copy of A */
    memcpy(trial, n, (size_t)R * E * R * sizeof(int32_t));
    const int e = best;
    for (int rt = 0; rt < R; ++rt) { /* locality first: dst's own tokens of e come home */
      if (rt == dst) continue;
      trial[IDX(dst, e, dst)] += trial[IDX(dst, e, rt)];
      trial[IDX(dst, e, rt)] = 0;
    }
    int64_t src_load = 0;
    for (int ee = 0; ee < E; ++ee)
      for (int rs = 0; rs < R; ++rs) src_load += trial[IDX(rs, ee, src)];
    int64_t want = src_load - avg;
    for (int rs = 0; rs < R && want > 0; ++rs) {
      if (rs == dst || host[(size_t)e * R + rs]) continue; /* only origins without a copy */
      int64_t mv = trial[IDX(rs, e, src)];
      if (mv > want) mv = want;
      trial[IDX(rs, e, src)] -= (int32_t)mv;
      trial[IDX(rs, e, dst)] += (int32_t)mv;
      want -= mv;
    }
    latencies(&m, trial, L2, NULL);
    const int64_t gain = max_of(L, R) - max_of(L2, R);

    /* converged, or the iteration budget is used up */
    if (gain <= eps || k >= k_max) break;

    /* accept the move */
    if (delta_out) delta_out[(size_t)src * budget + n_outc[src]] = e;
    delta_in[(size_t)dst * max_replicas + n_in[dst]] = e;
    n_outc[src] += 1;
    n_in[dst] += 1;
    host[(size_t)e * R + dst] = 1;
    moves[3 * k] = e;
    moves[3 * k + 1] = src;
    moves[3 * k + 2] = dst;
    memcpy(n, trial, (size_t)R * E * R * sizeof(int32_t));
    memcpy(L, L2, sizeof(int64_t) * R);
    k += 1;
  }

  latencies(&m, n, L, load);
  memcpy(n_out, n, (size_t)R * E * R * sizeof(int32_t));
  stats[0] = L_before;
  stats[1] = max_of(L, R);
  stats[2] = max_of(load, R);
  stats[3] = k;
  free(n); free(trial); free(host); free(invalid); free(n_in); free(n_outc);
  free(L); free(L2); free(load);
  return 0;
}

/*
 * The plan as one rank sees it, in the layout probe_permute consumes: expert e owns the
 * replicas rep_off[e] .. rep_off[e+1]-1, one per rank that holds a copy, in ascending rank
 * order; rep_weight = tokens planned for that copy (sum over origins); rep_slot = local slot
 * when the copy is on `rank` (native experts first, then replicas in the order of delta_in),
 * -1 otherwise.  An expert with no planned token keeps weight 1 on its home copy, so that
 * tokens the prediction missed still have somewhere to go.
 * slot_expert [E_loc + max_replicas]: expert held by each local slot, -1 = empty.
 */
int oracle_plan_for_rank(const int32_t* n, const int32_t* delta_in, int R, int E, int E_loc,
                         int max_replicas, int rank, int32_t* rep_off, int32_t* rep_slot,
                         int32_t* rep_weight, int32_t* slot_expert) {
  if (rank < 0 || rank >= R) return -1;
  const int S = E_loc + max_replicas;
  for (int s = 0; s < S; ++s) slot_expert[s] = -1;
  for (int e = 0; e < E; ++e)
    if (e / E_loc == rank) slot_expert[e - rank * E_loc] = e;
  for (int i = 0; i < max_replicas; ++i) slot_expert[E_loc + i] = delta_in[(size_t)rank * max_replicas + i];
  int pos = 0;
  for (int e = 0; e < E; ++e) {
    rep_off[e] = pos;
    int64_t planned = 0;
    int home_pos = pos;
    for (int r = 0; r < R; ++r) {
      int here = (e / E_loc == r);
      int slot = here ? e - r * E_loc : -1;
      if (here) home_pos = pos;
      for (int i = 0; i < max_replicas && !here; ++i)
        if (delta_in[(size_t)r * max_replicas + i] == e) {
          here = 1;
          slot = E_loc + i;
        }
      if (!here) continue;
      int64_t w = 0;
      for (int rs = 0; rs < R; ++rs) w += n[IDX(rs, e, r)];
      rep_slot[pos] = (r == rank) ? slot : -1;
      rep_weight[pos] = (int32_t)w;
      planned += w;
      pos += 1;
    }
    if (planned == 0) rep_weight[home_pos] = 1; /* nothing predicted: unforeseen tokens go home */
  }
  rep_off[E] = pos;
  return 0;
}

/*
 * The same plan as a SOURCE rank applies it to its own tokens ahead of the dispatch exchange
 * (assignment A of Sec. 3.1 with the locality-first rule of Sec. 4.3), in the layout of
 * probe_permute.  A "slot" here is one (destination rank, expert) pair: every copy of every expert
 * gets a slot of its own, numbered by destination rank first and expert second, so that permute
 * groups the source's pairs by destination rank (the send order of the exchange) and, inside a
 * rank, by expert.  Expert e lists its copies by ascending rank; rep_slot = the copy's slot;
 * rep_weight = n[rs][e][r], the tokens that originate on rs and are planned for the copy on r.
 * When no token of e was predicted from this origin, an unforeseen one stays on rs if rs holds a
 * copy and goes to e's home otherwise (weight 1 there).  The replica lists are those of
 * oracle_plan_for_rank (same rep_off).
 *   rank_off    [R+1]  slots rank_off[r] .. rank_off[r+1]-1 are sent to rank r
 *   slot_expert [rep_off[E]]  expert of each slot
 */
int oracle_plan_dispatch(const int32_t* n, const int32_t* delta_in, int R, int E, int E_loc,
                         int max_replicas, int rs, int32_t* rep_off, int32_t* rep_slot,
                         int32_t* rep_weight, int32_t* rank_off, int32_t* slot_expert) {
  if (rs < 0 || rs >= R) return -1;
  char* holds = (char*)calloc((size_t)E * R, 1); /* holds[e*R + r] */
  if (!holds) return -2;
  for (int e = 0; e < E; ++e) holds[(size_t)e * R + e / E_loc] = 1;
  for (int r = 0; r < R; ++r)
    for (int i = 0; i < max_replicas; ++i) {
      int e = delta_in[(size_t)r * max_replicas + i];
      if (e >= 0 && e < E) holds[(size_t)e * R + r] = 1;
    }
  /* slots: destination rank first, expert second */
  int slot = 0;
  for (int r = 0; r < R; ++r) {
    rank_off[r] = slot;
    for (int e = 0; e < E; ++e)
      if (holds[(size_t)e * R + r]) slot_expert[slot++] = e;
  }
  rank_off[R] = slot;
  int pos = 0;
  for (int e = 0; e < E; ++e) {
    rep_off[e] = pos;
    int64_t planned = 0;
    int home_pos = pos, own_pos = -1;
    for (int r = 0; r < R; ++r) {
      if (!holds[(size_t)e * R + r]) continue;
      if (r == e / E_loc) home_pos = pos;
      if (r == rs) own_pos = pos;
      int sl = rank_off[r];
      for (int e2 = 0; e2 < e; ++e2) sl += holds[(size_t)e2 * R + r];
      rep_slot[pos] = sl;
      rep_weight[pos] = n[IDX(rs, e, r)];
      planned += n[IDX(rs, e, r)];
      pos += 1;
    }
    if (planned == 0) rep_weight[own_pos >= 0 ? own_pos : home_pos] = 1;
  }
  rep_off[E] = pos;
  free(holds);
  return 0;
}
