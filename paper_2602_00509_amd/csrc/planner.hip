// probe_plan_greedy: the greedy balance-optimal planner (Sec. 4.3, Algorithm 1) as one workgroup.
//
// Input is the all-gathered prediction n_hat[R][E] (tokens that originate on rank rs and are predicted
// for expert e); output is the placement change (Delta^in / Delta^out per rank), the assignment
// n[rs][e][rt] and, for one rank, the plan in the layout probe_permute consumes - all in device
// memory, so that predict -> plan -> permute needs no host round trip (Sec. 2.3).
//
// The paper runs its solver as a single-block kernel with serial iterative updates (Sec. 5); the
// same shape fits here: the loop is inherently sequential (each move changes the bottleneck), and
// what one iteration touches is small once the per-rank aggregates are kept incrementally:
//   LDS   ner[e][r]   tokens of expert e processed on rank r
//         comp[r]     sum over experts with ner > 0 of (ner + n0)          (compute term)
//         vin[r], vout[r]   tokens received from / sent to other ranks      (network term)
//         load[r]     tokens processed on rank r
//   HBM   n[e][rs][rt]  the assignment, expert-major: a move rewrites one R x R slab
// Per iteration only SelectHeavyExpert looks at every expert (one thread each, block arg-max by a
// 64-bit LDS atomic); the water-filling of the chosen expert's slab and the new latencies are a few
// hundred integer operations done by one thread.  All arithmetic is integer, so the plan is
// bit-identical to the sequential definition.
//
// Cost model (a reading; the paper names the terms but not their constants):
//   L_r = g_den * comp[r] + 2 * g_num * max(vin[r], vout[r])
// with eta_g(n) = n / (n + n0) inside comp (Sec. 3.2) and g_num / g_den = network time per token over
// compute time per token (Sec. 3.3).
#include "common.hpp"

namespace probe {

constexpr int kPlanMaxRanks = 16;
constexpr int kPlanMaxReplicas = 8;
constexpr int kPlanMaxMoves = 64;

struct PlannerArgs {
  int R, E, E_loc, rank, max_replicas, budget, k_max;
  long long eps, n0, g_num, g_den;
};

__device__ __forceinline__ long long comp_term(long long tokens, long long n0) { return tokens > 0 ? tokens + n0 : 0; }

__global__ __launch_bounds__(256) void plan_greedy_kernel(const int32_t* __restrict__ n_hat, PlannerArgs a,
                                                          int32_t* __restrict__ g_n,  // [E][R][R] workspace
                                                          int32_t* __restrict__ rep_off, int32_t* __restrict__ rep_slot,
                                                          int32_t* __restrict__ rep_weight,
                                                          int32_t* __restrict__ slot_expert,
                                                          int32_t* __restrict__ delta_in, int32_t* __restrict__ delta_out,
                                                          int32_t* __restrict__ moves, long long* __restrict__ stats,
                                                          int32_t* __restrict__ n_assign) {
  const int R = a.R, E = a.E, E_loc = a.E_loc;
  __shared__ int32_t ner[PROBE_MAX_EXPERTS][kPlanMaxRanks];
  __shared__ uint32_t hostmask[PROBE_MAX_EXPERTS];
  __shared__ unsigned long long comp[kPlanMaxRanks], vin[kPlanMaxRanks], vout[kPlanMaxRanks], load[kPlanMaxRanks];
  __shared__ long long lat[kPlanMaxRanks], t_comp[kPlanMaxRanks], t_vin[kPlanMaxRanks], t_vout[kPlanMaxRanks],
      t_load[kPlanMaxRanks], t_lat[kPlanMaxRanks];
  __shared__ int32_t slab_old[kPlanMaxRanks][kPlanMaxRanks], slab_new[kPlanMaxRanks][kPlanMaxRanks];
  __shared__ uint32_t invalid[kPlanMaxRanks];
  __shared__ int32_t n_in[kPlanMaxRanks], n_out[kPlanMaxRanks];
  __shared__ int32_t d_in[kPlanMaxRanks][kPlanMaxReplicas];
  __shared__ long long best_key, lat_before;
  __shared__ int32_t wave_tot[4];
  const int tid = threadIdx.x, lane = tid & 63;

  // ---- initial assignment: every token to the expert's home rank (baseline placement P')
  if (tid < kPlanMaxRanks) {
    comp[tid] = vin[tid] = vout[tid] = load[tid] = 0;
    invalid[tid] = 0;
    n_in[tid] = n_out[tid] = 0;
    for (int i = 0; i < kPlanMaxReplicas; ++i) d_in[tid][i] = -1;
  }
  __syncthreads();
  if (tid < E) {
    const int e = tid, home = e / E_loc;
    long long tot = 0;
    for (int rs = 0; rs < R; ++rs) {
      const int v = max(n_hat[rs * E + e], 0);
      for (int rt = 0; rt < R; ++rt) g_n[(e * R + rs) * R + rt] = (rt == home) ? v : 0;
      tot += v;
      if (rs != home && v) {
        atomicAdd(&vin[home], static_cast<unsigned long long>(v));
        atomicAdd(&vout[rs], static_cast<unsigned long long>(v));
      }
    }
    for (int r = 0; r < R; ++r) ner[e][r] = (r == home) ? static_cast<int>(tot) : 0;
    hostmask[e] = 1u << home;
    if (tot) {
      atomicAdd(&comp[home], static_cast<unsigned long long>(comp_term(tot, a.n0)));
      atomicAdd(&load[home], static_cast<unsigned long long>(tot));
    }
  }
  for (int i = tid; i < R * a.max_replicas; i += 256) delta_in[i] = -1;
  if (delta_out)
    for (int i = tid; i < R * a.budget; i += 256) delta_out[i] = -1;
  for (int i = tid; i < a.k_max * 3; i += 256) moves[i] = -1;
  __syncthreads();
  if (tid == 0) {
    long long mx = 0;
    for (int r = 0; r < R; ++r) {
      lat[r] = a.g_den * static_cast<long long>(comp[r]) +
               2 * a.g_num * static_cast<long long>(max(vin[r], vout[r]));
      mx = r == 0 ? lat[r] : max(mx, lat[r]);
    }
    lat_before = mx;
  }
  __syncthreads();
  long long total = 0;
  for (int r = 0; r < R; ++r) total += static_cast<long long>(load[r]);
  const long long avg = (total + R - 1) / R;
  const int cap_in = min(a.budget, a.max_replicas);

  // ---- the loop of Algorithm 1; every thread follows the same control flow
  int k = 0;
  for (int guard = 0; guard < kPlanMaxMoves + kPlanMaxRanks * kPlanMaxRanks + 1; ++guard) {
    // bottleneck rank and the least-loaded helper whose pair with it is still valid (ties: lower rank)
    int src = 0;
    for (int r = 1; r < R; ++r)
      if (lat[r] > lat[src]) src = r;
    int dst = -1;
    for (int r = 0; r < R; ++r) {
      if (r == src || ((invalid[src] >> r) & 1u)) continue;
      if (dst < 0 || lat[r] < lat[dst]) dst = r;
    }
    if (dst < 0) break;

    // SelectHeavyExpert: most tokens on src among the experts src holds, dst does not, with something to move
    if (tid == 0) best_key = -1;
    __syncthreads();
    if (tid < E) {
      const uint32_t hm = hostmask[tid];
      if (((hm >> src) & 1u) && !((hm >> dst) & 1u)) {
        long long movable = 0;
        for (int rs = 0; rs < R; ++rs)
          if (rs == dst || !((hm >> rs) & 1u)) movable += g_n[(tid * R + rs) * R + src];
        if (movable > 0)
          atomicMax(&best_key, (static_cast<long long>(ner[tid][src]) << 9) | static_cast<long long>(511 - tid));
      }
    }
    __syncthreads();
    const long long bk = best_key;
    // dual-side budget check (an empty selection is treated the same way)
    if (bk < 0 || n_out[src] >= a.budget || n_in[dst] >= cap_in) {
      __syncthreads();  // everybody has read invalid[] and best_key
      if (tid == 0) invalid[src] |= 1u << dst;
      __syncthreads();
      continue;
    }
    const int es = 511 - static_cast<int>(bk & 511);

    // WaterFillingRebalance on the expert's slab
    if (tid < R * R) slab_new[tid / R][tid % R] = slab_old[tid / R][tid % R] = g_n[es * R * R + tid];
    __syncthreads();
    if (tid == 0) {
      const uint32_t hm = hostmask[es];
      for (int rt = 0; rt < R; ++rt) {  // locality first: dst's own tokens come home
        if (rt == dst) continue;
        slab_new[dst][dst] += slab_new[dst][rt];
        slab_new[dst][rt] = 0;
      }
      long long want = static_cast<long long>(load[src]) - slab_old[dst][src] - avg;
      for (int rs = 0; rs < R && want > 0; ++rs) {  // origins without a copy, ascending rank
        if (rs == dst || ((hm >> rs) & 1u)) continue;
        const long long mv = min(static_cast<long long>(slab_new[rs][src]), want);
        slab_new[rs][src] -= static_cast<int>(mv);
        slab_new[rs][dst] += static_cast<int>(mv);
        want -= mv;
      }
    }
    __syncthreads();
    if (tid < R) {  // what the move does to rank tid
      const int r = tid;
      long long o_ner = 0, n_ner = 0, o_in = 0, n_inv = 0, o_out = 0, n_outv = 0;
      for (int q = 0; q < R; ++q) {
        o_ner += slab_old[q][r];
        n_ner += slab_new[q][r];
        if (q != r) {
          o_in += slab_old[q][r];
          n_inv += slab_new[q][r];
          o_out += slab_old[r][q];
          n_outv += slab_new[r][q];
        }
      }
      t_comp[r] = static_cast<long long>(comp[r]) - comp_term(o_ner, a.n0) + comp_term(n_ner, a.n0);
      t_vin[r] = static_cast<long long>(vin[r]) - o_in + n_inv;
      t_vout[r] = static_cast<long long>(vout[r]) - o_out + n_outv;
      t_load[r] = static_cast<long long>(load[r]) - o_ner + n_ner;
      t_lat[r] = a.g_den * t_comp[r] + 2 * a.g_num * max(t_vin[r], t_vout[r]);
    }
    __syncthreads();
    long long mx_old = lat[0], mx_new = t_lat[0];
    for (int r = 1; r < R; ++r) {
      mx_old = max(mx_old, lat[r]);
      mx_new = max(mx_new, t_lat[r]);
    }
    if (mx_old - mx_new <= a.eps || k >= a.k_max) break;  // converged, or the iteration budget is used up
    __syncthreads();  // every thread has read lat[] before it is overwritten

    // accept the move
    if (tid < R * R) g_n[es * R * R + tid] = slab_new[tid / R][tid % R];
    if (tid < R) {
      int s = 0;
      for (int q = 0; q < R; ++q) s += slab_new[q][tid];
      ner[es][tid] = s;
      comp[tid] = static_cast<unsigned long long>(t_comp[tid]);
      vin[tid] = static_cast<unsigned long long>(t_vin[tid]);
      vout[tid] = static_cast<unsigned long long>(t_vout[tid]);
      load[tid] = static_cast<unsigned long long>(t_load[tid]);
      lat[tid] = t_lat[tid];
    }
    if (tid == 0) {
      if (delta_out) delta_out[src * a.budget + n_out[src]] = es;
      delta_in[dst * a.max_replicas + n_in[dst]] = es;
      d_in[dst][n_in[dst]] = es;
      n_out[src] += 1;
      n_in[dst] += 1;
      hostmask[es] |= 1u << dst;
      moves[3 * k] = es;
      moves[3 * k + 1] = src;
      moves[3 * k + 2] = dst;
    }
    k += 1;
    __syncthreads();
  }
  __syncthreads();

  // ---- outputs
  if (tid == 0) {
    long long mx = 0, ml = 0;
    for (int r = 0; r < R; ++r) {
      mx = r == 0 ? lat[r] : max(mx, lat[r]);
      ml = max(ml, static_cast<long long>(load[r]));
    }
    stats[0] = lat_before;
    stats[1] = mx;
    stats[2] = ml;
    stats[3] = k;
  }
  const int rank = a.rank, S = E_loc + a.max_replicas;
  for (int s = tid; s < S; s += 256) {
    int e = -1;
    if (s < E_loc) {
      e = rank * E_loc + s;
      if (e >= E) e = -1;
    } else {
      e = d_in[rank][s - E_loc];
    }
    slot_expert[s] = e;
  }
  // the plan as `rank` sees it: one replica per holding rank in ascending rank order, weights = planned tokens
  const int cnt = tid < E ? __popc(hostmask[tid]) : 0;
  int incl = cnt;
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    int o = __shfl_up(incl, d, kWave);
    if (lane >= d) incl += o;
  }
  if (lane == kWave - 1) wave_tot[tid >> 6] = incl;
  __syncthreads();
  int pos = incl - cnt;
  for (int i = 0; i < (tid >> 6); ++i) pos += wave_tot[i];
  if (tid < E) {
    const int e = tid, home = e / E_loc;
    const uint32_t hm = hostmask[e];
    rep_off[e] = pos;
    long long planned = 0;
    int home_pos = pos;
    for (int r = 0; r < R; ++r) {
      if (!((hm >> r) & 1u)) continue;
      int slot = -1;
      if (r == rank) {
        if (r == home) {
          slot = e - r * E_loc;
        } else {
          for (int i = 0; i < a.max_replicas; ++i)
            if (d_in[r][i] == e) slot = E_loc + i;
        }
      }
      if (r == home) home_pos = pos;
      rep_slot[pos] = slot;
      rep_weight[pos] = ner[e][r];
      planned += ner[e][r];
      pos += 1;
    }
    if (planned == 0) rep_weight[home_pos] = 1;  // nothing predicted: unforeseen tokens go home
    if (e == E - 1) rep_off[E] = pos;
  }
  if (n_assign) {
    for (int i = tid; i < R * E * R; i += 256) {
      const int rs = i / (E * R), e = (i / R) % E, rt = i % R;
      n_assign[i] = g_n[(e * R + rs) * R + rt];
    }
  }
}

// The plan as source rank `rank` applies it to its own tokens: one slot per (destination rank, expert
// copy), numbered by rank first and expert second.  One workgroup; thread e finds the ranks that hold
// expert e (home + the replicas listed in delta_in); per rank, wave ballots and per-wave totals give the
// number of lower experts held there (the slot inside the rank) and the rank's slot count; a block scan
// of the copies per expert gives rep_off.
__global__ __launch_bounds__(256) void plan_dispatch_kernel(const int32_t* __restrict__ n_assign,
                                                            const int32_t* __restrict__ delta_in, int R, int E,
                                                            int E_loc, int max_replicas, int rank,
                                                            int32_t* __restrict__ rep_off,
                                                            int32_t* __restrict__ rep_slot,
                                                            int32_t* __restrict__ rep_weight,
                                                            int32_t* __restrict__ rank_off,
                                                            int32_t* __restrict__ slot_expert) {
  __shared__ int32_t wave_tot[4];
  __shared__ int32_t wave_cnt[kPlanMaxRanks][4];
  __shared__ int32_t r_off[kPlanMaxRanks + 1];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, e = tid;
  uint32_t hm = 0;
  if (e < E) {
    hm = 1u << (e / E_loc);
    for (int r = 0; r < R; ++r)
      for (int i = 0; i < max_replicas; ++i)
        if (delta_in[r * max_replicas + i] == e) hm |= 1u << r;
  }
  const uint64_t lower = lane == 0 ? 0ull : (~0ull >> (64 - lane));
  int within[kPlanMaxRanks];  // experts below e, in this wave, held by rank r
#pragma unroll
  for (int r = 0; r < kPlanMaxRanks; ++r) {
    const uint64_t m = __ballot((hm >> r) & 1u);
    within[r] = __popcll(m & lower);
    if (lane == 0) wave_cnt[r][wv] = __popcll(m);
  }
  const int cnt = __popc(hm);
  int incl = cnt;
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    int o = __shfl_up(incl, d, kWave);
    if (lane >= d) incl += o;
  }
  if (lane == kWave - 1) wave_tot[wv] = incl;
  __syncthreads();
  if (tid == 0) {
    int run = 0;
    for (int r = 0; r < R; ++r) {
      r_off[r] = run;
      rank_off[r] = run;
      run += wave_cnt[r][0] + wave_cnt[r][1] + wave_cnt[r][2] + wave_cnt[r][3];
    }
    r_off[R] = run;
    rank_off[R] = run;
  }
  __syncthreads();
  int pos = incl - cnt;
  for (int i = 0; i < wv; ++i) pos += wave_tot[i];
  if (e < E) {
    const int home = e / E_loc;
    rep_off[e] = pos;
    long long planned = 0;
    int home_pos = pos, own_pos = -1;
#pragma unroll
    for (int r = 0; r < kPlanMaxRanks; ++r) {
      if (r < R && ((hm >> r) & 1u)) {
        int slot = r_off[r] + within[r];
        for (int i = 0; i < wv; ++i) slot += wave_cnt[r][i];
        const int w = n_assign[(static_cast<long>(rank) * E + e) * R + r];
        if (r == home) home_pos = pos;
        if (r == rank) own_pos = pos;
        rep_slot[pos] = slot;
        rep_weight[pos] = w;
        slot_expert[slot] = e;
        planned += w;
        pos += 1;
      }
    }
    // nothing predicted from this origin: an unforeseen token stays here if a copy is here, else goes home
    if (planned == 0) rep_weight[own_pos >= 0 ? own_pos : home_pos] = 1;
    if (e == E - 1) rep_off[E] = pos;
  }
}

}  // namespace probe

extern "C" int probe_plan_dispatch(const int32_t* n_assign, const int32_t* delta_in, int R, int E, int E_loc,
                                   int max_replicas, int rank, int32_t* rep_off, int32_t* rep_slot,
                                   int32_t* rep_weight, int32_t* rank_off, int32_t* slot_expert, void* stream) {
  using namespace probe;
  PROBE_REQUIRE(R >= 1 && E >= 1 && E_loc >= 1 && static_cast<long>(E_loc) * R >= E && rank >= 0 && rank < R &&
                    max_replicas >= 0,
                PROBE_EINVAL, "probe_plan_dispatch: bad dims R=%d E=%d E_loc=%d rank=%d max_replicas=%d", R, E, E_loc,
                rank, max_replicas);
  PROBE_REQUIRE(R <= kPlanMaxRanks && E <= PROBE_MAX_EXPERTS && max_replicas <= kPlanMaxReplicas, PROBE_EUNSUPPORTED,
                "probe_plan_dispatch: needs R <= %d, E <= %d, max_replicas <= %d", kPlanMaxRanks, PROBE_MAX_EXPERTS,
                kPlanMaxReplicas);
  PROBE_REQUIRE(n_assign && (delta_in || max_replicas == 0) && rep_off && rep_slot && rep_weight && rank_off &&
                    slot_expert,
                PROBE_EINVAL, "probe_plan_dispatch: null pointer");
  hipLaunchKernelGGL(plan_dispatch_kernel, dim3(1), dim3(256), 0, static_cast<hipStream_t>(stream), n_assign,
                     delta_in, R, E, E_loc, max_replicas, rank, rep_off, rep_slot, rep_weight, rank_off, slot_expert);
  return check_launch("probe_plan_dispatch");
}

extern "C" size_t probe_plan_greedy_workspace_bytes(int R, int E) {
  if (R <= 0 || E <= 0) return 0;
  return probe::align_up(static_cast<size_t>(E) * R * R * sizeof(int32_t), 256);
}

extern "C" int probe_plan_greedy(const int32_t* n_hat, int R, int E, int E_loc, int rank,
                                 const probe_planner_params* params, int32_t* rep_off, int32_t* rep_slot,
                                 int32_t* rep_weight, int32_t* slot_expert, int32_t* delta_in,
                                 int32_t* delta_out, int32_t* moves, int64_t* stats, int32_t* n_assign,
                                 void* workspace, size_t workspace_bytes, void* stream) {
  using namespace probe;
  PROBE_REQUIRE(params != nullptr, PROBE_EINVAL, "probe_plan_greedy: params is NULL");
  PROBE_REQUIRE(R >= 1 && E >= 1 && E_loc >= 1 && static_cast<long>(E_loc) * R >= E && rank >= 0 && rank < R,
                PROBE_EINVAL, "probe_plan_greedy: bad dims R=%d E=%d E_loc=%d rank=%d", R, E, E_loc, rank);
  PROBE_REQUIRE(params->max_replicas >= 0 && params->budget >= 0 && params->k_max >= 0 && params->g_den >= 1 &&
                    params->g_num >= 0 && params->n0 >= 0,
                PROBE_EINVAL, "probe_plan_greedy: bad parameters");
  PROBE_REQUIRE(R <= kPlanMaxRanks && E <= PROBE_MAX_EXPERTS && params->max_replicas <= kPlanMaxReplicas &&
                    params->budget <= kPlanMaxReplicas && params->k_max <= kPlanMaxMoves,
                PROBE_EUNSUPPORTED,
                "probe_plan_greedy: needs R <= %d, E <= %d, max_replicas <= %d, budget <= %d, k_max <= %d",
                kPlanMaxRanks, PROBE_MAX_EXPERTS, kPlanMaxReplicas, kPlanMaxReplicas, kPlanMaxMoves);
  PROBE_REQUIRE(n_hat && rep_off && rep_slot && rep_weight && slot_expert && stats &&
                    (delta_in || params->max_replicas == 0) && (moves || params->k_max == 0),
                PROBE_EINVAL, "probe_plan_greedy: null pointer");
  PROBE_REQUIRE(workspace && workspace_bytes >= probe_plan_greedy_workspace_bytes(R, E), PROBE_EWORKSPACE,
                "probe_plan_greedy: workspace too small (%zu < %zu)", workspace_bytes,
                probe_plan_greedy_workspace_bytes(R, E));
  PlannerArgs a;
  a.R = R; a.E = E; a.E_loc = E_loc; a.rank = rank;
  a.max_replicas = params->max_replicas; a.budget = params->budget; a.k_max = params->k_max;
  a.eps = params->eps; a.n0 = params->n0; a.g_num = params->g_num; a.g_den = params->g_den;
  hipLaunchKernelGGL(plan_greedy_kernel, dim3(1), dim3(256), 0, static_cast<hipStream_t>(stream), n_hat, a,
                     static_cast<int32_t*>(workspace), rep_off, rep_slot, rep_weight, slot_expert, delta_in, delta_out,
                     moves, reinterpret_cast<long long*>(stats), n_assign);
  return check_launch("probe_plan_greedy");
}
