// probe_permute: plan-driven grouping of (token, top-k position) pairs by weight slot.
//
// The sequential definition (walk the pairs in order, the j-th arrival of an expert goes to a
// replica by weighted round-robin, append to the slot's list) is reproduced exactly without
// atomics: a pair's destination row follows from (expert e, arrival rank j) alone.
//
//   1. hist     each workgroup counts the experts of its own contiguous block of 1024 pairs
//               (wave ballots, LDS counters)                             -> blk_hist[U][E]
//   2. index    every workgroup sums the block histograms (its exclusive base = the blocks before it,
//               n_e = all blocks), derives the rows per replica in closed form and the prefix sum over
//               slots (workgroup 0 writes slot_counts, slot_offsets, n_local), then re-walks its block
//               (each wave a 256-pair segment, bases of the later waves from the earlier waves' counts),
//               ranks each pair among equal experts with wave ballots and computes slot and row
//               analytically                                             -> pair_row, row_pair
//   3. scatter  one thread per 16-byte chunk of a token row: read x once, write it to each of
//               the token's local rows                                   -> xp
// A batch of at most 1024 pairs (decode) runs steps 1-2 as one workgroup in one launch; a batch of more than
// 262144 pairs runs step 2 as a one-workgroup scan kernel followed by the ranking kernel.
//
// Steps 1-2 touch only T*k integers; step 3 carries the HBM traffic (T*H*2 bytes read at
// most, n_local*H*2 written).
#include <mutex>

#include "common.hpp"

namespace probe {

constexpr int kPermWaves = 4;                 // waves per workgroup in steps 1 and 3
constexpr int kSegPairs = 256;                // pairs per wave segment
constexpr int kSegIters = kSegPairs / kWave;  // 4 wave-wide iterations per segment
constexpr int kRepLds = 2048;                 // replica-list entries staged in LDS by the index kernel
constexpr int kFusedBlocks = 256;             // up to this many blocks (262144 pairs) step 2 is one launch

__device__ __forceinline__ uint64_t lanemask_lt() {
  int l = lane_id();
  return l == 0 ? 0ull : (~0ull >> (64 - l));
}

// Lanes of the wave holding the same 8-bit key as this lane (inactive lanes excluded by
// passing valid = false; they get an empty mask).
__device__ __forceinline__ uint64_t match_key8(int key, bool valid) {
  uint64_t m = __ballot(valid);
#pragma unroll
  for (int b = 0; b < 8; ++b) {
    uint64_t bal = __ballot(valid && ((key >> b) & 1));
    m &= ((key >> b) & 1) ? bal : ~bal;
  }
  return valid ? m : 0ull;
}

// Step 1.
__global__ __launch_bounds__(kPermWaves* kWave) void permute_hist_kernel(
    const int32_t* __restrict__ topk_idx, int N, int E, int32_t* __restrict__ blk_hist) {
  __shared__ int32_t cnt_mem[kPermWaves][PROBE_MAX_EXPERTS];
  int w = threadIdx.x / kWave, lane = lane_id();
  volatile int32_t* cnt_w = cnt_mem[w];  // volatile: keep every lane's read before the leader's update
  for (int e = lane; e < E; e += kWave) cnt_w[e] = 0;
  long base = (static_cast<long>(blockIdx.x) * kPermWaves + w) * kSegPairs;
  // same-wave LDS accesses execute in program order; no barrier needed for a wave's own row
  for (int it = 0; it < kSegIters; ++it) {
    long p = base + it * kWave + lane;
    int e = p < N ? topk_idx[p] : -1;
    bool valid = static_cast<unsigned>(e) < static_cast<unsigned>(E);  // bad ids count nowhere
    uint64_t m = match_key8(e, valid);
    if (valid && (m & lanemask_lt()) == 0) cnt_w[e] += __popcll(m);
  }
  __syncthreads();
  for (int e = threadIdx.x; e < E; e += kPermWaves * kWave) {
    int tot = 0;
#pragma unroll
    for (int q = 0; q < kPermWaves; ++q) tot += cnt_mem[q][e];
    blk_hist[static_cast<long>(blockIdx.x) * E + e] = tot;
  }
}

// Steps 2a / 2b for batches of more than kFusedBlocks blocks, where every workgroup summing all block
// histograms itself would cost more than a scan kernel in between (the work of step 2 grows with the square
// of the number of blocks).
// 2a.  One workgroup of 1024 threads: expert e = tid % 256 is scanned by four threads, each over a quarter
// of the blocks (sum pass, then a pass that writes the exclusive bases).
__global__ __launch_bounds__(1024) void permute_scan_kernel(
    int32_t* __restrict__ seg_hist /* in: counts, out: exclusive bases */, int U, int E,
    const int32_t* __restrict__ rep_off, const int32_t* __restrict__ rep_slot,
    const int32_t* __restrict__ rep_weight, int S, int32_t* __restrict__ slot_counts,
    int32_t* __restrict__ slot_offsets, int32_t* __restrict__ n_local) {
  __shared__ int32_t sc[PROBE_MAX_SLOTS];
  __shared__ int32_t part_tot[4][PROBE_MAX_EXPERTS];
  __shared__ int32_t wave_tot[4];
  const int tid = threadIdx.x;
  const int e = tid & 255, part = tid >> 8;
  const int chunk = (U + 3) / 4;
  const int u0 = min(part * chunk, U), u1 = min(u0 + chunk, U);
  for (int s = tid; s < S; s += 1024) sc[s] = 0;
  // this expert's replica range, its total weight and its first replica are fetched now, under
  // the histogram passes
  int lo = 0, hi = 0, P = 0, w_first = 0, s_first = -1;
  if (part == 0 && e < E) {
    lo = rep_off[e];
    hi = rep_off[e + 1];
    for (int i = lo; i < hi; ++i) P += rep_weight[i];
    if (hi > lo) {
      w_first = rep_weight[lo];
      s_first = rep_slot[lo];
    }
  }
  int tot = 0;
  if (e < E) {
    int u = u0;
    for (; u + 16 <= u1; u += 16) {  // sixteen independent loads in flight
      int c[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) c[i] = seg_hist[static_cast<long>(u + i) * E + e];
#pragma unroll
      for (int i = 0; i < 16; ++i) tot += c[i];
    }
    for (; u < u1; ++u) tot += seg_hist[static_cast<long>(u) * E + e];
  }
  part_tot[part][e] = tot;
  __syncthreads();
  if (e < E) {
    int run = 0;
    for (int q = 0; q < part; ++q) run += part_tot[q][e];
    int u = u0;
    for (; u + 16 <= u1; u += 16) {
      int c[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) c[i] = seg_hist[static_cast<long>(u + i) * E + e];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        seg_hist[static_cast<long>(u + i) * E + e] = run;
        run += c[i];
      }
    }
    for (; u < u1; ++u) {
      long i = static_cast<long>(u) * E + e;
      int c = seg_hist[i];
      seg_hist[i] = run;
      run += c;
    }
  }
  if (part == 0 && e < E) {
    const int n_e = part_tot[0][e] + part_tot[1][e] + part_tot[2][e] + part_tot[3][e];
    // rows each replica of this expert receives: floor(n/P) w_i + clamp(n mod P - c_{i-1}, 0, w_i)
    if (P > 0) {
      int full = n_e / P, rem = n_e - full * P, cum = 0;
      for (int i = lo; i < hi; ++i) {
        int wgt = i == lo ? w_first : rep_weight[i];
        int part_rows = min(max(rem - cum, 0), wgt);
        int slot = i == lo ? s_first : rep_slot[i];
        if (slot >= 0 && slot < S) sc[slot] = full * wgt + part_rows;
        cum += wgt;
      }
    }
  }
  __syncthreads();
  // exclusive prefix sum over S <= 1024 slots: 4 consecutive slots per thread, first 256 threads
  int v[4] = {0, 0, 0, 0}, local = 0, incl = 0;
  if (tid < 256) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int s = tid * 4 + i;
      v[i] = s < S ? sc[s] : 0;
      local += v[i];
    }
    incl = local;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
      int o = __shfl_up(incl, d, kWave);
      if (lane_id() >= d) incl += o;
    }
    if (lane_id() == kWave - 1) wave_tot[tid / kWave] = incl;
  }
  __syncthreads();
  if (tid < 256) {
    int wave_base = 0;
    for (int i = 0; i < tid / kWave; ++i) wave_base += wave_tot[i];
    int excl = wave_base + incl - local;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int s = tid * 4 + i;
      if (s < S) {
        slot_counts[s] = v[i];
        slot_offsets[s] = excl;
      }
      excl += v[i];
    }
    if (tid == 255) {
      slot_offsets[S] = excl;
      n_local[0] = excl;
    }
  }
}

// 2b.  Ranks and rows of a block from the exclusive bases and slot offsets written by 2a.
__global__ __launch_bounds__(kPermWaves* kWave) void permute_index_kernel(
    const int32_t* __restrict__ topk_idx, int N, int E, const int32_t* __restrict__ blk_base,
    const int32_t* __restrict__ rep_off, const int32_t* __restrict__ rep_slot,
    const int32_t* __restrict__ rep_weight, const int32_t* __restrict__ slot_offsets, int S,
    int32_t* __restrict__ pair_row, int32_t* __restrict__ row_pair) {
  __shared__ int32_t cnt_mem[kPermWaves][PROBE_MAX_EXPERTS];
  __shared__ int32_t e_lo[PROBE_MAX_EXPERTS], e_hi[PROBE_MAX_EXPERTS], e_P[PROBE_MAX_EXPERTS];
  __shared__ int32_t s_off[PROBE_MAX_SLOTS + 1];
  __shared__ int32_t s_rw[kRepLds], s_rs[kRepLds];
  int w = threadIdx.x / kWave, lane = lane_id();
  volatile int32_t* cnt_w = cnt_mem[w];  // volatile: keep every lane's read before the leader's update
  long base = (static_cast<long>(blockIdx.x) * kPermWaves + w) * kSegPairs;
  // every global load that depends on nothing is issued first, so that their latencies overlap:
  // this wave's pairs, the block's bases, the size of the replica list
  int seg_e[kSegIters];
#pragma unroll
  for (int it = 0; it < kSegIters; ++it) {
    long p = base + it * kWave + lane;
    seg_e[it] = p < N ? topk_idx[p] : -1;
  }
  int start[PROBE_MAX_EXPERTS / kWave];
#pragma unroll
  for (int i = 0; i < PROBE_MAX_EXPERTS / kWave; ++i) {
    int e = lane + i * kWave;
    start[i] = e < E ? blk_base[static_cast<long>(blockIdx.x) * E + e] : 0;
  }
  const int R = rep_off[E];
  // the plan, once per workgroup: replica lists (in LDS when they fit), replica range and total
  // weight of every expert, slot offsets
  const bool staged = R <= kRepLds;
  if (staged)
    for (int i = threadIdx.x; i < R; i += kPermWaves * kWave) {
      s_rw[i] = rep_weight[i];
      s_rs[i] = rep_slot[i];
    }
  const int32_t* rw = staged ? s_rw : rep_weight;  // flat pointers: LDS or global
  const int32_t* rs = staged ? s_rs : rep_slot;
  for (int e = threadIdx.x; e < E; e += kPermWaves * kWave) {
    e_lo[e] = rep_off[e];
    e_hi[e] = rep_off[e + 1];
  }
  for (int i = threadIdx.x; i <= S; i += kPermWaves * kWave) s_off[i] = slot_offsets[i];
  // counts of this wave's own segment (the same walk as in step 1)
  for (int e = lane; e < E; e += kWave) cnt_w[e] = 0;
#pragma unroll
  for (int it = 0; it < kSegIters; ++it) {
    int e = seg_e[it];
    bool valid = static_cast<unsigned>(e) < static_cast<unsigned>(E);
    uint64_t m = match_key8(e, valid);
    if (valid && (m & lanemask_lt()) == 0) cnt_w[e] += __popcll(m);
  }
  __syncthreads();
  // total weight of every expert, from the staged list when there is one
  for (int e = threadIdx.x; e < E; e += kPermWaves * kWave) {
    int P = 0;
    for (int i = e_lo[e]; i < e_hi[e]; ++i) P += rw[i];
    e_P[e] = P;
  }
  // arrival rank at the start of this wave's segment: block base + counts of the earlier waves
#pragma unroll
  for (int i = 0; i < PROBE_MAX_EXPERTS / kWave; ++i) {
    int e = lane + i * kWave;
    if (e < E)
      for (int q = 0; q < w; ++q) start[i] += cnt_mem[q][e];
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < PROBE_MAX_EXPERTS / kWave; ++i) {
    int e = lane + i * kWave;
    if (e < E) cnt_w[e] = start[i];
  }
  int n_loc = s_off[S];
#pragma unroll
  for (int it = 0; it < kSegIters; ++it) {
    long p = base + it * kWave + lane;
    int e = seg_e[it];
    bool valid = static_cast<unsigned>(e) < static_cast<unsigned>(E);
    uint64_t m = match_key8(e, valid);
    if (p < N && !valid) {  // expert id out of range: the pair is computed nowhere on this GPU
      pair_row[p] = -1;
      if (p >= n_loc) row_pair[p] = -1;
    }
    if (valid) {
      int before = __popcll(m & lanemask_lt());
      int j = cnt_w[e] + before;                       // arrival rank of this pair for expert e
      int lo = e_lo[e], hi = e_hi[e], P = e_P[e];
      int row = -1;
      if (P > 0) {
        int full = j / P, u = j - full * P, cum = 0;
        for (int i = lo; i < hi; ++i) {
          int wgt = rw[i];
          if (u < cum + wgt) {
            int slot = rs[i];
            if (slot >= 0 && slot < S) row = s_off[slot] + full * wgt + (u - cum);
            if (row >= N) row = -1;  // only an inconsistent plan (two replicas in one slot) gets here
            break;
          }
          cum += wgt;
        }
      }
      pair_row[p] = row;
      if (row >= 0) row_pair[row] = static_cast<int32_t>(p);
      if (p >= n_loc) row_pair[p] = -1;
    }
    // all lanes of a key have read the counter above; the key's first lane now advances it
    if (valid && (m & lanemask_lt()) == 0) cnt_w[e] += __popcll(m);
  }
}

// Steps 1-2 in one workgroup, for batches of at most 1024 pairs (decode): the block histogram is the
// global one, so the scan over blocks disappears and the whole index computation is one launch.
__global__ __launch_bounds__(kPermWaves* kWave) void permute_small_kernel(
    const int32_t* __restrict__ topk_idx, int N, int E, const int32_t* __restrict__ rep_off,
    const int32_t* __restrict__ rep_slot, const int32_t* __restrict__ rep_weight, int S,
    int32_t* __restrict__ slot_counts, int32_t* __restrict__ slot_offsets, int32_t* __restrict__ n_local,
    int32_t* __restrict__ pair_row, int32_t* __restrict__ row_pair) {
  __shared__ int32_t cnt_mem[kPermWaves][PROBE_MAX_EXPERTS];
  __shared__ int32_t e_lo[PROBE_MAX_EXPERTS], e_hi[PROBE_MAX_EXPERTS], e_P[PROBE_MAX_EXPERTS];
  __shared__ int32_t s_off[PROBE_MAX_SLOTS + 1], sc[PROBE_MAX_SLOTS];
  __shared__ int32_t s_rw[kRepLds], s_rs[kRepLds];
  __shared__ int32_t wave_tot[kPermWaves];
  const int tid = threadIdx.x, w = tid / kWave, lane = lane_id();
  volatile int32_t* cnt_w = cnt_mem[w];  // volatile: keep every lane's read before the leader's update
  const long base = static_cast<long>(w) * kSegPairs;
  // The kernel is a chain of dependent global loads, so every load that depends on nothing is issued first: the
  // segment's expert ids, the size of the replica list and this thread's replica range (E <= 256 = threads).
  static_assert(kPermWaves * kWave >= PROBE_MAX_EXPERTS, "one expert per thread");
  int seg_e[kSegIters];
#pragma unroll
  for (int it = 0; it < kSegIters; ++it) {
    const long p = base + it * kWave + lane;
    seg_e[it] = p < N ? topk_idx[p] : -1;
  }
  const int R = rep_off[E];
  int my_lo = 0, my_hi = 0;
  if (tid < E) {
    my_lo = rep_off[tid];
    my_hi = rep_off[tid + 1];
  }
  const bool staged = R <= kRepLds;
  if (staged)
    for (int i = tid; i < R; i += kPermWaves * kWave) {
      s_rw[i] = rep_weight[i];
      s_rs[i] = rep_slot[i];
    }
  const int32_t* rw = staged ? s_rw : rep_weight;
  const int32_t* rs = staged ? s_rs : rep_slot;
  if (tid < E) {
    int P = 0;
    for (int i = my_lo; i < my_hi; ++i) P += rep_weight[i];
    e_lo[tid] = my_lo;
    e_hi[tid] = my_hi;
    e_P[tid] = P;
  }
  for (int s = tid; s < S; s += kPermWaves * kWave) sc[s] = 0;
  // counts of this wave's segment
  for (int e = lane; e < E; e += kWave) cnt_w[e] = 0;
#pragma unroll
  for (int it = 0; it < kSegIters; ++it) {
    const int e = seg_e[it];
    bool valid = static_cast<unsigned>(e) < static_cast<unsigned>(E);
    uint64_t m = match_key8(e, valid);
    if (valid && (m & lanemask_lt()) == 0) cnt_w[e] += __popcll(m);
  }
  __syncthreads();
  // rows each replica receives: floor(n/P) w_i + clamp(n mod P - c_{i-1}, 0, w_i)
  for (int e = tid; e < E; e += kPermWaves * kWave) {
    int n_e = 0;
#pragma unroll
    for (int q = 0; q < kPermWaves; ++q) n_e += cnt_mem[q][e];
    const int P = e_P[e];
    if (P > 0) {
      int full = n_e / P, rem = n_e - full * P, cum = 0;
      for (int i = e_lo[e]; i < e_hi[e]; ++i) {
        int wgt = rw[i];
        int part_rows = min(max(rem - cum, 0), wgt);
        int slot = rs[i];
        if (slot >= 0 && slot < S) sc[slot] = full * wgt + part_rows;
        cum += wgt;
      }
    }
  }
  __syncthreads();
  // exclusive prefix sum over the slots, 4 consecutive slots per thread
  int v[4], local = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int s = tid * 4 + i;
    v[i] = s < S ? sc[s] : 0;
    local += v[i];
  }
  int incl = local;
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    int o = __shfl_up(incl, d, kWave);
    if (lane >= d) incl += o;
  }
  if (lane == kWave - 1) wave_tot[w] = incl;
  __syncthreads();
  {
    int excl = incl - local;
    for (int i = 0; i < w; ++i) excl += wave_tot[i];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int s = tid * 4 + i;
      if (s < S) {
        slot_counts[s] = v[i];
        slot_offsets[s] = excl;
        s_off[s] = excl;
      }
      excl += v[i];
    }
    if (tid == kPermWaves * kWave - 1) {
      slot_offsets[S] = excl;
      n_local[0] = excl;
      s_off[S] = excl;
    }
  }
  // arrival rank at the start of this wave's segment = counts of the earlier waves
  int start[PROBE_MAX_EXPERTS / kWave];
#pragma unroll
  for (int i = 0; i < PROBE_MAX_EXPERTS / kWave; ++i) {
    int e = lane + i * kWave;
    int a = 0;
    if (e < E)
      for (int q = 0; q < w; ++q) a += cnt_mem[q][e];
    start[i] = a;
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < PROBE_MAX_EXPERTS / kWave; ++i) {
    int e = lane + i * kWave;
    if (e < E) cnt_w[e] = start[i];
  }
  const int n_loc = s_off[S];
#pragma unroll
  for (int it = 0; it < kSegIters; ++it) {
    long p = base + it * kWave + lane;
    int e = seg_e[it];
    bool valid = static_cast<unsigned>(e) < static_cast<unsigned>(E);
    uint64_t m = match_key8(e, valid);
    if (p < N && !valid) {  // expert id out of range: the pair is computed nowhere on this GPU
      pair_row[p] = -1;
      if (p >= n_loc) row_pair[p] = -1;
    }
    if (valid) {
      int before = __popcll(m & lanemask_lt());
      int j = cnt_w[e] + before;
      int lo = e_lo[e], hi = e_hi[e], P = e_P[e];
      int row = -1;
      if (P > 0) {
        int full = j / P, u = j - full * P, cum = 0;
        for (int i = lo; i < hi; ++i) {
          int wgt = rw[i];
          if (u < cum + wgt) {
            int slot = rs[i];
            if (slot >= 0 && slot < S) row = s_off[slot] + full * wgt + (u - cum);
            if (row >= N) row = -1;
            break;
          }
          cum += wgt;
        }
      }
      pair_row[p] = row;
      if (row >= 0) row_pair[row] = static_cast<int32_t>(p);
      if (p >= n_loc) row_pair[p] = -1;
    }
    if (valid && (m & lanemask_lt()) == 0) cnt_w[e] += __popcll(m);
  }
}

// Step 2: every workgroup sums the block histograms itself (its own exclusive base =
// the blocks before it, the totals n_e = all blocks), derives the slot counts and offsets from the totals
// (each workgroup redundantly, workgroup 0 writes them out) and then ranks its own 1024 pairs as above.
// Reading U*E counters per workgroup costs less than a one-workgroup scan kernel between two launches.
__global__ __launch_bounds__(kPermWaves* kWave) void permute_scan_index_kernel(
    const int32_t* __restrict__ topk_idx, int N, int E, const int32_t* __restrict__ blk_hist, int U,
    const int32_t* __restrict__ rep_off, const int32_t* __restrict__ rep_slot,
    const int32_t* __restrict__ rep_weight, int S, int32_t* __restrict__ slot_counts,
    int32_t* __restrict__ slot_offsets, int32_t* __restrict__ n_local, int32_t* __restrict__ pair_row,
    int32_t* __restrict__ row_pair) {
  __shared__ int32_t cnt_mem[kPermWaves][PROBE_MAX_EXPERTS];
  __shared__ int32_t before_mem[kPermWaves][PROBE_MAX_EXPERTS], total_mem[kPermWaves][PROBE_MAX_EXPERTS];
  __shared__ int32_t e_lo[PROBE_MAX_EXPERTS], e_hi[PROBE_MAX_EXPERTS], e_P[PROBE_MAX_EXPERTS];
  __shared__ int32_t s_off[PROBE_MAX_SLOTS + 1], sc[PROBE_MAX_SLOTS];
  __shared__ int32_t s_rw[kRepLds], s_rs[kRepLds];
  __shared__ int32_t wave_tot[kPermWaves];
  const int tid = threadIdx.x, w = tid / kWave, lane = lane_id();
  const int b = blockIdx.x;
  volatile int32_t* cnt_w = cnt_mem[w];  // volatile: keep every lane's read before the leader's update
  const long base = (static_cast<long>(b) * kPermWaves + w) * kSegPairs;
  // loads that depend on nothing first: this wave's pairs, the size of the replica list
  int seg_e[kSegIters];
#pragma unroll
  for (int it = 0; it < kSegIters; ++it) {
    long p = base + it * kWave + lane;
    seg_e[it] = p < N ? topk_idx[p] : -1;
  }
  const int R = rep_off[E];
  // block histograms: wave w adds the blocks u = w, w + 4, ... for the experts lane, lane + 64, ...
  {
    int before[PROBE_MAX_EXPERTS / kWave], total[PROBE_MAX_EXPERTS / kWave];
#pragma unroll
    for (int i = 0; i < PROBE_MAX_EXPERTS / kWave; ++i) before[i] = total[i] = 0;
    constexpr int kBatch = 16;  // blocks per wave whose loads are in flight together (64 blocks per round)
    for (int u0 = w; u0 < U; u0 += kBatch * kPermWaves) {
      int c[kBatch][PROBE_MAX_EXPERTS / kWave];
#pragma unroll
      for (int q = 0; q < kBatch; ++q) {
        const int u = u0 + q * kPermWaves;
#pragma unroll
        for (int i = 0; i < PROBE_MAX_EXPERTS / kWave; ++i) {
          const int e = lane + i * kWave;
          c[q][i] = (u < U && e < E) ? blk_hist[static_cast<long>(u) * E + e] : 0;
        }
      }
#pragma unroll
      for (int q = 0; q < kBatch; ++q) {
        const int u = u0 + q * kPermWaves;
#pragma unroll
        for (int i = 0; i < PROBE_MAX_EXPERTS / kWave; ++i) {
          total[i] += c[q][i];
          before[i] += u < b ? c[q][i] : 0;
        }
      }
    }
#pragma unroll
    for (int i = 0; i < PROBE_MAX_EXPERTS / kWave; ++i) {
      before_mem[w][lane + i * kWave] = before[i];
      total_mem[w][lane + i * kWave] = total[i];
    }
  }
  const bool staged = R <= kRepLds;
  if (staged)
    for (int i = tid; i < R; i += kPermWaves * kWave) {
      s_rw[i] = rep_weight[i];
      s_rs[i] = rep_slot[i];
    }
  const int32_t* rw = staged ? s_rw : rep_weight;
  const int32_t* rs = staged ? s_rs : rep_slot;
  for (int e = tid; e < E; e += kPermWaves * kWave) {
    e_lo[e] = rep_off[e];
    e_hi[e] = rep_off[e + 1];
  }
  for (int s = tid; s < S; s += kPermWaves * kWave) sc[s] = 0;
  // counts of this wave's own segment (the same walk as in step 1)
  for (int e = lane; e < E; e += kWave) cnt_w[e] = 0;
#pragma unroll
  for (int it = 0; it < kSegIters; ++it) {
    int e = seg_e[it];
    bool valid = static_cast<unsigned>(e) < static_cast<unsigned>(E);
    uint64_t m = match_key8(e, valid);
    if (valid && (m & lanemask_lt()) == 0) cnt_w[e] += __popcll(m);
  }
  __syncthreads();
  // rows each replica receives: floor(n/P) w_i + clamp(n mod P - c_{i-1}, 0, w_i)
  for (int e = tid; e < E; e += kPermWaves * kWave) {
    int n_e = 0, P = 0;
#pragma unroll
    for (int q = 0; q < kPermWaves; ++q) n_e += total_mem[q][e];
    for (int i = e_lo[e]; i < e_hi[e]; ++i) P += rw[i];
    e_P[e] = P;
    if (P > 0) {
      int full = n_e / P, rem = n_e - full * P, cum = 0;
      for (int i = e_lo[e]; i < e_hi[e]; ++i) {
        int wgt = rw[i];
        int part_rows = min(max(rem - cum, 0), wgt);
        int slot = rs[i];
        if (slot >= 0 && slot < S) sc[slot] = full * wgt + part_rows;
        cum += wgt;
      }
    }
  }
  __syncthreads();
  // exclusive prefix sum over the slots, 4 consecutive slots per thread
  int v[4], local = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int s = tid * 4 + i;
    v[i] = s < S ? sc[s] : 0;
    local += v[i];
  }
  int incl = local;
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    int o = __shfl_up(incl, d, kWave);
    if (lane >= d) incl += o;
  }
  if (lane == kWave - 1) wave_tot[w] = incl;
  __syncthreads();
  {
    int excl = incl - local;
    for (int i = 0; i < w; ++i) excl += wave_tot[i];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int s = tid * 4 + i;
      if (s < S) {
        if (b == 0) {
          slot_counts[s] = v[i];
          slot_offsets[s] = excl;
        }
        s_off[s] = excl;
      }
      excl += v[i];
    }
    if (tid == kPermWaves * kWave - 1) {
      if (b == 0) {
        slot_offsets[S] = excl;
        n_local[0] = excl;
      }
      s_off[S] = excl;
    }
  }
  // arrival rank at the start of this wave's segment: the blocks before this one + the earlier waves
  int start[PROBE_MAX_EXPERTS / kWave];
#pragma unroll
  for (int i = 0; i < PROBE_MAX_EXPERTS / kWave; ++i) {
    int e = lane + i * kWave;
    int a = 0;
    if (e < E) {
#pragma unroll
      for (int q = 0; q < kPermWaves; ++q) a += before_mem[q][e];
      for (int q = 0; q < w; ++q) a += cnt_mem[q][e];
    }
    start[i] = a;
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < PROBE_MAX_EXPERTS / kWave; ++i) {
    int e = lane + i * kWave;
    if (e < E) cnt_w[e] = start[i];
  }
  const int n_loc = s_off[S];
#pragma unroll
  for (int it = 0; it < kSegIters; ++it) {
    long p = base + it * kWave + lane;
    int e = seg_e[it];
    bool valid = static_cast<unsigned>(e) < static_cast<unsigned>(E);
    uint64_t m = match_key8(e, valid);
    if (p < N && !valid) {  // expert id out of range: the pair is computed nowhere on this GPU
      pair_row[p] = -1;
      if (p >= n_loc) row_pair[p] = -1;
    }
    if (valid) {
      int before = __popcll(m & lanemask_lt());
      int j = cnt_w[e] + before;                       // arrival rank of this pair for expert e
      int lo = e_lo[e], hi = e_hi[e], P = e_P[e];
      int row = -1;
      if (P > 0) {
        int full = j / P, u = j - full * P, cum = 0;
        for (int i = lo; i < hi; ++i) {
          int wgt = rw[i];
          if (u < cum + wgt) {
            int slot = rs[i];
            if (slot >= 0 && slot < S) row = s_off[slot] + full * wgt + (u - cum);
            if (row >= N) row = -1;  // only an inconsistent plan (two replicas in one slot) gets here
            break;
          }
          cum += wgt;
        }
      }
      pair_row[p] = row;
      if (row >= 0) row_pair[row] = static_cast<int32_t>(p);
      if (p >= n_loc) row_pair[p] = -1;
    }
    // all lanes of a key have read the counter above; the key's first lane now advances it
    if (valid && (m & lanemask_lt()) == 0) cnt_w[e] += __popcll(m);
  }
}

// Step 3.
template <int K>
__global__ __launch_bounds__(256) void permute_scatter_kernel(const u32x4* __restrict__ x,
                                                              const int32_t* __restrict__ pair_row,
                                                              long total_chunks, int chunks_per_row,
                                                              u32x4* __restrict__ xp) {
  long gid = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (gid >= total_chunks) return;
  int t = static_cast<int>(gid / chunks_per_row);
  int c = static_cast<int>(gid - static_cast<long>(t) * chunks_per_row);
  int rows[K];
  bool any = false;
#pragma unroll
  for (int s = 0; s < K; ++s) {
    rows[s] = pair_row[static_cast<long>(t) * K + s];
    any |= rows[s] >= 0;
  }
  if (!any) return;
  u32x4 v = __builtin_nontemporal_load(&x[gid]);
#pragma unroll
  for (int s = 0; s < K; ++s)
    if (rows[s] >= 0) __builtin_nontemporal_store(v, &xp[static_cast<long>(rows[s]) * chunks_per_row + c]);
}

static int num_blocks(long N) {
  const long per = static_cast<long>(kSegPairs) * kPermWaves;
  return static_cast<int>((N + per - 1) / per);
}

}  // namespace probe

extern "C" size_t probe_permute_workspace_bytes(int T, int E, int k, int S) {
  (void)S;
  if (T < 0 || E <= 0 || k <= 0) return 0;
  long N = static_cast<long>(T) * k;
  int U = probe::num_blocks(N);
  return probe::align_up(static_cast<size_t>(U > 0 ? U : 1) * E * sizeof(int32_t), 256);
}

namespace probe {

// Shared body of probe_permute (block histograms in the caller's workspace) and
// probe_permute_static (block histograms in the library's own static scratch array).
static int permute_impl(const char* name, const int32_t* topk_idx, const probe_plan* plan, const void* x_bf16,
                        int T, int H, int E, int k, int32_t* slot_counts, int32_t* slot_offsets,
                        int32_t* row_pair, int32_t* pair_row, void* xp_bf16, int32_t* n_local, int32_t* seg,
                        hipStream_t st) {
  const int S = plan->num_slots;
  int N = T * k;
  int U = num_blocks(N);
  int seg_blocks = U;
  if (U <= 1) {
    hipLaunchKernelGGL(permute_small_kernel, dim3(1), dim3(kPermWaves * kWave), 0, st, topk_idx, N, E,
                       plan->rep_off, plan->rep_slot, plan->rep_weight, S, slot_counts, slot_offsets, n_local,
                       pair_row, row_pair);
  } else {
    hipLaunchKernelGGL(permute_hist_kernel, dim3(seg_blocks), dim3(kPermWaves * kWave), 0, st, topk_idx, N, E,
                       seg);
    if (U <= kFusedBlocks) {
      hipLaunchKernelGGL(permute_scan_index_kernel, dim3(seg_blocks), dim3(kPermWaves * kWave), 0, st, topk_idx, N,
                         E, seg, U, plan->rep_off, plan->rep_slot, plan->rep_weight, S, slot_counts, slot_offsets,
                         n_local, pair_row, row_pair);
    } else {
      hipLaunchKernelGGL(permute_scan_kernel, dim3(1), dim3(1024), 0, st, seg, U, E, plan->rep_off,
                         plan->rep_slot, plan->rep_weight, S, slot_counts, slot_offsets, n_local);
      hipLaunchKernelGGL(permute_index_kernel, dim3(seg_blocks), dim3(kPermWaves * kWave), 0, st, topk_idx, N, E,
                         seg, plan->rep_off, plan->rep_slot, plan->rep_weight, slot_offsets, S, pair_row, row_pair);
    }
  }
  if (U > 0 && xp_bf16 != nullptr) {  // xp == NULL: the caller gathers rows on load instead
    int cpr = H / 8;
    long total = static_cast<long>(T) * cpr;
    unsigned grid = static_cast<unsigned>((total + 255) / 256);
    const u32x4* x = static_cast<const u32x4*>(x_bf16);
    u32x4* xp = static_cast<u32x4*>(xp_bf16);
#define PROBE_SCATTER_CASE(K) \
  case K: hipLaunchKernelGGL(permute_scatter_kernel<K>, dim3(grid), dim3(256), 0, st, x, pair_row, total, cpr, xp); break;
    switch (k) {
      PROBE_SCATTER_CASE(1) PROBE_SCATTER_CASE(2) PROBE_SCATTER_CASE(3) PROBE_SCATTER_CASE(4)
      PROBE_SCATTER_CASE(5) PROBE_SCATTER_CASE(6) PROBE_SCATTER_CASE(7) PROBE_SCATTER_CASE(8)
    }
#undef PROBE_SCATTER_CASE
  }
  return check_launch(name);
}

// Argument checks common to both entry points (everything but the scratch memory).
static int permute_check(const char* name, const int32_t* topk_idx, const probe_plan* plan, const void* x_bf16,
                         int T, int H, int E, int k, int32_t* slot_counts, int32_t* slot_offsets,
                         int32_t* row_pair, int32_t* pair_row, void* xp_bf16, int32_t* n_local) {
  PROBE_REQUIRE(T >= 0 && H > 0 && E > 0 && k > 0, PROBE_EINVAL, "%s: bad dims T=%d H=%d E=%d k=%d", name, T, H,
                E, k);
  PROBE_REQUIRE(plan != nullptr, PROBE_EINVAL, "%s: plan is NULL", name);
  int S = plan->num_slots;
  PROBE_REQUIRE(S >= 1, PROBE_EINVAL, "%s: plan->num_slots=%d", name, S);
  PROBE_REQUIRE(E <= PROBE_MAX_EXPERTS && k <= PROBE_MAX_TOPK && S <= PROBE_MAX_SLOTS && H % 8 == 0,
                PROBE_EUNSUPPORTED, "%s: needs E <= %d, k <= %d, S <= %d, H %% 8 == 0 (E=%d k=%d S=%d H=%d)", name,
                PROBE_MAX_EXPERTS, PROBE_MAX_TOPK, PROBE_MAX_SLOTS, E, k, S, H);
  PROBE_REQUIRE(static_cast<long>(T) * k < (1l << 31), PROBE_EUNSUPPORTED, "%s: T*k >= 2^31", name);
  PROBE_REQUIRE(plan->rep_off && plan->rep_slot && plan->rep_weight, PROBE_EINVAL, "%s: plan array is NULL", name);
  PROBE_REQUIRE(slot_counts && slot_offsets && n_local, PROBE_EINVAL, "%s: null output", name);
  PROBE_REQUIRE(T == 0 || (topk_idx && row_pair && pair_row && (xp_bf16 == nullptr || x_bf16)), PROBE_EINVAL,
                "%s: null pointer", name);
  PROBE_REQUIRE(aligned16(x_bf16) && aligned16(xp_bf16), PROBE_EALIGN, "%s: x/xp must be 16-byte aligned", name);
  return PROBE_OK;
}

}  // namespace probe

extern "C" int probe_permute(const int32_t* topk_idx, const probe_plan* plan, const void* x_bf16,
                             int T, int H, int E, int k, int32_t* slot_counts,
                             int32_t* slot_offsets, int32_t* row_pair, int32_t* pair_row,
                             void* xp_bf16, int32_t* n_local, void* workspace,
                             size_t workspace_bytes, void* stream) {
  using namespace probe;
  int rc = permute_check("probe_permute", topk_idx, plan, x_bf16, T, H, E, k, slot_counts, slot_offsets, row_pair,
                         pair_row, xp_bf16, n_local);
  if (rc != PROBE_OK) return rc;
  PROBE_REQUIRE(workspace && workspace_bytes >= probe_permute_workspace_bytes(T, E, k, plan->num_slots),
                PROBE_EWORKSPACE, "probe_permute: workspace too small (%zu < %zu)", workspace_bytes,
                probe_permute_workspace_bytes(T, E, k, plan->num_slots));
  return permute_impl("probe_permute", topk_idx, plan, x_bf16, T, H, E, k, slot_counts, slot_offsets, row_pair,
                      pair_row, xp_bf16, n_local, static_cast<int32_t*>(workspace),
                      static_cast<hipStream_t>(stream));
}

// ---- probe_permute_static: the same call for callers that cannot allocate ------------------
// The block histograms live in a file-scope device array instead of a caller-supplied workspace.
// Each GPU the library runs on holds its own copy of the array at its own address until the process
// ends; the address is looked up once per device (hipGetSymbolAddress, no allocation) and passed to
// the kernels like any workspace pointer.  The histogram kernel writes every entry the later kernels
// read, so nothing has to be cleared between calls.
namespace probe {

constexpr size_t kStaticScratchBytes = PROBE_PERMUTE_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) int32_t scratch[kStaticScratchBytes / sizeof(int32_t)];

static int static_scratch(int32_t** out) {
  static std::mutex mu;
  static int32_t* ptr_of[64] = {nullptr};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
    set_error("probe_permute_static: no current device");
    return PROBE_EHIP;
  }
  std::lock_guard<std::mutex> lock(mu);
  if (ptr_of[dev] == nullptr) {
    void* p = nullptr;
    hipError_t err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (err != hipSuccess || p == nullptr) {
      set_error("probe_permute_static: cannot locate the scratch array on device %d: %s", dev,
                hipGetErrorString(err));
      return PROBE_EHIP;
    }
    ptr_of[dev] = static_cast<int32_t*>(p);
  }
  *out = ptr_of[dev];
  return PROBE_OK;
}

}  // namespace probe

extern "C" size_t probe_permute_static_max_pairs(int E) {
  if (E <= 0 || E > PROBE_MAX_EXPERTS) return 0;
  const size_t blocks = probe::kStaticScratchBytes / (static_cast<size_t>(E) * sizeof(int32_t));
  return blocks * probe::kSegPairs * probe::kPermWaves;
}

extern "C" int probe_permute_static(const int32_t* topk_idx, const probe_plan* plan, const void* x_bf16, int T,
                                    int H, int E, int k, int32_t* slot_counts, int32_t* slot_offsets,
                                    int32_t* row_pair, int32_t* pair_row, void* xp_bf16, int32_t* n_local,
                                    void* stream) {
  using namespace probe;
  int rc = permute_check("probe_permute_static", topk_idx, plan, x_bf16, T, H, E, k, slot_counts, slot_offsets,
                         row_pair, pair_row, xp_bf16, n_local);
  if (rc != PROBE_OK) return rc;
  const size_t need = probe_permute_workspace_bytes(T, E, k, plan->num_slots);
  PROBE_REQUIRE(need <= kStaticScratchBytes, PROBE_EUNSUPPORTED,
                "probe_permute_static: T*k = %ld pairs with E = %d need %zu bytes of block histograms, the static "
                "scratch holds %zu (at most %zu pairs at this E); use probe_permute with a workspace",
                static_cast<long>(T) * k, E, need, kStaticScratchBytes, probe_permute_static_max_pairs(E));
  int32_t* seg = nullptr;
  rc = static_scratch(&seg);
  if (rc != PROBE_OK) return rc;
  return permute_impl("probe_permute_static", topk_idx, plan, x_bf16, T, H, E, k, slot_counts, slot_offsets,
                      row_pair, pair_row, xp_bf16, n_local, seg, static_cast<hipStream_t>(stream));
}
