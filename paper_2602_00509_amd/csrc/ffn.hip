// probe_grouped_ffn: grouped SwiGLU expert FFN on the bf16 matrix cores.
//
//   0. schedule  turn slot_offsets into a table of row tiles (slot, first row, height), on device
//   1. gemm1     h[r, f] = silu(xp[r] . W1[f]) * (xp[r] . W3[f])        (K = H)
//   2. gemm2     y[r, n] = h[r] . W2[n]                                  (K = F)
//
// Both GEMMs are "NT": activations [rows, K] and weights [out, K] are K-contiguous, which is
// the 8-consecutive-k-per-lane operand layout of v_mfma_f32_32x32x16_bf16, so an MFMA operand
// is one 16-byte LDS read.
//
// One workgroup = 8 waves (2 x 4) computes a 256 x 256 output tile (320, 192, 128 or 64 rows x 256
// where a slot's row count is not a multiple of 256) in steps of 64 k:
//   * global -> LDS goes through buffer_load ... lds (no register staging).  The per-lane
//     offset is fixed for the whole K loop; the k position travels in a scalar offset.
//   * two LDS stages of up to 72 KB (three smaller ones for the 128- and 64-row tiles).  Rows are
//     128 bytes; 16-byte chunk c of row r is stored at chunk position c ^ ((r >> 1) & 7), which makes sixteen consecutive rows reading the same
//     logical chunk cover all 64 banks exactly once.
//   * per k-step a wave runs four groups of MFMAs; the fragments of group g+1 are read from LDS
//     while group g executes.  The workgroup barrier sits before the last group, whose MFMAs
//     are interleaved one-to-one with the DMA instructions that prefetch tile k+2 into the
//     stage that was just vacated, and overlap the first fragment reads of tile k+1.
//
// In gemm1 a workgroup's 256 weight rows are 128 gate rows plus the 128 matching up rows,
// arranged so that each lane holds gate and up of the same output element; SwiGLU is applied
// on the accumulators.  Ragged row counts: a tile row past the slot's last row lies past the end
// of the activation tile's buffer descriptor, so its loads return zeros, and its stores are
// dropped the same way; the row space is never padded.
#include <mutex>

#include "common.hpp"
#include "mfma_pipeline.hpp"

namespace probe {

constexpr int FBN = 256;
// LDS: tiles of 192 rows and more run two stages (72 KB each for the 320-row tile); the short
// tiles (128 / 64 rows) are bound by load latency rather than by the matrix cores and run three
// stages of 48 / 40 KB, which gives every DMA batch two k-steps to land.
constexpr int kFfnLdsBytes = 3 * (128 + 256) * 128;  // 144 KB
static_assert(kFfnLdsBytes >= 2 * (320 + 256) * 128, "two stages of the tallest tile");


// ---- 0. schedule ----------------------------------------------------------------------
// The table is one 32-byte header (first word = number of tiles) followed by one 32-byte TileEntry
// per row tile, which holds everything a workgroup needs to start loading: first row, number
// of valid rows from there to the end of the slot, tile height (320, 256, 192, 128 or 64) and
// the slot's two weight pointers.
//
// How a slot is cut.  Every tile streams 256 weight rows per k-step whatever its height, so a
// short tile costs far more than its share of rows (64 rows take almost half the time of 256).
// A slot of M rows, u = ceil(M / 64), becomes a tiles of 320 and b tiles of 256 with 5a + 4b = u
// and a as large as possible: b = 4u mod 5, which exists whenever 4b <= u (every u >= 12).  The
// six values of u without such a cut end in one short tile, chosen by measured tile cost:
//   u = 1, 2, 3: one tile of 64u rows;  6: 256 + 128;  7: 320 + 128;  11: 320 + 256 + 128.
// Inside a slot the 320s come first, then the 256s, then the short tile.
//
// Order of the table.  Slots are taken by descending row count (ties: lower slot first) and a
// slot's tiles stay together: the workgroups that run side by side then share a slot's weight
// slices in L2, the long slots start early and the single short tiles fill the tail of the launch.
struct alignas(16) TileEntry {
  int32_t row0, rows, height, slot;
  const void* w13;
  const void* w2;
};
static_assert(sizeof(TileEntry) == 32, "one 32-byte record per tile");
// Table header, 128 bytes: word 0 = number of tiles; words 8..15 and 16..23 = the work-queue tickets of
// gemm1 and gemm2 (one counter per XCD), cleared by the schedule kernel of the same call.
constexpr int kTableHeaderInts = 32, kQueue1 = 8, kQueue2 = 16;

constexpr bool kInterleave = true;

struct SlotCut {
  int n320, n256, tail;  // tail = height of the one short tile (64, 128 or 192), 0 if there is none
  __device__ __forceinline__ int tiles() const { return n320 + n256 + (tail ? 1 : 0); }
};

__device__ __forceinline__ SlotCut cut_slot(int m) {
  SlotCut c = {0, 0, 0};
  const int u = (m + 63) >> 6;
  if (u == 0) return c;
  if (u <= 3) {
    c.tail = 64 * u;
    return c;
  }
  const int b = (4 * u) % 5;
  if (4 * b <= u) {
    c.n256 = b;
    c.n320 = (u - 4 * b) / 5;
  } else {  // u == 6, 7 or 11
    c.n320 = u == 6 ? 0 : 1;
    c.n256 = u == 7 ? 0 : 1;
    c.tail = 128;
  }
  return c;
}

__global__ __launch_bounds__(256) void ffn_schedule_kernel(const int32_t* __restrict__ slot_offsets,
                                                           const void* const* __restrict__ w13_ptrs,
                                                           const void* const* __restrict__ w2_ptrs,
                                                           int S, int max_tiles,
                                                           int32_t* __restrict__ table) {
  __shared__ int32_t rows_of[PROBE_MAX_SLOTS];
  __shared__ int32_t first_of[PROBE_MAX_SLOTS];
  __shared__ const void* w13_of[PROBE_MAX_SLOTS];
  __shared__ const void* w2_of[PROBE_MAX_SLOTS];
  __shared__ int32_t slot_at[PROBE_MAX_SLOTS];       // slot at each position of the sorted order
  __shared__ int32_t start[PROBE_MAX_SLOTS + 1];     // first tile of each position (exclusive prefix)
  __shared__ int32_t wave_tot[4];
  const int tid = threadIdx.x, lane = tid & 63;
  int m[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int s = tid * 4 + i;
    m[i] = 0;
    if (s < S) {
      const int first = slot_offsets[s];
      m[i] = max(slot_offsets[s + 1] - first, 0);
      rows_of[s] = m[i];
      first_of[s] = first;
      w13_of[s] = w13_ptrs[s];
      w2_of[s] = w2_ptrs[s];
    }
  }
  __syncthreads();
  // position of a slot = number of slots that come before it
  int pos[4] = {0, 0, 0, 0};
  for (int u = 0; u < S; ++u) {
    const int ru = rows_of[u];
#pragma unroll
    for (int i = 0; i < 4; ++i) pos[i] += (ru > m[i] || (ru == m[i] && u < tid * 4 + i)) ? 1 : 0;
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (tid * 4 + i < S) slot_at[pos[i]] = tid * 4 + i;
  __syncthreads();
  // exclusive prefix of tiles over positions tid*4 .. tid*4+3
  int v[4], local = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int p = tid * 4 + i;
    v[i] = p < S ? cut_slot(rows_of[slot_at[p]]).tiles() : 0;
    local += v[i];
  }
  int incl = local;
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    int o = __shfl_up(incl, d, kWave);
    if (lane >= d) incl += o;
  }
  if (lane == kWave - 1) wave_tot[tid >> 6] = incl;
  __syncthreads();
  int excl = incl - local;
  for (int i = 0; i < (tid >> 6); ++i) excl += wave_tot[i];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int p = tid * 4 + i;
    if (p < S) start[p] = excl;
    excl += v[i];
  }
  if (tid == 255) start[S] = excl;  // the last thread's running sum is the total
  __syncthreads();
  const int total = min(start[S], max_tiles);
  if (tid == 0) table[0] = total;
  if (tid >= kQueue1 && tid < kTableHeaderInts) table[tid] = 0;
  TileEntry* entries = reinterpret_cast<TileEntry*>(table + kTableHeaderInts);
  // positions [0, big) hold the slots of more than 192 rows: tiles [0, nb) are theirs, the ns single
  // short tiles follow
  int big = 0;
  for (int hi = S; big < hi;) {
    const int mid = (big + hi) >> 1;
    if (rows_of[slot_at[mid]] > 192) big = mid + 1; else hi = mid;
  }
  const int nb = min(start[big], total), ns = total - nb;
  for (int p = tid; p < total; p += 256) {
    // entry p of the table: the short tiles are spread evenly over the table
    const int before = static_cast<int>(static_cast<long>(p) * ns / total);
    const bool is_short = static_cast<int>(static_cast<long>(p + 1) * ns / total) > before;
    const int t = kInterleave ? (is_short ? nb + before : p - before) : p;
    int lo = 0, hi = S;  // last position with start[position] <= t
    while (hi - lo > 1) {
      int mid = (lo + hi) >> 1;
      if (start[mid] <= t) lo = mid; else hi = mid;
    }
    const int slot = slot_at[lo], first = first_of[slot];
    const SlotCut c = cut_slot(rows_of[slot]);
    int i = t - start[lo], row0 = first, height;
    if (i < c.n320) {
      row0 += i * 320;
      height = 320;
    } else if ((i -= c.n320) < c.n256) {
      row0 += c.n320 * 320 + i * 256;
      height = 256;
    } else {
      row0 += c.n320 * 320 + c.n256 * 256;
      height = c.tail;
    }
    TileEntry e;
    e.row0 = row0;
    e.rows = first + rows_of[slot] - row0;
    e.height = height;
    e.slot = slot;
    e.w13 = w13_of[slot];
    e.w2 = w2_of[slot];
    entries[p] = e;
  }
}

template <int MI, int NI>
__device__ __forceinline__ void zero_acc(f32x16 (&acc)[MI][NI]) {
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
}


// ---- workgroup -> (row tile, column block) -----------------------------------------------
// Workgroups are dealt to the 8 XCDs round-robin by their linear id, and each XCD has its own
// L2.  The launch is one-dimensional; workgroup L is the (L / 8)-th of XCD L % 8.  Work items
// are numbered so that the 32 workgroups an XCD runs side by side form a compact 8 x 4 block
// (8 consecutive row tiles x 4 consecutive column blocks): per k-step they pull 12 distinct
// operand slices through that L2 instead of 18 for a 16 x 2 strip.
constexpr int kXcds = 8, kBlkM = 8, kBlkN = 4, kBlk = kBlkM * kBlkN;

__device__ __forceinline__ bool ffn_item_of(int q, int n_tiles, int n_cols, int& tile, int& col) {
  // item number q: blocks of 32 items; block blk = (tile group, column group), column groups fastest
  const int col_groups = (n_cols + kBlkN - 1) / kBlkN;
  const int blk = q / kBlk, w = q % kBlk;
  const int tg = blk / col_groups, cg = blk % col_groups;
  tile = tg * kBlkM + w / kBlkN;
  col = cg * kBlkN + w % kBlkN;
  return tile < n_tiles && col < n_cols;
}

__device__ __forceinline__ bool ffn_work_item(int n_tiles, int n_cols, int& tile, int& col) {
  const int L = blockIdx.x;
  const int xcd = L % kXcds, j = L / kXcds;
  const int q = ((j / kBlk) * kXcds + xcd) * kBlk + (j % kBlk);  // item number: blocks of 32 per XCD
  return ffn_item_of(q, n_tiles, n_cols, tile, col);
}

// Work queue of the persistent launch (one workgroup per CU).  Blocks of 32 items are dealt to the XCDs
// round-robin as above (block b belongs to XCD b % 8), but which workgroup runs which item is decided at
// run time: a workgroup draws tickets from the counter of the XCD it runs on (ticket t = item t % 32 of
// that XCD's (t / 32)-th block), so the 32 workgroups of an XCD still walk one block side by side; when
// its own XCD's blocks are used up it draws from the next XCD's counter, and so on round the ring, until
// all eight are exhausted.  Counters only grow and nobody waits for anybody, so every workgroup ends after
// at most 8 unsuccessful draws.  Returns false when no work is left.
struct WorkQueue {
  int32_t* counters;  // [8], cleared by the schedule kernel
  int victim, misses;
  __device__ __forceinline__ void init(int32_t* c) {
    counters = c;
    victim = __builtin_amdgcn_s_getreg((20 << 0) | (0 << 6) | (3 << 11)) & (kXcds - 1);  // XCC_ID
    misses = 0;
  }
  // What ticket t of counter `victim` stands for; false (and the bookkeeping of an unsuccessful draw) if nothing.
  __device__ __forceinline__ bool accept(int t, int n_tiles, int n_cols, int& tile, int& col) {
    const int col_groups = (n_cols + kBlkN - 1) / kBlkN, tile_groups = (n_tiles + kBlkM - 1) / kBlkM;
    const int b = (t / kBlk) * kXcds + victim;
    if (b >= tile_groups * col_groups) {  // this XCD's blocks are used up: go on to the next one's
      victim = (victim + 1) & (kXcds - 1);
      ++misses;
      return false;
    }
    misses = 0;
    return ffn_item_of(b * kBlk + t % kBlk, n_tiles, n_cols, tile, col);
  }
  // all threads of the workgroup call this together; *slot is one int of static LDS
  __device__ __forceinline__ bool next(int n_tiles, int n_cols, volatile int* slot, int& tile, int& col) {
    while (misses < kXcds) {
      __syncthreads();  // the previous item is finished by every wave (LDS stages, *slot)
      if (threadIdx.x == 0) *slot = atomicAdd(&counters[victim], 1);
      __syncthreads();
      if (accept(__builtin_amdgcn_readfirstlane(*slot), n_tiles, n_cols, tile, col)) return true;
    }
    return false;
  }
  // The same when thread 0 has already drawn a ticket during the last k-steps of the previous item (gemm_mainloop,
  // DRAW) and every wave is past that loop's last barrier: no barrier is needed to read it, and none before the next
  // item's loads either, because no wave reads the LDS stages after that barrier.  Falls back to next() when the
  // ticket names no item (the end of a queue).
  __device__ __forceinline__ bool next_drawn(bool drew, int n_tiles, int n_cols, volatile int* slot, int& tile,
                                             int& col) {
    if (drew && accept(__builtin_amdgcn_readfirstlane(*slot), n_tiles, n_cols, tile, col)) return true;
    return next(n_tiles, n_cols, slot, tile, col);
  }
};

static int ffn_grid(int max_tiles, int n_cols) {
  const int tile_groups = (max_tiles + kBlkM - 1) / kBlkM, col_groups = (n_cols + kBlkN - 1) / kBlkN;
  const int blocks = tile_groups * col_groups;                       // blocks of 32 work items
  return (blocks + kXcds - 1) / kXcds * kXcds * kBlk;                // whole rounds over the 8 XCDs
}

// ---- 1. gemm1 + SwiGLU ----------------------------------------------------------------
// Where the activation rows of gemm1 come from: the permuted copy xp (row r of the row space), or,
// gathered on load, the token rows themselves: row r is x[row_pair[r] / k] (no xp is ever written).
struct RowSource {
  const bf16_t* base;         // xp, or x when gathering
  const int32_t* row_pair;    // nullptr = rows are stored in row-space order
  int k, n_tokens;
};

// NI = 32-row weight fragments per wave: 2 = a column block of 128 h columns (128 gate + 128 up weight
// rows per workgroup), 1 = 64 h columns (the skinny tiles of the decode schedule).  NST = LDS stages.
template <int MI, bool GATHER, int NI = 2, int NST = (MI >= 3 ? 2 : 3), bool DRAW = false>
__device__ __forceinline__ bool gemm1_tile(const RowSource& src, const bf16_t* __restrict__ w13,
                                           int row0, int rows, int n0, int H, int F,
                                           bf16_t* __restrict__ hbuf, u32x4* smem, int32_t* draw_counter = nullptr,
                                           volatile int* draw_slot = nullptr) {
  // rows = valid rows from row0 to the end of the slot (may exceed the tile height)
  constexpr int HALF = 16 * NI;  // h columns per wave; its 32*NI weight rows are HALF gate rows, then the HALF up rows
  const int lane = threadIdx.x & 63;
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wv / 4, wn = wv % 4;
  __amdgpu_buffer_rsrc_t rA =
      GATHER ? make_rsrc(src.base, static_cast<size_t>(src.n_tokens) * H * 2)
             : make_rsrc(src.base + static_cast<size_t>(row0) * H, static_cast<size_t>(rows) * H * 2);
  __amdgpu_buffer_rsrc_t rB = make_rsrc(w13, static_cast<size_t>(2) * F * H * 2);
  int voff[MI + 2 * NI];
  dma_offsets<MI>(wv, lane, H * 2,
                  [&](int r) {
                    // a tile row past the slot's last row gets an offset past the end of the descriptor: the
                    // load returns zeros, which also cost the matrix cores less than a copy of a real row
                    if (!GATHER) return r;
                    if (r >= rows) return src.n_tokens;
                    const int pair = src.row_pair[row0 + r];  // a valid row always names a pair
                    return min(max(pair, 0) / src.k, src.n_tokens - 1);
                  },
                  voff);
  // weight tile row j: wave column block q = j / (2 HALF); inside it HALF gate rows, then the HALF up rows
  dma_offsets<2 * NI>(wv, lane, H * 2,
                      [&](int j) {
                        int q = j / (2 * HALF), r = j % (2 * HALF);
                        int f = min(n0 + HALF * q + (r % HALF), F - 1);  // columns past F are masked at the store
                        return (r < HALF) ? f : F + f;
                      },
                      voff + MI);
  f32x16 acc[MI][NI];
  zero_acc<MI, NI>(acc);
  const bool drew =
      gemm_mainloop<MI, NI, 1, NST, true, DRAW>(rA, rB, voff, 0, H, smem, wv, lane, acc, draw_counter, draw_slot);

  // Accumulator registers 8g .. 8g+7 of a lane are eight consecutive output columns of one output
  // row (see gemm_mainloop, PERM): one 16-byte store each.  The stores go through a buffer
  // descriptor that ends with the tile's last valid row, so rows past it are dropped by the
  // bounds check instead of a branch.
  const int valid = min(rows, 64 * MI);
  __amdgpu_buffer_rsrc_t rH = make_rsrc(hbuf + static_cast<size_t>(row0) * F, static_cast<size_t>(valid) * F * 2);
  const int row_in = 32 * MI * wm + (lane & 31);
  const int cbase = n0 + HALF * wn + 8 * (lane >> 5);
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
    const int off = ((row_in + 32 * mi) * F + cbase) * 2;
#pragma unroll
    for (int g = 0; g < NI; ++g) {
      if (cbase + 16 * g < F) {  // F % 8 == 0: an 8-column group is in or out as a whole
        float hv[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          // NI = 2: fragment 0 holds the gate rows, fragment 1 the up rows; NI = 1: registers 0..7 / 8..15
          float gt = NI == 2 ? acc[mi][0][8 * g + e] : acc[mi][0][e];
          float up = NI == 2 ? acc[mi][NI - 1][8 * g + e] : acc[mi][0][8 + e];
          hv[e] = gt / (1.f + __expf(-gt)) * up;
        }
        u32x4 pk;
        pk[0] = pack_bf16x2(hv[0], hv[1]);
        pk[1] = pack_bf16x2(hv[2], hv[3]);
        pk[2] = pack_bf16x2(hv[4], hv[5]);
        pk[3] = pack_bf16x2(hv[6], hv[7]);
        __builtin_amdgcn_raw_buffer_store_b128(pk, rH, off + 32 * g, 0, 0);
      }
    }
  }
  return drew;
}

// one-dimensional launch over (row tile, column block) work items; a column block is 128 gate +
// 128 up weight rows
// queue != 0: persistent launch, items drawn from the work queue; 0: one workgroup per item
template <bool GATHER>
__global__ __launch_bounds__(512, 2) void ffn_gemm1_kernel(RowSource src, const int32_t* __restrict__ table,
                                                           int32_t* table_rw, int queue, int H, int F,
                                                           bf16_t* __restrict__ hbuf) {
#if defined(__HIP_DEVICE_COMPILE__)
  extern __shared__ u32x4 smem[];
  __shared__ int ticket;
  const int n_tiles = table[0], n_cols = (F + 127) / 128;
  int tile, col;
  if (queue) {
    // persistent launch: the ticket of the next item is drawn while the last k-steps of this one run
    WorkQueue wq;
    wq.init(table_rw + kQueue1);
    bool more = wq.next(n_tiles, n_cols, &ticket, tile, col);
    while (more) {
      const TileEntry e = reinterpret_cast<const TileEntry*>(table + kTableHeaderInts)[tile];
      const int n0 = col * 128;
      const bf16_t* w13 = static_cast<const bf16_t*>(e.w13);
      int32_t* ctr = wq.counters + wq.victim;
      bool drew;
      if (e.height > 256)
        drew = gemm1_tile<5, GATHER, 2, 2, true>(src, w13, e.row0, e.rows, n0, H, F, hbuf, smem, ctr, &ticket);
      else if (e.height > 192)
        drew = gemm1_tile<4, GATHER, 2, 2, true>(src, w13, e.row0, e.rows, n0, H, F, hbuf, smem, ctr, &ticket);
      else if (e.height > 128)
        drew = gemm1_tile<3, GATHER, 2, 2, true>(src, w13, e.row0, e.rows, n0, H, F, hbuf, smem, ctr, &ticket);
      else if (e.height > 64)
        drew = gemm1_tile<2, GATHER, 2, 3, true>(src, w13, e.row0, e.rows, n0, H, F, hbuf, smem, ctr, &ticket);
      else
        drew = gemm1_tile<1, GATHER, 2, 3, true>(src, w13, e.row0, e.rows, n0, H, F, hbuf, smem, ctr, &ticket);
      more = wq.next_drawn(drew, n_tiles, n_cols, &ticket, tile, col);
    }
    return;
  }
  if (!ffn_work_item(n_tiles, n_cols, tile, col)) return;
  const TileEntry e = reinterpret_cast<const TileEntry*>(table + kTableHeaderInts)[tile];
  const int n0 = col * 128;
  const bf16_t* w13 = static_cast<const bf16_t*>(e.w13);
  if (e.height > 256)
    gemm1_tile<5, GATHER>(src, w13, e.row0, e.rows, n0, H, F, hbuf, smem);
  else if (e.height > 192)
    gemm1_tile<4, GATHER>(src, w13, e.row0, e.rows, n0, H, F, hbuf, smem);
  else if (e.height > 128)
    gemm1_tile<3, GATHER>(src, w13, e.row0, e.rows, n0, H, F, hbuf, smem);
  else if (e.height > 64)
    gemm1_tile<2, GATHER>(src, w13, e.row0, e.rows, n0, H, F, hbuf, smem);
  else
    gemm1_tile<1, GATHER>(src, w13, e.row0, e.rows, n0, H, F, hbuf, smem);
#endif
}

// ---- 2. gemm2 -------------------------------------------------------------------------
template <int MI, int NI = 2, int NST = (MI >= 3 ? 2 : 3), bool DRAW = false>
__device__ __forceinline__ bool gemm2_tile(const bf16_t* __restrict__ hbuf, const bf16_t* __restrict__ w2,
                                           int row0, int rows, int n0, int H, int F,
                                           bf16_t* __restrict__ y, u32x4* smem, int32_t* draw_counter = nullptr,
                                           volatile int* draw_slot = nullptr) {
  const int lane = threadIdx.x & 63;
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wv / 4, wn = wv % 4;
  __amdgpu_buffer_rsrc_t rA = make_rsrc(hbuf + static_cast<size_t>(row0) * F, static_cast<size_t>(rows) * F * 2);
  __amdgpu_buffer_rsrc_t rB = make_rsrc(w2, static_cast<size_t>(H) * F * 2);
  int voff[MI + 2 * NI];
  dma_offsets<MI>(wv, lane, F * 2, [&](int r) { return r; }, voff);  // rows past the slot read as zeros (out of range)
  dma_offsets<2 * NI>(wv, lane, F * 2, [&](int j) { return min(n0 + j, H - 1); }, voff + MI);
  f32x16 acc[MI][NI];
  zero_acc<MI, NI>(acc);
  const bool drew =
      gemm_mainloop<MI, NI, 1, NST, true, DRAW>(rA, rB, voff, 0, F, smem, wv, lane, acc, draw_counter, draw_slot);

  const int valid = min(rows, 64 * MI);  // rows past it are dropped by the descriptor's bounds check
  __amdgpu_buffer_rsrc_t rY = make_rsrc(y + static_cast<size_t>(row0) * H, static_cast<size_t>(valid) * H * 2);
  const int row_in = 32 * MI * wm + (lane & 31);
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
      const int cbase = n0 + 32 * NI * wn + 32 * ni + 8 * (lane >> 5);
      const int off = ((row_in + 32 * mi) * H + cbase) * 2;
#pragma unroll
      for (int g = 0; g < 2; ++g) {
        if (cbase + 16 * g < H) {
          u32x4 pk;
          pk[0] = pack_bf16x2(acc[mi][ni][8 * g + 0], acc[mi][ni][8 * g + 1]);
          pk[1] = pack_bf16x2(acc[mi][ni][8 * g + 2], acc[mi][ni][8 * g + 3]);
          pk[2] = pack_bf16x2(acc[mi][ni][8 * g + 4], acc[mi][ni][8 * g + 5]);
          pk[3] = pack_bf16x2(acc[mi][ni][8 * g + 6], acc[mi][ni][8 * g + 7]);
          __builtin_amdgcn_raw_buffer_store_b128(pk, rY, off + 32 * g, 0, 0);
        }
      }
    }
  }
  return drew;
}

// one-dimensional launch over (row tile, column block of 256 output columns) work items
__global__ __launch_bounds__(512, 2) void ffn_gemm2_kernel(const bf16_t* __restrict__ hbuf,
                                                           const int32_t* __restrict__ table, int32_t* table_rw,
                                                           int queue, int H, int F, bf16_t* __restrict__ y) {
#if defined(__HIP_DEVICE_COMPILE__)
  extern __shared__ u32x4 smem[];
  __shared__ int ticket;
  const int n_tiles = table[0], n_cols = (H + FBN - 1) / FBN;
  int tile, col;
  if (queue) {
    WorkQueue wq;
    wq.init(table_rw + kQueue2);
    bool more = wq.next(n_tiles, n_cols, &ticket, tile, col);
    while (more) {
      const TileEntry e = reinterpret_cast<const TileEntry*>(table + kTableHeaderInts)[tile];
      const int n0 = col * FBN;
      const bf16_t* w2 = static_cast<const bf16_t*>(e.w2);
      int32_t* ctr = wq.counters + wq.victim;
      bool drew;
      if (e.height > 256)
        drew = gemm2_tile<5, 2, 2, true>(hbuf, w2, e.row0, e.rows, n0, H, F, y, smem, ctr, &ticket);
      else if (e.height > 192)
        drew = gemm2_tile<4, 2, 2, true>(hbuf, w2, e.row0, e.rows, n0, H, F, y, smem, ctr, &ticket);
      else if (e.height > 128)
        drew = gemm2_tile<3, 2, 2, true>(hbuf, w2, e.row0, e.rows, n0, H, F, y, smem, ctr, &ticket);
      else if (e.height > 64)
        drew = gemm2_tile<2, 2, 3, true>(hbuf, w2, e.row0, e.rows, n0, H, F, y, smem, ctr, &ticket);
      else
        drew = gemm2_tile<1, 2, 3, true>(hbuf, w2, e.row0, e.rows, n0, H, F, y, smem, ctr, &ticket);
      more = wq.next_drawn(drew, n_tiles, n_cols, &ticket, tile, col);
    }
    return;
  }
  if (!ffn_work_item(n_tiles, n_cols, tile, col)) return;
  const TileEntry e = reinterpret_cast<const TileEntry*>(table + kTableHeaderInts)[tile];
  const int n0 = col * FBN;
  const bf16_t* w2 = static_cast<const bf16_t*>(e.w2);
  if (e.height > 256)
    gemm2_tile<5>(hbuf, w2, e.row0, e.rows, n0, H, F, y, smem);
  else if (e.height > 192)
    gemm2_tile<4>(hbuf, w2, e.row0, e.rows, n0, H, F, y, smem);
  else if (e.height > 128)
    gemm2_tile<3>(hbuf, w2, e.row0, e.rows, n0, H, F, y, smem);
  else if (e.height > 64)
    gemm2_tile<2>(hbuf, w2, e.row0, e.rows, n0, H, F, y, smem);
  else
    gemm2_tile<1>(hbuf, w2, e.row0, e.rows, n0, H, F, y, smem);
#endif
}

// ---- decode schedule: skinny tiles -------------------------------------------------------------
// When every slot holds a few rows (a decode step: rows per slot of the order of ten), the grouped GEMM does
// almost no arithmetic per weight byte (the small-n end of eta_g(n), Sec. 3.2) and the call is a stream
// of every active slot's weights through the chip.  What matters then is that every CU pulls a distinct
// slice at all times, so the work is cut finer and kept resident: tiles of 64 rows x 64 h columns (gemm1:
// 64 gate + 64 up weight rows) or 64 rows x 128 output columns (gemm2), three LDS stages of 24 KB, two
// workgroups per CU (sixteen waves, 72 KB of LDS each), one work item per workgroup in table order.  A
// slot with more than 64 rows is simply several row tiles: correct for any input, tuned for short slots.
constexpr int kSkinnyLdsBytes = 3 * (64 + 128) * 128;  // 72 KB
constexpr int kSkinnyCols1 = 64, kSkinnyCols2 = 128;   // h columns / y columns per work item

// Tile number -> (slot, first row, rows to the end of the slot, weight pointer) without a tile table: slots
// in their own order, ceil(M / 64) tiles each.  Every workgroup finds its own tile with one scan over the
// (at most 1024) slots, two per thread, so the decode schedule needs no schedule kernel in front of it.
// Returns false if the tile number is past the last tile (the launch is sized for the capacity).
struct SkinnyTile {
  int row0, rows;
  const void* w;
};

__device__ __forceinline__ bool skinny_locate(const int32_t* __restrict__ slot_offsets,
                                              const void* const* __restrict__ w_ptrs, int S, int tile,
                                              SkinnyTile& out) {
  __shared__ int32_t wave_tot[8];
  __shared__ int32_t found_row0, found_rows;
  __shared__ const void* found_w;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  if (tid == 0) found_rows = 0;
  int first[2], m[2], t[2];
  const void* w[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int sl = 2 * tid + i;
    first[i] = m[i] = 0;
    w[i] = nullptr;
    if (sl < S) {
      first[i] = slot_offsets[sl];
      m[i] = max(slot_offsets[sl + 1] - first[i], 0);
      w[i] = w_ptrs[sl];
    }
    t[i] = (m[i] + 63) >> 6;
  }
  const int local = t[0] + t[1];
  int incl = local;
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    int o = __shfl_up(incl, d, kWave);
    if (lane >= d) incl += o;
  }
  if (lane == kWave - 1) wave_tot[wv] = incl;
  __syncthreads();
  int excl = incl - local;
  for (int i = 0; i < wv; ++i) excl += wave_tot[i];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    if (tile >= excl && tile < excl + t[i]) {  // true for exactly one (thread, i) when the tile exists
      const int r = (tile - excl) * 64;
      found_row0 = first[i] + r;
      found_rows = m[i] - r;
      found_w = w[i];
    }
    excl += t[i];
  }
  __syncthreads();
  out.row0 = found_row0;
  out.rows = found_rows;
  out.w = found_w;
  return found_rows > 0;
}

template <bool GATHER>
__global__ __launch_bounds__(512, 4) void ffn_gemm1_skinny_kernel(RowSource src,
                                                                  const int32_t* __restrict__ slot_offsets,
                                                                  const void* const* __restrict__ w13_ptrs, int S,
                                                                  int H, int F, bf16_t* __restrict__ hbuf) {
#if defined(__HIP_DEVICE_COMPILE__)
  extern __shared__ u32x4 smem[];
  const int n_cols = (F + kSkinnyCols1 - 1) / kSkinnyCols1;
  const int tile = blockIdx.x / n_cols, col = blockIdx.x % n_cols;
  SkinnyTile e;
  if (!skinny_locate(slot_offsets, w13_ptrs, S, tile, e)) return;
  gemm1_tile<1, GATHER, 1, 3>(src, static_cast<const bf16_t*>(e.w), e.row0, e.rows, col * kSkinnyCols1, H, F, hbuf,
                              smem);
#endif
}

__global__ __launch_bounds__(512, 4) void ffn_gemm2_skinny_kernel(const bf16_t* __restrict__ hbuf,
                                                                  const int32_t* __restrict__ slot_offsets,
                                                                  const void* const* __restrict__ w2_ptrs, int S,
                                                                  int H, int F, bf16_t* __restrict__ y) {
#if defined(__HIP_DEVICE_COMPILE__)
  extern __shared__ u32x4 smem[];
  const int n_cols = (H + kSkinnyCols2 - 1) / kSkinnyCols2;
  const int tile = blockIdx.x / n_cols, col = blockIdx.x % n_cols;
  SkinnyTile e;
  if (!skinny_locate(slot_offsets, w2_ptrs, S, tile, e)) return;
  gemm2_tile<1, 1, 3>(hbuf, static_cast<const bf16_t*>(e.w), e.row0, e.rows, col * kSkinnyCols2, H, F, y, smem);
#endif
}

struct FfnShape {
  bool skinny;  // the decode schedule
  int max_tiles;
  size_t h_bytes, table_bytes;
};

// The decode schedule is chosen on the host from the capacity of the row space alone (the row counts live
// on the device): at most kSkinnyRowsPerSlot rows per slot on average even if every pair were local.
constexpr int kSkinnyRowsPerSlot = 64;

static FfnShape ffn_shape(int S, int F, int max_rows) {
  FfnShape s;
  s.skinny = static_cast<long>(max_rows) <= static_cast<long>(kSkinnyRowsPerSlot) * S;
  s.max_tiles = s.skinny ? max_rows / 64 + S : max_rows / 256 + S;
  s.h_bytes = align_up(static_cast<size_t>(max_rows > 0 ? max_rows : 1) * F * sizeof(bf16_t), 256);
  s.table_bytes = align_up(kTableHeaderInts * sizeof(int32_t) + static_cast<size_t>(s.max_tiles) * sizeof(TileEntry), 256);
  return s;
}

// The GEMM kernels use 144 KB of dynamic LDS, which has to be opted into once per device.  *cus receives
// the device's CU count (the size of the persistent launch).
static int ffn_prepare(int* cus) {
  static std::mutex mu;
  static bool done[64] = {false};
  static int cu_count[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
    set_error("probe_grouped_ffn: no current device");
    return PROBE_EHIP;
  }
  std::lock_guard<std::mutex> lock(mu);
  if (done[dev]) {
    *cus = cu_count[dev];
    return PROBE_OK;
  }
  if (hipDeviceGetAttribute(&cu_count[dev], hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
      cu_count[dev] <= 0) {
    set_error("probe_grouped_ffn: cannot read the CU count of device %d", dev);
    return PROBE_EHIP;
  }
  *cus = cu_count[dev];
  hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(ffn_gemm1_kernel<false>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kFfnLdsBytes);
  if (err == hipSuccess)
    err = hipFuncSetAttribute(reinterpret_cast<const void*>(ffn_gemm1_kernel<true>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, kFfnLdsBytes);
  if (err == hipSuccess)
    err = hipFuncSetAttribute(reinterpret_cast<const void*>(ffn_gemm2_kernel),
                              hipFuncAttributeMaxDynamicSharedMemorySize, kFfnLdsBytes);
  if (err == hipSuccess)
    err = hipFuncSetAttribute(reinterpret_cast<const void*>(ffn_gemm1_skinny_kernel<false>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, kSkinnyLdsBytes);
  if (err == hipSuccess)
    err = hipFuncSetAttribute(reinterpret_cast<const void*>(ffn_gemm1_skinny_kernel<true>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, kSkinnyLdsBytes);
  if (err == hipSuccess)
    err = hipFuncSetAttribute(reinterpret_cast<const void*>(ffn_gemm2_skinny_kernel),
                              hipFuncAttributeMaxDynamicSharedMemorySize, kSkinnyLdsBytes);
  if (err != hipSuccess) {
    set_error("probe_grouped_ffn: cannot reserve %d bytes of LDS: %s", kFfnLdsBytes, hipGetErrorString(err));
    return PROBE_EHIP;
  }
  done[dev] = true;
  return PROBE_OK;
}

}  // namespace probe

extern "C" size_t probe_grouped_ffn_workspace_bytes(int S, int H, int F, int max_rows) {
  (void)H;
  if (S <= 0 || F <= 0 || max_rows < 0) return 0;
  probe::FfnShape s = probe::ffn_shape(S, F, max_rows);
  return s.h_bytes + s.table_bytes;
}

namespace probe {

// Shared body of probe_grouped_ffn (row_pair == nullptr: activations from xp) and
// probe_grouped_ffn_gather (activations gathered from the token rows through row_pair).
static int ffn_impl(const char* name, const void* act_bf16, const int32_t* row_pair, int k, int T,
                    const int32_t* slot_offsets, const void* const* w13_ptrs, const void* const* w2_ptrs, int S,
                    int H, int F, int max_rows, void* y_bf16, void* workspace, size_t workspace_bytes,
                    void* stream) {
  PROBE_REQUIRE(S >= 1 && H > 0 && F > 0 && max_rows >= 0, PROBE_EINVAL,
                "%s: bad dims S=%d H=%d F=%d max_rows=%d", name, S, H, F, max_rows);
  PROBE_REQUIRE(S <= PROBE_MAX_SLOTS && H % 64 == 0 && F % 64 == 0, PROBE_EUNSUPPORTED,
                "%s: needs S <= %d, H %% 64 == 0, F %% 64 == 0 (S=%d H=%d F=%d)", name, PROBE_MAX_SLOTS, S, H, F);
  PROBE_REQUIRE(static_cast<size_t>(2) * F * H * 2 <= 0x7fffffffull, PROBE_EUNSUPPORTED,
                "%s: one expert's w13 must stay below 2 GiB (H=%d F=%d)", name, H, F);
  PROBE_REQUIRE(H <= (1 << 21) && F <= (1 << 21), PROBE_EUNSUPPORTED,
                "%s: H and F must not exceed 2^21 (32-bit byte offsets inside a row tile)", name);
  const bool gather = row_pair != nullptr;
  if (gather) {
    PROBE_REQUIRE(k >= 1 && k <= PROBE_MAX_TOPK && T >= 0, PROBE_EINVAL, "%s: bad k=%d or T=%d", name, k, T);
    PROBE_REQUIRE(static_cast<size_t>(T) * H * 2 <= 0x7fffffffull, PROBE_EUNSUPPORTED,
                  "%s: x must stay below 2 GiB (T=%d H=%d)", name, T, H);
  }
  if (max_rows == 0 || (gather && T == 0)) return PROBE_OK;
  PROBE_REQUIRE(act_bf16 && slot_offsets && w13_ptrs && w2_ptrs && y_bf16, PROBE_EINVAL, "%s: null pointer", name);
  PROBE_REQUIRE(aligned16(act_bf16) && aligned16(y_bf16), PROBE_EALIGN,
                "%s: activations and y must be 16-byte aligned", name);
  FfnShape sh = ffn_shape(S, F, max_rows);
  PROBE_REQUIRE(workspace && aligned16(workspace) && workspace_bytes >= sh.h_bytes + sh.table_bytes,
                PROBE_EWORKSPACE, "%s: workspace too small or misaligned (%zu < %zu)", name, workspace_bytes,
                sh.h_bytes + sh.table_bytes);
  PROBE_REQUIRE(static_cast<long>(sh.max_tiles + 8) * ((F + 127) / 128 + 4) < (1l << 30) &&
                    static_cast<long>(sh.max_tiles + 8) * ((H + 255) / 256 + 4) < (1l << 30),
                PROBE_EUNSUPPORTED, "%s: max_rows too large (%d)", name, max_rows);
  int cus = 0;
  int rc = ffn_prepare(&cus);
  if (rc != PROBE_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  bf16_t* hbuf = static_cast<bf16_t*>(workspace);
  int32_t* table = reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + sh.h_bytes);
  RowSource src;
  src.base = static_cast<const bf16_t*>(act_bf16);
  src.row_pair = row_pair;
  src.k = gather ? k : 1;
  src.n_tokens = gather ? T : 0;
  if (sh.skinny) {
    const dim3 g1(sh.max_tiles * ((F + kSkinnyCols1 - 1) / kSkinnyCols1));
    const dim3 g2(sh.max_tiles * ((H + kSkinnyCols2 - 1) / kSkinnyCols2));
    if (gather)
      hipLaunchKernelGGL(ffn_gemm1_skinny_kernel<true>, g1, dim3(512), kSkinnyLdsBytes, st, src, slot_offsets,
                         w13_ptrs, S, H, F, hbuf);
    else
      hipLaunchKernelGGL(ffn_gemm1_skinny_kernel<false>, g1, dim3(512), kSkinnyLdsBytes, st, src, slot_offsets,
                         w13_ptrs, S, H, F, hbuf);
    hipLaunchKernelGGL(ffn_gemm2_skinny_kernel, g2, dim3(512), kSkinnyLdsBytes, st, hbuf, slot_offsets, w2_ptrs, S, H,
                       F, static_cast<bf16_t*>(y_bf16));
    return check_launch(name);
  }
  hipLaunchKernelGGL(ffn_schedule_kernel, dim3(1), dim3(256), 0, st, slot_offsets, w13_ptrs, w2_ptrs, S, sh.max_tiles,
                     table);
  // persistent launch (one workgroup per CU, items drawn from the work queue) unless the capacity of the
  // row space gives fewer items than that
  const int cap1 = ffn_grid(sh.max_tiles, (F + 127) / 128), cap2 = ffn_grid(sh.max_tiles, (H + FBN - 1) / FBN);
  const int q1 = cap1 > cus ? 1 : 0, q2 = cap2 > cus ? 1 : 0;
  const dim3 grid1(q1 ? cus : cap1), grid2(q2 ? cus : cap2);
  if (gather)
    hipLaunchKernelGGL(ffn_gemm1_kernel<true>, grid1, dim3(512), kFfnLdsBytes, st, src, table, table, q1, H, F, hbuf);
  else
    hipLaunchKernelGGL(ffn_gemm1_kernel<false>, grid1, dim3(512), kFfnLdsBytes, st, src, table, table, q1, H, F, hbuf);
  hipLaunchKernelGGL(ffn_gemm2_kernel, grid2, dim3(512), kFfnLdsBytes, st, hbuf, table, table, q2, H, F,
                     static_cast<bf16_t*>(y_bf16));
  return check_launch(name);
}

}  // namespace probe

extern "C" int probe_grouped_ffn(const void* xp_bf16, const int32_t* slot_offsets,
                                 const void* const* w13_ptrs, const void* const* w2_ptrs, int S,
                                 int H, int F, int max_rows, void* y_bf16, void* workspace,
                                 size_t workspace_bytes, void* stream) {
  return probe::ffn_impl("probe_grouped_ffn", xp_bf16, nullptr, 1, 0, slot_offsets, w13_ptrs, w2_ptrs, S, H, F,
                         max_rows, y_bf16, workspace, workspace_bytes, stream);
}

extern "C" int probe_grouped_ffn_gather(const void* x_bf16, const int32_t* row_pair, int T, int k,
                                        const int32_t* slot_offsets, const void* const* w13_ptrs,
                                        const void* const* w2_ptrs, int S, int H, int F, int max_rows,
                                        void* y_bf16, void* workspace, size_t workspace_bytes, void* stream) {
  PROBE_REQUIRE(row_pair != nullptr || max_rows == 0 || T == 0, PROBE_EINVAL,
                "probe_grouped_ffn_gather: row_pair is NULL");
  return probe::ffn_impl("probe_grouped_ffn_gather", x_bf16, row_pair, k, T, slot_offsets, w13_ptrs, w2_ptrs, S, H,
                         F, max_rows, y_bf16, workspace, workspace_bytes, stream);
}
