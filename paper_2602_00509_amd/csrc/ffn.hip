// probe_grouped_ffn: grouped SwiGLU expert FFN on the bf16 matrix cores.
//
//   0. schedule  turn slot_offsets into a table of 128-row tiles (slot, first row), on device
//   1. gemm1     h[r, f] = silu(xp[r] . W1[f]) * (xp[r] . W3[f])        (K = H)
//   2. gemm2     y[r, n] = h[r] . W2[n]                                  (K = F)
//
// Both GEMMs are "NT": activations [rows, K] and weights [out, K] are K-contiguous, which is
// exactly the 8-consecutive-k-per-lane operand layout of v_mfma_f32_32x32x16_bf16, so LDS
// fragments are single 16-byte reads.  A workgroup (4 waves, 2x2) computes a 128x128 output
// tile in steps of 64 k: global -> registers (prefetch of the next step) -> swizzled LDS ->
// MFMA.  In gemm1 a workgroup's 128 weight rows are 64 gate rows plus the 64 matching up rows,
// arranged so that each lane holds gate and up of the same output element and SwiGLU is
// applied on the accumulators.  Ragged row counts are handled by clamping loads to the
// slot's last row and masking stores; no padding of the row space is required.
#include "common.hpp"

namespace probe {

constexpr int FBM = 128, FBN = 128, FBK = 64;

// ---- 0. schedule ----------------------------------------------------------------------
// table[0] = number of tiles; table[1 + 2*i] = slot, table[2 + 2*i] = first row of tile i.
__global__ __launch_bounds__(256) void ffn_schedule_kernel(const int32_t* __restrict__ slot_offsets,
                                                           int S, int max_tiles,
                                                           int32_t* __restrict__ table) {
  __shared__ int32_t tile_start[PROBE_MAX_SLOTS + 1];
  __shared__ int32_t wave_tot[4];
  const int tid = threadIdx.x, lane = tid & 63;
  int v[4], local = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int s = tid * 4 + i;
    int m = 0;
    if (s < S) m = max(slot_offsets[s + 1] - slot_offsets[s], 0);
    v[i] = (m + FBM - 1) / FBM;
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
    int s = tid * 4 + i;
    if (s < S) tile_start[s] = excl;
    excl += v[i];
  }
  if (tid == 255) tile_start[S] = excl;  // the last thread's running sum is the total
  __syncthreads();
  int total = min(tile_start[S], max_tiles);
  if (tid == 0) table[0] = total;
  for (int t = tid; t < total; t += 256) {
    int lo = 0, hi = S;  // last slot with tile_start[slot] <= t
    while (hi - lo > 1) {
      int mid = (lo + hi) >> 1;
      if (tile_start[mid] <= t) lo = mid; else hi = mid;
    }
    table[1 + 2 * t] = lo;
    table[2 + 2 * t] = slot_offsets[lo] + (t - tile_start[lo]) * FBM;
  }
}

// ---- shared main loop -----------------------------------------------------------------
// acc += A_tile[128, K] * B_tile[128, K]^T.  a_row(i) / b_row(j) give the K-contiguous global
// row behind tile row i / j (already clamped to valid memory).  Wave (wm, wn) accumulates the
// 64x64 block at tile rows 64*wm and tile columns 64*wn as 2x2 MFMA tiles.
template <typename AF, typename BF>
__device__ __forceinline__ void mainloop_128x128(AF a_row, BF b_row, int K, u32x4* sA, u32x4* sB,
                                                 f32x16 (&acc)[2][2]) {
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int wm = wv >> 1, wn = wv & 1;
  const bf16_t* pa[4];
  const bf16_t* pb[4];
  int soff[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    int idx = tid + 256 * j;
    int row = idx >> 3, c = idx & 7;
    pa[j] = a_row(row) + c * 8;
    pb[j] = b_row(row) + c * 8;
    soff[j] = lds_chunk_off(row, c);
  }
  u32x4 ra[4], rb[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    ra[j] = *reinterpret_cast<const u32x4*>(pa[j]);
    rb[j] = *reinterpret_cast<const u32x4*>(pb[j]);
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    sA[soff[j]] = ra[j];
    sB[soff[j]] = rb[j];
  }
  __syncthreads();
  for (int k0 = 0; k0 < K; k0 += FBK) {
    const bool more = k0 + FBK < K;
    if (more) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        ra[j] = *reinterpret_cast<const u32x4*>(pa[j] + k0 + FBK);
        rb[j] = *reinterpret_cast<const u32x4*>(pb[j] + k0 + FBK);
      }
    }
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const int c = 2 * kk + (lane >> 5);
      u32x4 a[2], b[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        a[i] = sA[lds_chunk_off(64 * wm + 32 * i + (lane & 31), c)];
        b[i] = sB[lds_chunk_off(64 * wn + 32 * i + (lane & 31), c)];
      }
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) acc[mi][ni] = mfma_32x32x16(a[mi], b[ni], acc[mi][ni]);
    }
    __syncthreads();
    if (more) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        sA[soff[j]] = ra[j];
        sB[soff[j]] = rb[j];
      }
      __syncthreads();
    }
  }
}

__device__ __forceinline__ void zero_acc(f32x16 (&acc)[2][2]) {
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
}

// ---- 1. gemm1 + SwiGLU ----------------------------------------------------------------
// grid.x = F/64 column blocks (64 gate + 64 up weight rows each), grid.y = tile capacity.
__global__ __launch_bounds__(256, 2) void ffn_gemm1_kernel(const bf16_t* __restrict__ xp,
                                                           const int32_t* __restrict__ table,
                                                           const int32_t* __restrict__ slot_offsets,
                                                           const void* const* __restrict__ w13_ptrs,
                                                           int H, int F, bf16_t* __restrict__ hbuf) {
  __shared__ u32x4 sA[FBM * 8];
  __shared__ u32x4 sB[FBN * 8];
  const int tile = blockIdx.y;
  if (tile >= table[0]) return;
  const int slot = table[1 + 2 * tile], row0 = table[2 + 2 * tile];
  const int row_end = slot_offsets[slot + 1];
  const int n0 = blockIdx.x * 64;
  const bf16_t* w13 = static_cast<const bf16_t*>(w13_ptrs[slot]);
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int wm = wv >> 1, wn = wv & 1;

  f32x16 acc[2][2];
  zero_acc(acc);
  auto a_row = [&](int i) { return xp + static_cast<long>(min(row0 + i, row_end - 1)) * H; };
  // tile column j: wave column block q = j/64; inside it 32 gate rows then the 32 up rows
  auto b_row = [&](int j) {
    int q = j >> 6, r = j & 63;
    int wrow = (r < 32) ? (n0 + 32 * q + r) : (F + n0 + 32 * q + (r - 32));
    return w13 + static_cast<long>(wrow) * H;
  };
  mainloop_128x128(a_row, b_row, H, sA, sB, acc);

  const int col = n0 + 32 * wn + mfma32_col(lane);
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      int row = row0 + 64 * wm + 32 * mi + mfma32_row(r, lane);
      if (row < row_end) {
        float g = acc[mi][0][r], u = acc[mi][1][r];
        float hval = g / (1.f + __expf(-g)) * u;
        hbuf[static_cast<long>(row) * F + col] = f32_to_bf16(hval);
      }
    }
}

// ---- 2. gemm2 -------------------------------------------------------------------------
// grid.x = ceil(H/128) column blocks, grid.y = tile capacity.
__global__ __launch_bounds__(256, 2) void ffn_gemm2_kernel(const bf16_t* __restrict__ hbuf,
                                                           const int32_t* __restrict__ table,
                                                           const int32_t* __restrict__ slot_offsets,
                                                           const void* const* __restrict__ w2_ptrs,
                                                           int H, int F, bf16_t* __restrict__ y) {
  __shared__ u32x4 sA[FBM * 8];
  __shared__ u32x4 sB[FBN * 8];
  const int tile = blockIdx.y;
  if (tile >= table[0]) return;
  const int slot = table[1 + 2 * tile], row0 = table[2 + 2 * tile];
  const int row_end = slot_offsets[slot + 1];
  const int n0 = blockIdx.x * FBN;
  const bf16_t* w2 = static_cast<const bf16_t*>(w2_ptrs[slot]);
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int wm = wv >> 1, wn = wv & 1;

  f32x16 acc[2][2];
  zero_acc(acc);
  auto a_row = [&](int i) { return hbuf + static_cast<long>(min(row0 + i, row_end - 1)) * F; };
  auto b_row = [&](int j) { return w2 + static_cast<long>(min(n0 + j, H - 1)) * F; };
  mainloop_128x128(a_row, b_row, F, sA, sB, acc);

#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
      int col = n0 + 64 * wn + 32 * ni + mfma32_col(lane);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        int row = row0 + 64 * wm + 32 * mi + mfma32_row(r, lane);
        if (row < row_end && col < H) y[static_cast<long>(row) * H + col] = f32_to_bf16(acc[mi][ni][r]);
      }
    }
}

struct FfnShape {
  int max_tiles;
  size_t h_bytes, table_bytes;
};

static FfnShape ffn_shape(int S, int F, int max_rows) {
  FfnShape s;
  s.max_tiles = max_rows / FBM + S;
  s.h_bytes = align_up(static_cast<size_t>(max_rows > 0 ? max_rows : 1) * F * sizeof(bf16_t), 256);
  s.table_bytes = align_up((1 + 2 * static_cast<size_t>(s.max_tiles)) * sizeof(int32_t), 256);
  return s;
}

}  // namespace probe

extern "C" size_t probe_grouped_ffn_workspace_bytes(int S, int H, int F, int max_rows) {
  (void)H;
  if (S <= 0 || F <= 0 || max_rows < 0) return 0;
  probe::FfnShape s = probe::ffn_shape(S, F, max_rows);
  return s.h_bytes + s.table_bytes;
}

extern "C" int probe_grouped_ffn(const void* xp_bf16, const int32_t* slot_offsets,
                                 const void* const* w13_ptrs, const void* const* w2_ptrs, int S,
                                 int H, int F, int max_rows, void* y_bf16, void* workspace,
                                 size_t workspace_bytes, void* stream) {
  using namespace probe;
  PROBE_REQUIRE(S >= 1 && H > 0 && F > 0 && max_rows >= 0, PROBE_EINVAL,
                "probe_grouped_ffn: bad dims S=%d H=%d F=%d max_rows=%d", S, H, F, max_rows);
  PROBE_REQUIRE(S <= PROBE_MAX_SLOTS && H % 64 == 0 && F % 64 == 0, PROBE_EUNSUPPORTED,
                "probe_grouped_ffn: needs S <= %d, H %% 64 == 0, F %% 64 == 0 (S=%d H=%d F=%d)",
                PROBE_MAX_SLOTS, S, H, F);
  if (max_rows == 0) return PROBE_OK;
  PROBE_REQUIRE(xp_bf16 && slot_offsets && w13_ptrs && w2_ptrs && y_bf16, PROBE_EINVAL,
                "probe_grouped_ffn: null pointer");
  PROBE_REQUIRE(aligned16(xp_bf16) && aligned16(y_bf16), PROBE_EALIGN,
                "probe_grouped_ffn: xp/y must be 16-byte aligned");
  FfnShape sh = ffn_shape(S, F, max_rows);
  PROBE_REQUIRE(workspace && aligned16(workspace) && workspace_bytes >= sh.h_bytes + sh.table_bytes,
                PROBE_EWORKSPACE, "probe_grouped_ffn: workspace too small or misaligned (%zu < %zu)",
                workspace_bytes, sh.h_bytes + sh.table_bytes);
  PROBE_REQUIRE(sh.max_tiles <= 65535, PROBE_EUNSUPPORTED, "probe_grouped_ffn: max_rows too large (%d)",
                max_rows);
  hipStream_t st = static_cast<hipStream_t>(stream);
  bf16_t* hbuf = static_cast<bf16_t*>(workspace);
  int32_t* table = reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + sh.h_bytes);
  hipLaunchKernelGGL(ffn_schedule_kernel, dim3(1), dim3(256), 0, st, slot_offsets, S, sh.max_tiles, table);
  hipLaunchKernelGGL(ffn_gemm1_kernel, dim3(F / 64, sh.max_tiles), dim3(256), 0, st,
                     static_cast<const bf16_t*>(xp_bf16), table, slot_offsets, w13_ptrs, H, F, hbuf);
  hipLaunchKernelGGL(ffn_gemm2_kernel, dim3((H + FBN - 1) / FBN, sh.max_tiles), dim3(256), 0, st, hbuf,
                     table, slot_offsets, w2_ptrs, H, F, static_cast<bf16_t*>(y_bf16));
  return check_launch("probe_grouped_ffn");
}
