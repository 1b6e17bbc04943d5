// Software-pipelined NT bf16 GEMM main loop on v_mfma_f32_32x32x16_bf16, shared by the grouped FFN
// and the gate.  See the comments of ffn.hip for the pipeline; this header only holds the loop.
#pragma once

#include <type_traits>

#include "common.hpp"

namespace probe {

constexpr int FBK = 64;  // k per step
#define PROBE_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

template <int N>
__device__ __forceinline__ void wait_vm_lgkm0() {  // s_waitcnt vmcnt(N) lgkmcnt(0), N < 64
  __builtin_amdgcn_s_waitcnt(0x0070 | (N & 15) | ((N >> 4) << 14));
}

// ---- shared main loop -----------------------------------------------------------------
// 8 waves as 2 (rows) x 4 (columns).  The A tile has 64*MI rows; the B tile has PL planes of
// 128*NI rows each (plane p, column c at B-tile row p*128*NI + c).  The calling wave accumulates
//   acc[i][j] += sum_p  A[32*MI*wm + 32*i .. +32, :] * B_p[32*NI*wn + 32*j .. +32, :]^T
// (PL = 1: a plain GEMM; PL = 3: one logical weight held as three bf16 planes).
// rA / rB are buffer descriptors of the tile's first A row / of the weight matrix; voff[j] is
// this lane's byte offset for DMA instruction j (MI instructions for A, then BW for B); k0 is
// the first k of this call's K range and K its length (a multiple of 64).
// NST = LDS stages (2 or 3); a DMA batch is issued NST k-steps ahead of its use.
//
// Accumulator layout.  The B fragment is the MFMA's row operand, so with PERM = false registers
// 4q .. 4q+3 of lane l hold output row (l % 32) of the A block and the four consecutive output
// columns 8q + 4(l / 32) .. +3 of the B block.  With PERM = true, MFMA row position i is fed B row
// i with bits 2 and 3 exchanged; registers 8g .. 8g+7 then hold the EIGHT consecutive columns
// 16g + 8(l / 32) .. +7, a 16-byte bf16 store per lane and 32 contiguous bytes per row and store
// instruction.  Sixteen consecutive positions still read sixteen consecutive LDS rows, so the
// fragment reads stay free of bank conflicts.
//
// DRAW: thread 0 of the workgroup draws the next ticket of a work queue (atomic add of 1 on *draw_counter) at the
// start of the second-to-last k-step, which issues no DMA and ends with a wait for everything in flight, and
// leaves it in *draw_slot (LDS) before that step's barrier; after the loop every thread can read it.  Returns
// whether that happened (it needs K >= 128).  After the barrier of the last k-step no wave reads the LDS stages.
template <int MI, int NI, int PL, int NST, bool PERM = false, bool DRAW = false>
__device__ __forceinline__ bool gemm_mainloop(__amdgpu_buffer_rsrc_t rA, __amdgpu_buffer_rsrc_t rB,
                                              const int (&voff)[MI + NI * PL * 2], int k0, int K,
                                              u32x4* smem, int wv, int lane, f32x16 (&acc)[MI][NI],
                                              int32_t* draw_counter = nullptr, volatile int* draw_slot = nullptr) {
  constexpr int WN = 4, BROWS = 128 * NI * PL, AW = MI, BW = BROWS / 64, LPW = AW + BW, BM = 64 * MI;
  constexpr int NB = NI * PL;             // B fragments per k16
  constexpr int kStage = (BM + BROWS) * 8;  // 16-byte units per stage
  static_assert(NST == 2 || NST == 3, "two or three stages");
  static_assert(NST * kStage * 16 <= 160 * 1024, "LDS budget");
  const int wm = wv / WN, wn = wv % WN;

  auto issue_one = [&](int st, int j, int kbytes) {
    if (j < AW)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rA, PROBE_LDS_PTR(smem + st * kStage + (wv * AW + j) * 64), 16,
                                               voff[j], kbytes, 0, 0);
    else
      __builtin_amdgcn_raw_ptr_buffer_load_lds(
          rB, PROBE_LDS_PTR(smem + st * kStage + BM * 8 + (wv * BW + (j - AW)) * 64), 16, voff[j], kbytes, 0, 0);
  };
  auto issue_all = [&](int st, int kt) {
#pragma unroll
    for (int j = 0; j < LPW; ++j) issue_one(st, j, (k0 + kt * FBK) * 2);
  };
  int offA[MI], offB[NB];
  const int brow = PERM ? ((lane & 19) | ((lane & 4) << 1) | ((lane & 8) >> 1)) : (lane & 31);
#pragma unroll
  for (int i = 0; i < MI; ++i) offA[i] = (32 * MI * wm + 32 * i + (lane & 31)) * 8;
#pragma unroll
  for (int j = 0; j < NI; ++j)
#pragma unroll
    for (int p = 0; p < PL; ++p)
      offB[j * PL + p] = BM * 8 + (p * 128 * NI + 32 * NI * wn + 32 * j + brow) * 8;
  const int swz = ((lane & 31) >> 1) & 7;  // (row >> 1) & 7: every 32-row block starts at a multiple of 32
  const int swzB = (brow >> 1) & 7;
  auto read_frags = [&](int st, int kk, u32x4(&a)[MI], u32x4(&b)[NB]) {
    const u32x4* sbase = smem + st * kStage;
    const int pc = (2 * kk + (lane >> 5)) ^ swz, pcB = (2 * kk + (lane >> 5)) ^ swzB;
#pragma unroll
    for (int i = 0; i < MI; ++i) a[i] = sbase[offA[i] + pc];
#pragma unroll
    for (int j = 0; j < NB; ++j) b[j] = sbase[offB[j] + pcB];
  };
  // the weight fragment is the row operand: a lane's accumulator registers 4q..4q+3 are four
  // consecutive output columns of one output row
  // MFMA number t of a group: plane slowest, so consecutive MFMAs hit different accumulators
  auto mfma_t = [&](int t, u32x4(&a)[MI], u32x4(&b)[NB]) {
    const int p = t / (MI * NI), i = (t / NI) % MI, j = t % NI;
    acc[i][j] = mfma_32x32x16(b[j * PL + p], a[i], acc[i][j]);
  };
  auto mma = [&](u32x4(&a)[MI], u32x4(&b)[NB]) {
#pragma unroll
    for (int t = 0; t < MI * NI * PL; ++t) mfma_t(t, a, b);
  };

  const int KT = K / FBK;
  u32x4 a0[MI], b0[NB], a1[MI], b1[NB];
  // prologue: NST batches in flight, wait for the first
  issue_all(0, 0);
  if (KT > 1) issue_all(1, 1);
  bool waited = false;
  if constexpr (NST == 3) {
    if (KT > 2) {
      issue_all(2, 2);
      wait_vm_lgkm0<2 * LPW>();
      waited = true;
    }
  }
  if (!waited) {
    if (KT > 1) wait_vm_lgkm0<LPW>(); else wait_vm_lgkm0<0>();
  }
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  read_frags(0, 0, a0, b0);
  // One k-step on stage `cur`.  DMA: issue tile kt+NST into the stage being vacated.
  // YOUNGER: a batch younger than tile kt+1 is in flight at the barrier (it may stay in flight).
  // NEXT: tile kt+1 exists.
  // `hook` runs between the step's wait and its barrier (LDS writes made there are seen by every wave after it).
  auto k_step = [&](int kt, int cur, auto dma_c, auto younger_c, auto next_c, auto hook) {
    constexpr bool DMA = decltype(dma_c)::value, YOUNGER = decltype(younger_c)::value,
                   NEXT = decltype(next_c)::value;
    const int nxt = (cur + 1 == NST) ? 0 : cur + 1;
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): a0/b0 have arrived
    read_frags(cur, 1, a1, b1);
    __builtin_amdgcn_sched_barrier(0);
    mma(a0, b0);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(0xC07F);
    read_frags(cur, 2, a0, b0);
    __builtin_amdgcn_sched_barrier(0);
    mma(a1, b1);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(0xC07F);
    read_frags(cur, 3, a1, b1);
    __builtin_amdgcn_sched_barrier(0);
    mma(a0, b0);
    __builtin_amdgcn_sched_barrier(0);
    // every read of stage cur is issued: wait for them and for this wave's share of tile kt+1
    if constexpr (YOUNGER) wait_vm_lgkm0<LPW>(); else wait_vm_lgkm0<0>();
    hook();
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if constexpr (NEXT) read_frags(nxt, 0, a0, b0);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (DMA) {
      const int kbytes = (k0 + (kt + NST) * FBK) * 2;
      constexpr int NM = MI * NI * PL;
#pragma unroll
      for (int t = 0; t < NM; ++t) {
        mfma_t(t, a1, b1);
        if (t < LPW) issue_one(cur, t, kbytes);
      }
#pragma unroll
      for (int t = NM; t < LPW; ++t) issue_one(cur, t, kbytes);
#pragma unroll
      for (int t = 0; t < (NM < LPW ? NM : LPW); ++t) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one MFMA
        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);  // one VMEM read
      }
    } else {
      mma(a1, b1);
    }
  };
  using T_ = std::integral_constant<bool, true>;
  using F_ = std::integral_constant<bool, false>;
  int kt = 0, cur = 0;
  auto advance = [&]() {
    ++kt;
    cur = (cur + 1 == NST) ? 0 : cur + 1;
  };
  auto none = []() {};
  bool drew = false;
  auto step_before_last = [&]() {
    if constexpr (DRAW) {
      int ticket = 0;
      if (threadIdx.x == 0) ticket = atomicAdd(draw_counter, 1);
      k_step(kt, cur, F_{}, F_{}, T_{}, [&]() {
        if (threadIdx.x == 0) *draw_slot = ticket;
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the write has landed before the barrier
      });
      drew = true;
    } else {
      k_step(kt, cur, F_{}, F_{}, T_{}, none);
    }
  };
  if constexpr (NST == 2) {
    while (kt + 2 < KT) {
      k_step(kt, cur, T_{}, F_{}, T_{}, none);
      advance();
    }
    if (kt + 1 < KT) {
      step_before_last();
      advance();
    }
  } else {
    while (kt + 3 < KT) {
      k_step(kt, cur, T_{}, T_{}, T_{}, none);
      advance();
    }
    if (kt + 2 < KT) {
      k_step(kt, cur, F_{}, T_{}, T_{}, none);
      advance();
    }
    if (kt + 1 < KT) {
      step_before_last();
      advance();
    }
  }
  k_step(kt, cur, F_{}, F_{}, F_{}, none);
  return drew;
}

// Raw buffer descriptor over [base, base + bytes): loads past the end return zero.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, size_t bytes) {
  unsigned n = bytes > 0xffffffffull ? 0xffffffffu : static_cast<unsigned>(bytes);
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, static_cast<int>(n), 0x00020000);
}

// Per-lane byte offsets of the DMA instructions of this wave: instruction j covers tile rows
// (wv*CNT + j)*8 .. +8; lane l reads row +l/8, the chunk that belongs at LDS position l%8.
template <int CNT, typename RowFn>
__device__ __forceinline__ void dma_offsets(int wv, int lane, int row_bytes, RowFn row_of, int* out) {
#pragma unroll
  for (int j = 0; j < CNT; ++j) {
    int row = (wv * CNT + j) * 8 + (lane >> 3);
    int c = (lane & 7) ^ ((row >> 1) & 7);
    out[j] = row_of(row) * row_bytes + c * 16;
  }
}

}  // namespace probe
