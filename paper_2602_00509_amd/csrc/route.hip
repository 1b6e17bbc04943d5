// probe_route_topk / probe_predict_topk: gate logits on the matrix cores, softmax, top-k.
//
// The gate is x[T,H] (bf16) times w_gate[E,H] (fp32).  At E = 128..256 this is far above the
// fp32 vector ridge of the chip, so the product runs on the bf16 MFMA units without giving up
// fp32 weights: every weight is split (once, by probe_pack_gate, or inside the call) into three bf16 planes hi + mid + lo
// (each the round-to-nearest bf16 of what the previous planes left over), which together
// carry all 24 significand bits.  x is bf16 already, every bf16 x bf16 product is exact in
// fp32, and the MFMA accumulates in fp32.
//
//   1. split    w_gate -> planes[3][E][H] bf16 in the workspace (skipped by the *_packed entry points,
//               which are handed planes made once by probe_pack_gate)
//   2. gemm     split-K tiled GEMM (128 tokens x 128 experts x 64 k per step), three MFMAs per
//               operand pair (one per plane) into one accumulator  -> partial[KS][T][E] fp32;
//               its first workgroup clears the expert counts
//               H % 64 == 0: DMA-to-LDS software pipeline shared with the grouped FFN;
//               otherwise a register-staged kernel that zero-fills the K tail
//   3. softmax  sixteen lanes per token: sum the KS partials in fixed order, add the bias,
//               softmax over E, k rounds of row arg-max (ties to the lower index), weights, counts
//
// The predictor's residual MLP (Eq. 7) adds W2_hat silu(W1_hat h) to the logits before step 3:
//   a. the same GEMM with one bf16 plane of W1_hat (D rows in place of experts) -> u partials
//   b. sum of the u partials, SiLU in fp32, split of s = silu(u) into three bf16 planes laid side
//      by side along K: A' = [s_hi | s_mid | s_lo], [T][3D]
//   c. W2_hat split into planes arranged as B' = {[hi hi hi], [mid mid 0], [lo 0 0]}, [3][E][3D],
//      so that step 2's three-plane GEMM over K = 3D forms the six largest of the nine plane
//      products (what is dropped is below 2^-24 of the result)
//   d. that GEMM; its split-K slices are written behind the gate's own, and step 3 sums them all
#include <limits.h>

#include <mutex>

#include "common.hpp"
#include "mfma_pipeline.hpp"

namespace probe {

constexpr int GBM = 128, GBN = 128, GBK = 64;

// ---- 1. split -------------------------------------------------------------------------
// planes + plane_stride * p is plane p; `planes` already points at this gate's rows inside a plane
__global__ __launch_bounds__(256) void gate_split_kernel(const float* __restrict__ w, long n,
                                                         bf16_t* __restrict__ planes, long plane_stride,
                                                         int32_t* __restrict__ counts, int E) {
  long gid = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (counts && gid < E) counts[gid] = 0;
  if (gid >= n) return;
  float v = w[gid];
  bf16_t hi = f32_to_bf16(v);
  float r1 = v - bf16_to_f32(hi);  // exact
  bf16_t mid = f32_to_bf16(r1);
  float r2 = r1 - bf16_to_f32(mid);  // exact
  bf16_t lo = f32_to_bf16(r2);
  planes[gid] = hi;
  planes[plane_stride + gid] = mid;
  planes[2 * plane_stride + gid] = lo;
}

// The expert counts that the softmax / top-k kernel adds to are cleared by the first workgroup of
// the GEMM that precedes it on the stream (n <= 256 <= threads per workgroup).
__device__ __forceinline__ void zero_counts(int32_t* __restrict__ a, int32_t* __restrict__ b, int n) {
  if (blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && static_cast<int>(threadIdx.x) < n) {
    if (a) a[threadIdx.x] = 0;
    if (b) b[threadIdx.x] = 0;
  }
}

// ---- 2. gemm --------------------------------------------------------------------------
template <int PL>
__global__ __launch_bounds__(256, 2) void gate_gemm_kernel(const bf16_t* __restrict__ x,
                                                           const bf16_t* __restrict__ planes,
                                                           int T, int H, int E, int k_chunk,
                                                           float* __restrict__ partial,
                                                           int32_t* __restrict__ zero0, int32_t* __restrict__ zero1,
                                                           int n_zero) {
  __shared__ u32x4 sA[GBM * 8];
  __shared__ u32x4 sB[PL][GBN * 8];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int wm = wv >> 1, wn = wv & 1;
  const int m0 = blockIdx.x * GBM, n0 = blockIdx.y * GBN, ks = blockIdx.z;
  zero_counts(zero0, zero1, n_zero);
  const int kbeg = ks * k_chunk, kend = min(H, kbeg + k_chunk);
  const long plane_elems = static_cast<long>(E) * H;

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  u32x4 ra[4], rb[PL][4];
  auto gload = [&](int k0) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int idx = tid + 256 * j;
      int row = idx >> 3, c = idx & 7;
      int kk = k0 + c * 8;
      bool kin = kk < kend;
      int grow = m0 + row, brow = n0 + row;
      ra[j] = u32x4{0u, 0u, 0u, 0u};
      if (kin && grow < T) ra[j] = *reinterpret_cast<const u32x4*>(x + static_cast<long>(grow) * H + kk);
#pragma unroll
      for (int p = 0; p < PL; ++p) {
        rb[p][j] = u32x4{0u, 0u, 0u, 0u};
        if (kin && brow < E)
          rb[p][j] = *reinterpret_cast<const u32x4*>(planes + p * plane_elems + static_cast<long>(brow) * H + kk);
      }
    }
  };
  auto sstore = [&]() {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int idx = tid + 256 * j;
      int row = idx >> 3, c = idx & 7;
      sA[lds_chunk_off(row, c)] = ra[j];
#pragma unroll
      for (int p = 0; p < PL; ++p) sB[p][lds_chunk_off(row, c)] = rb[p][j];
    }
  };

  if (kbeg < kend) {
    gload(kbeg);
    sstore();
  }
  __syncthreads();
  for (int k0 = kbeg; k0 < kend; k0 += GBK) {
    const bool more = k0 + GBK < kend;
    if (more) gload(k0 + GBK);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const int c = 2 * kk + (lane >> 5);
      u32x4 a[2];
#pragma unroll
      for (int mi = 0; mi < 2; ++mi) a[mi] = sA[lds_chunk_off(64 * wm + 32 * mi + (lane & 31), c)];
#pragma unroll
      for (int p = PL - 1; p >= 0; --p) {
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
          u32x4 b = sB[p][lds_chunk_off(64 * wn + 32 * ni + (lane & 31), c)];
#pragma unroll
          for (int mi = 0; mi < 2; ++mi) acc[mi][ni] = mfma_32x32x16(a[mi], b, acc[mi][ni]);
        }
      }
    }
    __syncthreads();
    if (more) {
      sstore();
      __syncthreads();
    }
  }
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
      int col = n0 + 64 * wn + 32 * ni + mfma32_col(lane);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        int row = m0 + 64 * wm + 32 * mi + mfma32_row(r, lane);
        if (row < T && col < E) partial[(static_cast<long>(ks) * T + row) * E + col] = acc[mi][ni][r];
      }
    }
}

// ---- 2b. gemm, DMA pipeline (H % 64 == 0) --------------------------------------------
// Same split-K tiling (128 tokens x 128 experts per workgroup), on the software pipeline of the
// grouped FFN: 8 waves (2 x 4, wave tile 64 tokens x 32 experts), buffer_load-to-LDS, two LDS
// stages of 64 KB = 128 token rows + 3 planes x 128 expert rows, three MFMAs (one per plane) per
// operand pair into one accumulator.  The weight fragment is the MFMA's row operand, so a lane
// ends with four consecutive experts of one token per register quad: 16-byte stores.
// MI = 2: 128 tokens per workgroup; MI = 4: 256 tokens (two stages of 80 KB, all of the LDS), which
// moves a third less operand data per MFMA and is used for large batches.
constexpr int kGateLdsBytes = 2 * (256 + 384) * 128;

template <int MI, int PL>
__global__ __launch_bounds__(512, 2) void gate_gemm_dma_kernel(const bf16_t* __restrict__ x,
                                                               const bf16_t* __restrict__ planes,
                                                               int T, int H, int E, int k_chunk,
                                                               float* __restrict__ partial,
                                                               int32_t* __restrict__ zero0,
                                                               int32_t* __restrict__ zero1, int n_zero) {
#if defined(__HIP_DEVICE_COMPILE__)
  extern __shared__ u32x4 smem[];
  const int lane = threadIdx.x & 63;
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wv / 4, wn = wv % 4;
  const int m0 = blockIdx.x * (64 * MI), n0 = blockIdx.y * GBN, ks = blockIdx.z;
  zero_counts(zero0, zero1, n_zero);
  const int kbeg = ks * k_chunk, klen = min(H, kbeg + k_chunk) - kbeg;
  if (klen <= 0) return;
  const int rows = T - m0;
  __amdgpu_buffer_rsrc_t rA = make_rsrc(x + static_cast<size_t>(m0) * H, static_cast<size_t>(rows) * H * 2);
  __amdgpu_buffer_rsrc_t rB = make_rsrc(planes, static_cast<size_t>(PL) * E * H * 2);
  int voff[MI + 2 * PL];
  dma_offsets<MI>(wv, lane, H * 2, [&](int r) { return min(r, rows - 1); }, voff);
  // B-tile row j: plane j / 128, expert n0 + j % 128 (clamped; columns past E are masked at the store)
  dma_offsets<2 * PL>(wv, lane, H * 2, [&](int j) { return (j >> 7) * E + min(n0 + (j & 127), E - 1); }, voff + MI);
  f32x16 acc[MI][1];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][0][r] = 0.f;
  gemm_mainloop<MI, 1, PL, 2>(rA, rB, voff, kbeg, klen, smem, wv, lane, acc);

  const bool vec = (E & 3) == 0;
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
    const int row = 32 * MI * wm + 32 * mi + (lane & 31);
    if (row < rows) {
      float* dst = partial + (static_cast<long>(ks) * T + m0 + row) * E;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int col = n0 + 32 * wn + 8 * q + 4 * (lane >> 5);
        if (vec) {
          if (col < E)
            *reinterpret_cast<float4*>(dst + col) =
                make_float4(acc[mi][0][4 * q], acc[mi][0][4 * q + 1], acc[mi][0][4 * q + 2], acc[mi][0][4 * q + 3]);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (col + e < E) dst[col + e] = acc[mi][0][4 * q + e];
        }
      }
    }
  }
#endif
}

static int gate_prepare() {
  static std::mutex mu;
  static bool done[64] = {false};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
    set_error("probe_route_topk: no current device");
    return PROBE_EHIP;
  }
  std::lock_guard<std::mutex> lock(mu);
  if (done[dev]) return PROBE_OK;
  hipError_t err = hipSuccess;
  const void* kernels[4] = {reinterpret_cast<const void*>(gate_gemm_dma_kernel<2, 3>),
                            reinterpret_cast<const void*>(gate_gemm_dma_kernel<4, 3>),
                            reinterpret_cast<const void*>(gate_gemm_dma_kernel<2, 1>),
                            reinterpret_cast<const void*>(gate_gemm_dma_kernel<4, 1>)};
  for (int i = 0; i < 4 && err == hipSuccess; ++i)
    err = hipFuncSetAttribute(kernels[i], hipFuncAttributeMaxDynamicSharedMemorySize, kGateLdsBytes);
  if (err != hipSuccess) {
    set_error("probe_route_topk: cannot reserve %d bytes of LDS: %s", kGateLdsBytes, hipGetErrorString(err));
    return PROBE_EHIP;
  }
  done[dev] = true;
  return PROBE_OK;
}

// ---- 3. softmax + top-k ---------------------------------------------------------------
// Sixteen lanes (one DPP row) own one token, a wave owns four.  Lane `sub` of a row holds the
// experts 64*i + 4*sub + j (i < NV, j < 4), i.e. 16-byte pieces of the logit row, so partial
// sums are read with float4 loads and every reduction stays inside a row: four rotate-and-
// combine DPP steps give all 16 lanes the same result bit for bit.
template <int N>
__device__ __forceinline__ float dpp_ror(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x120 | N, 0xf, 0xf, false));
}
template <int N>
__device__ __forceinline__ int dpp_ror(int v) {
  return __builtin_amdgcn_update_dpp(0, v, 0x120 | N, 0xf, 0xf, false);
}
__device__ __forceinline__ float row_max(float v) {
  v = fmaxf(v, dpp_ror<8>(v));
  v = fmaxf(v, dpp_ror<4>(v));
  v = fmaxf(v, dpp_ror<2>(v));
  v = fmaxf(v, dpp_ror<1>(v));
  return v;
}
__device__ __forceinline__ float row_sum(float v) {
  v += dpp_ror<8>(v);
  v += dpp_ror<4>(v);
  v += dpp_ror<2>(v);
  v += dpp_ror<1>(v);
  return v;
}
// arg-max of (value, expert): larger value wins, equal values go to the lower expert id
template <int N>
__device__ __forceinline__ void argmax_step(float& v, int& e) {
  float ov = dpp_ror<N>(v);
  int oe = dpp_ror<N>(e);
  bool take = (oe != INT_MAX) && (e == INT_MAX || ov > v || (ov == v && oe < e));
  v = take ? ov : v;
  e = take ? oe : e;
}

__device__ __forceinline__ int row_min_i(int v) {
  v = min(v, dpp_ror<8>(v));
  v = min(v, dpp_ror<4>(v));
  v = min(v, dpp_ror<2>(v));
  v = min(v, dpp_ror<1>(v));
  return v;
}

// Pairwise (tree) reductions over a register array: depth log2(N) instead of a chain of N - 1
// dependent operations; max and min are exact, so the result does not depend on the order.
template <int N>
__device__ __forceinline__ float tree_max(const float (&v)[N]) {
  float t[N];
#pragma unroll
  for (int i = 0; i < N; ++i) t[i] = v[i];
#pragma unroll
  for (int st = 1; st < N; st *= 2)
#pragma unroll
    for (int i = 0; i + st < N; i += 2 * st) t[i] = fmaxf(t[i], t[i + st]);
  return t[0];
}
template <int N>
__device__ __forceinline__ int tree_min(const int (&v)[N]) {
  int t[N];
#pragma unroll
  for (int i = 0; i < N; ++i) t[i] = v[i];
#pragma unroll
  for (int st = 1; st < N; st *= 2)
#pragma unroll
    for (int i = 0; i + st < N; i += 2 * st) t[i] = min(t[i], t[i + st]);
  return t[0];
}

// Logit row pieces of U tokens: the KS split-K slices are added in ascending order, then the bias row
// of the token's group.  Lane `sub` receives the experts 64*i + 4*sub + j; entries past E are zero.
template <int NV, int U, int R = 2>
__device__ __forceinline__ void load_logit_rows(const float* __restrict__ partial, int ld, int KS,
                                                const float* __restrict__ bias, int G, int tpg, int T, int E,
                                                bool vec, int sub, const int (&tt)[U], float (&l)[U][NV * 4]) {
  constexpr int NL = NV * 4;
  if (vec) {
    float4 accv[U][NV];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int i = 0; i < NV; ++i) accv[u][i] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int q0 = 0; q0 < KS; q0 += R) {
      // all loads of a round of R split-K slices (of every token of the row) are issued before any is consumed
      float4 tmp[R][U][NV];
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const int q = min(q0 + r, KS - 1);
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
          for (int i = 0; i < NV; ++i) {
            const int e0 = min(64 * i + 4 * sub, E - 4);
            tmp[r][u][i] = *reinterpret_cast<const float4*>(partial + (static_cast<long>(q) * T + tt[u]) * ld + e0);
          }
      }
#pragma unroll
      for (int r = 0; r < R; ++r)
        if (q0 + r < KS) {
#pragma unroll
          for (int u = 0; u < U; ++u)
#pragma unroll
            for (int i = 0; i < NV; ++i) {
              accv[u][i].x += tmp[r][u][i].x; accv[u][i].y += tmp[r][u][i].y;
              accv[u][i].z += tmp[r][u][i].z; accv[u][i].w += tmp[r][u][i].w;
            }
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int g = 0;
      if (bias) g = min(tt[u] / tpg, G - 1);
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int e0 = 64 * i + 4 * sub;
        float4 bv = make_float4(0.f, 0.f, 0.f, 0.f);
        if (bias && e0 < E) bv = *reinterpret_cast<const float4*>(bias + static_cast<long>(g) * E + e0);
        l[u][4 * i] = accv[u][i].x + bv.x;
        l[u][4 * i + 1] = accv[u][i].y + bv.y;
        l[u][4 * i + 2] = accv[u][i].z + bv.z;
        l[u][4 * i + 3] = accv[u][i].w + bv.w;
      }
    }
  } else {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int g = 0;
      if (bias) g = min(tt[u] / tpg, G - 1);
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        const int e = 64 * (i >> 2) + 4 * sub + (i & 3);
        float sacc = 0.f;
        if (e < E) {
          for (int q = 0; q < KS; ++q) sacc += partial[(static_cast<long>(q) * T + tt[u]) * ld + e];
          if (bias) sacc += bias[static_cast<long>(g) * E + e];
        }
        l[u][i] = sacc;
      }
    }
  }
}

// Two tokens per row are in flight (U = 2) so that the dependent DPP chains of one overlap the
// other's.  A chosen logit is overwritten with -inf; incoming logits are clamped to >= -FLT_MAX
// (NaN too), so -inf only ever means "taken".  The weight of a winner is recomputed from its
// logit with the same expression as its probability, so both agree bit for bit.
template <int NV, int U = 2, int R = 2>
__global__ __launch_bounds__(256) void gate_softmax_topk_kernel(
    const float* __restrict__ partial, int ld, int KS, const float* __restrict__ bias, int G, int tpg, int T,
    int E, int k, int renorm, int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
    float* __restrict__ probs, int32_t* __restrict__ counts) {
  // `partial` points at this gate's first column; a row of a partial plane has ld entries
  constexpr int NL = NV * 4;
  __shared__ int32_t hist[PROBE_MAX_EXPERTS];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int sub = lane & 15, grp = lane >> 4;
  hist[tid] = 0;
  __syncthreads();
  const float ninf = -__builtin_inff(), fmin_ = -3.402823466e38f;
  const bool vec = (E & 3) == 0 && (ld & 3) == 0;
  const int tokens_per_pass = gridDim.x * 16 * U;
  for (int t0 = ((blockIdx.x * 4 + wv) * U) * 4 + grp; t0 < T; t0 += tokens_per_pass) {
    // token u of this row is t0 + 4u; the rows of a wave are independent under DPP row operations
    int tt[U];
    bool live[U];
    float l[U][NL];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      live[u] = t0 + 4 * u < T;
      tt[u] = live[u] ? t0 + 4 * u : t0;
    }
    load_logit_rows<NV, U, R>(partial, ld, KS, bias, G, tpg, T, E, vec, sub, tt, l);
    float mx[U], inv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      // clamp (NaN and -inf become the most negative finite value); experts past E are "taken"
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        const int e = 64 * (i >> 2) + 4 * sub + (i & 3);
        float v = l[u][i];
        v = (v >= fmin_) ? v : fmin_;
        l[u][i] = (e < E) ? v : ninf;
      }
      mx[u] = row_max(tree_max(l[u]));
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float p[NL], sum = 0.f;
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        p[i] = expf(l[u][i] - mx[u]);  // exp(-inf) = 0 for the experts past E
        sum += p[i];
      }
      sum = row_sum(sum);
      inv[u] = 1.f / sum;
      if (probs && live[u]) {
        const long t = t0 + 4 * u;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
          const int e0 = 64 * i + 4 * sub;
          if (vec) {
            if (e0 < E)
              *reinterpret_cast<float4*>(probs + t * E + e0) =
                  make_float4(p[4 * i] * inv[u], p[4 * i + 1] * inv[u], p[4 * i + 2] * inv[u], p[4 * i + 3] * inv[u]);
          } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
              if (e0 + j < E) probs[t * E + e0 + j] = p[4 * i + j] * inv[u];
          }
        }
      }
    }
    int isel[U];
    float wsel[U], wtot[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      isel[u] = 0;
      wsel[u] = 0.f;
      wtot[u] = 0.f;
    }
    for (int s = 0; s < k; ++s) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const float best = row_max(tree_max(l[u]));
        // lowest expert id among the entries that hold the row maximum
        int cand[NL];
#pragma unroll
        for (int i = 0; i < NL; ++i) {
          const int e = 64 * (i >> 2) + 4 * sub + (i & 3);
          cand[i] = (l[u][i] == best) ? e : INT_MAX;
        }
        const int be = row_min_i(tree_min(cand));
        // its owner marks it taken
#pragma unroll
        for (int i = 0; i < NL; ++i) {
          const int e = 64 * (i >> 2) + 4 * sub + (i & 3);
          l[u][i] = (e == be) ? ninf : l[u][i];
        }
        const float pw = expf(best - mx[u]) * inv[u];
        wtot[u] += pw;
        if (sub == s) {
          isel[u] = be;
          wsel[u] = pw;
        }
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (renorm) wsel[u] /= wtot[u];
      if (live[u] && sub < k) {
        const long t = t0 + 4 * u;
        topk_idx[t * k + sub] = isel[u];
        topk_w[t * k + sub] = wsel[u];
        if (counts) atomicAdd(&hist[isel[u]], 1);
      }
    }
  }
  __syncthreads();
  if (counts && tid < E && hist[tid] != 0) atomicAdd(&counts[tid], hist[tid]);
}

// (m1, m2) = the two largest of this lane's pair and the pair N lanes away in the row
template <int N>
__device__ __forceinline__ void top2_merge(float& m1, float& m2) {
  const float o1 = dpp_ror<N>(m1), o2 = dpp_ror<N>(m2);
  m2 = fmaxf(fminf(m1, o1), fmaxf(m2, o2));
  m1 = fmaxf(m1, o1);
}

// ---- 3b. group-limited gate -----------------------------------------------------------------
// Same lane layout and logit loading as above.  Per token: scores s (sigmoid of each logit, or the
// softmax), selection scores c = s + select_bias, a score per group of E / n_group consecutive
// experts (sum of its group_top largest c), the topk_group best groups, the k largest c among their
// experts, gating values from s.  Every decision is an arg-max over a DPP row with ties to the
// lower index, so all sixteen lanes of a token agree bit for bit.  Lane j keeps the score of group
// j (n_group <= 16); sets of groups and of consumed entries are bit masks.
template <int NV>
__global__ __launch_bounds__(256) void gate_grouped_topk_kernel(
    const float* __restrict__ partial, int ld, int KS, const float* __restrict__ bias, int G, int tpg,
    const float* __restrict__ select_bias, int T, int E, int k, int scoring, int n_group, int topk_group,
    int group_top, int renorm, float routed_scale, int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
    float* __restrict__ scores, int32_t* __restrict__ counts) {
  constexpr int U = 2, NL = NV * 4;
  __shared__ int32_t hist[PROBE_MAX_EXPERTS];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int sub = lane & 15, grp = lane >> 4;
  hist[tid] = 0;
  __syncthreads();
  const float ninf = -__builtin_inff(), fmin_ = -3.402823466e38f;
  const bool vec = (E & 3) == 0 && (ld & 3) == 0;
  const int gs = E / n_group;
  int gid[NL];      // group of entry i, -1 past E
  float sb[NL];
#pragma unroll
  for (int i = 0; i < NL; ++i) {
    const int e = 64 * (i >> 2) + 4 * sub + (i & 3);
    gid[i] = e < E ? e / gs : -1;
    sb[i] = (select_bias && e < E) ? select_bias[e] : 0.f;
  }
  const int tokens_per_pass = gridDim.x * 16 * U;
  for (int t0 = ((blockIdx.x * 4 + wv) * U) * 4 + grp; t0 < T; t0 += tokens_per_pass) {
    int tt[U];
    bool live[U];
    float sc[U][NL], c[U][NL];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      live[u] = t0 + 4 * u < T;
      tt[u] = live[u] ? t0 + 4 * u : t0;
    }
    load_logit_rows<NV, U>(partial, ld, KS, bias, G, tpg, T, E, vec, sub, tt, sc);
    // scores (in place of the logits) and selection scores
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        float v = sc[u][i];
        v = (v >= fmin_) ? v : fmin_;  // NaN and -inf become the most negative finite value
        sc[u][i] = (gid[i] >= 0) ? v : ninf;
      }
      if (scoring == 1) {
#pragma unroll
        for (int i = 0; i < NL; ++i) sc[u][i] = 1.f / (1.f + expf(-sc[u][i]));  // 0 past E
      } else {
        const float m = row_max(tree_max(sc[u]));
        float sum = 0.f;
#pragma unroll
        for (int i = 0; i < NL; ++i) {
          sc[u][i] = expf(sc[u][i] - m);
          sum += sc[u][i];
        }
        const float inv = 1.f / row_sum(sum);
#pragma unroll
        for (int i = 0; i < NL; ++i) sc[u][i] *= inv;
      }
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        float v = sc[u][i] + sb[i];
        v = (v >= fmin_) ? v : fmin_;
        c[u][i] = (gid[i] >= 0) ? v : ninf;
      }
      if (scores && live[u]) {
        const long t = t0 + 4 * u;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
          const int e0 = 64 * i + 4 * sub;
          if (vec) {
            if (e0 < E)
              *reinterpret_cast<float4*>(scores + t * E + e0) =
                  make_float4(sc[u][4 * i], sc[u][4 * i + 1], sc[u][4 * i + 2], sc[u][4 * i + 3]);
          } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
              if (e0 + j < E) scores[t * E + e0 + j] = sc[u][4 * i + j];
          }
        }
      }
    }
    // group scores.  Only the VALUES of a group's largest selection scores matter, so for
    // group_top <= 2 a (largest, second) pair is merged across the row with max / min, which is
    // exact and order-free; otherwise group_top rounds of arg-max inside the group.
    float gscore[U];
#pragma unroll
    for (int u = 0; u < U; ++u) gscore[u] = ninf;
    if (group_top <= 2) {
      for (int j = 0; j < n_group; ++j) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
          float m1 = ninf, m2 = ninf;
#pragma unroll
          for (int i = 0; i < NL; ++i) {
            const float v = (gid[i] == j) ? c[u][i] : ninf;
            m2 = fmaxf(m2, fminf(m1, v));
            m1 = fmaxf(m1, v);
          }
          top2_merge<8>(m1, m2);
          top2_merge<4>(m1, m2);
          top2_merge<2>(m1, m2);
          top2_merge<1>(m1, m2);
          const float sum = (group_top == 2) ? m1 + m2 : m1;
          gscore[u] = (sub == j) ? sum : gscore[u];
        }
      }
    } else {
      unsigned used[U];
#pragma unroll
      for (int u = 0; u < U; ++u) used[u] = 0u;
      for (int j = 0; j < n_group; ++j) {
        float sum[U];
#pragma unroll
        for (int u = 0; u < U; ++u) sum[u] = 0.f;
        for (int r = 0; r < group_top; ++r) {
#pragma unroll
          for (int u = 0; u < U; ++u) {
            float m = ninf;
#pragma unroll
            for (int i = 0; i < NL; ++i) {
              const bool open = gid[i] == j && !((used[u] >> i) & 1u);
              m = open ? fmaxf(m, c[u][i]) : m;
            }
            const float best = row_max(m);
            int cand = INT_MAX;
#pragma unroll
            for (int i = NL - 1; i >= 0; --i) {
              const int e = 64 * (i >> 2) + 4 * sub + (i & 3);
              const bool open = gid[i] == j && !((used[u] >> i) & 1u);
              cand = (open && c[u][i] == best) ? e : cand;
            }
            const int be = row_min_i(cand);
#pragma unroll
            for (int i = 0; i < NL; ++i) {
              const int e = 64 * (i >> 2) + 4 * sub + (i & 3);
              used[u] |= (e == be) ? (1u << i) : 0u;
            }
            sum[u] += best;
          }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) gscore[u] = (sub == j) ? sum[u] : gscore[u];
      }
    }
    // allowed groups
    unsigned allowed[U];
#pragma unroll
    for (int u = 0; u < U; ++u) allowed[u] = 0u;
    for (int r = 0; r < topk_group; ++r) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const bool open = sub < n_group && !((allowed[u] >> sub) & 1u);
        const float best = row_max(open ? gscore[u] : ninf);
        const int bg = row_min_i((open && gscore[u] == best) ? sub : INT_MAX);
        allowed[u] |= 1u << (bg & 15);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        const bool ok = gid[i] >= 0 && ((allowed[u] >> (gid[i] & 15)) & 1u);
        c[u][i] = ok ? c[u][i] : ninf;
      }
    // k largest selection scores among the allowed experts; -inf now means "not available"
    int isel[U];
    float wsel[U], wtot[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      isel[u] = 0;
      wsel[u] = 0.f;
      wtot[u] = 0.f;
    }
    for (int s = 0; s < k; ++s) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const float best = row_max(tree_max(c[u]));
        int cand[NL];
#pragma unroll
        for (int i = 0; i < NL; ++i) {
          const int e = 64 * (i >> 2) + 4 * sub + (i & 3);
          cand[i] = (c[u][i] == best) ? e : INT_MAX;
        }
        const int be = row_min_i(tree_min(cand));
        float mine = ninf;  // the owner's score of the winner, without the selection bias
#pragma unroll
        for (int i = 0; i < NL; ++i) {
          const int e = 64 * (i >> 2) + 4 * sub + (i & 3);
          mine = (e == be) ? sc[u][i] : mine;
          c[u][i] = (e == be) ? ninf : c[u][i];
        }
        const float pw = row_max(mine);
        wtot[u] += pw;
        if (sub == s) {
          isel[u] = be;
          wsel[u] = pw;
        }
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (renorm) wsel[u] /= wtot[u];
      wsel[u] *= routed_scale;
      if (live[u] && sub < k) {
        const long t = t0 + 4 * u;
        topk_idx[t * k + sub] = isel[u];
        topk_w[t * k + sub] = wsel[u];
        if (counts) atomicAdd(&hist[isel[u]], 1);
      }
    }
  }
  __syncthreads();
  if (counts && tid < E && hist[tid] != 0) atomicAdd(&counts[tid], hist[tid]);
}

// ---- 4. residual of the predictor (Eq. 7) ------------------------------------------------
// r[t,e] = sum_d w2_hat[e,d] * s[t,d],  s = silu(u),  u = W1_hat h summed over its split-K partials.
// Both factors are fp32; the product runs on the matrix cores at fp32 accuracy by splitting each
// factor into bf16 planes (hi + mid + lo, as for the gate) and keeping the six largest of the nine
// plane products: with the planes of s laid side by side along K,
//     A'[t]   = [ s_hi | s_mid | s_lo ]                         (bf16 [T, 3D])
//     B'_0[e] = [ w_hi | w_hi  | w_hi ],  B'_1[e] = [ w_mid | w_mid | 0 ],  B'_2[e] = [ w_lo | 0 | 0 ]
// the three-plane GEMM of the gate computes  s_hi (w_hi + w_mid + w_lo) + s_mid (w_hi + w_mid) + s_lo w_hi;
// the dropped products are below 2^-24 of the result.  Its split-K slices are written behind the
// gate's own, so the softmax / top-k kernel adds the residual like further slices of the logits.
__global__ __launch_bounds__(256) void resid_silu_split_kernel(const float* __restrict__ upartial, int KS2, int T,
                                                               int D, bf16_t* __restrict__ a_planes) {
  // one thread per 8 consecutive hidden units of one token
  const long gid = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x;
  const int groups = D / 8;
  if (gid >= static_cast<long>(T) * groups) return;
  const int t = static_cast<int>(gid / groups), d0 = static_cast<int>(gid % groups) * 8;
  float u[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) u[j] = 0.f;
  for (int q = 0; q < KS2; ++q) {
    const float4* src = reinterpret_cast<const float4*>(upartial + (static_cast<long>(q) * T + t) * D + d0);
    const float4 lo = src[0], hi = src[1];
    u[0] += lo.x; u[1] += lo.y; u[2] += lo.z; u[3] += lo.w;
    u[4] += hi.x; u[5] += hi.y; u[6] += hi.z; u[7] += hi.w;
  }
  uint32_t pk[3][4];
#pragma unroll
  for (int j = 0; j < 8; j += 2) {
    float v[2], p1[2], p2[2], p3[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      v[i] = u[j + i] / (1.f + expf(-u[j + i]));
      p1[i] = bf16_to_f32(f32_to_bf16(v[i]));
      const float r1 = v[i] - p1[i];          // exact
      p2[i] = bf16_to_f32(f32_to_bf16(r1));
      p3[i] = r1 - p2[i];                     // exact; rounded to bf16 by the pack below
    }
    pk[0][j / 2] = pack_bf16x2(p1[0], p1[1]);
    pk[1][j / 2] = pack_bf16x2(p2[0], p2[1]);
    pk[2][j / 2] = pack_bf16x2(p3[0], p3[1]);
  }
  bf16_t* row = a_planes + static_cast<long>(t) * 3 * D + d0;
#pragma unroll
  for (int p = 0; p < 3; ++p) {
    u32x4 v = {pk[p][0], pk[p][1], pk[p][2], pk[p][3]};
    *reinterpret_cast<u32x4*>(row + p * D) = v;
  }
}

__global__ __launch_bounds__(256) void resid_w2_split_kernel(const float* __restrict__ w2_hat, int E, int D,
                                                             bf16_t* __restrict__ b_planes) {
  const long gid = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (gid >= static_cast<long>(E) * D) return;
  const int e = static_cast<int>(gid / D), d = static_cast<int>(gid % D);
  const float v = w2_hat[gid];
  const bf16_t hi = f32_to_bf16(v);
  const float r1 = v - bf16_to_f32(hi);
  const bf16_t mid = f32_to_bf16(r1);
  const bf16_t lo = f32_to_bf16(r1 - bf16_to_f32(mid));
  const long plane = static_cast<long>(E) * 3 * D;
  bf16_t* row = b_planes + static_cast<long>(e) * 3 * D + d;
  row[0] = hi;          row[D] = hi;            row[2 * D] = hi;
  row[plane] = mid;     row[plane + D] = mid;   row[plane + 2 * D] = 0;
  row[2 * plane] = lo;  row[2 * plane + D] = 0; row[2 * plane + 2 * D] = 0;
}

struct RouteShape {
  bool dma;  // H % 64 == 0: the DMA-to-LDS pipeline; otherwise the register-staged kernel
  int bm;    // tokens per workgroup of the gemm (128 or 256)
  int mt, nt, ks, k_chunk;
  size_t planes_bytes, partial_bytes;
};

constexpr int kMaxSplitK = 16;

static RouteShape route_shape(int T, int H, int E, int max_split = kMaxSplitK) {
  RouteShape s;
  // 256-token tiles when a split of 8 or less still gives every CU a workgroup; they aim at one
  // workgroup per CU (fewer, longer K ranges and half the partial sums), 128-token tiles at two
  s.dma = H % 64 == 0 && static_cast<size_t>(3) * E * H * 2 <= 0x7fffffffull;
  s.nt = (E + GBN - 1) / GBN;
  s.bm = (s.dma && static_cast<long>((T + 255) / 256) * s.nt * 8 >= 256) ? 256 : GBM;
  s.mt = (T + s.bm - 1) / s.bm;
  int tiles = s.mt * s.nt;
  int ksteps = (H + GBK - 1) / GBK;
  const int target = s.bm == 256 ? 256 : 512;
  int want = tiles > 0 ? (target + tiles - 1) / tiles : 1;
  if (want < 1) want = 1;
  if (want > max_split) want = max_split;  // the softmax kernel adds the slices one after another
  if (want > ksteps) want = ksteps;
  int steps_per = (ksteps + want - 1) / want;
  s.k_chunk = steps_per * GBK;
  s.ks = (ksteps + steps_per - 1) / steps_per;
  s.planes_bytes = align_up(static_cast<size_t>(3) * E * H * sizeof(bf16_t), 256);
  s.partial_bytes = align_up(static_cast<size_t>(s.ks) * (T > 0 ? T : 1) * E * sizeof(float), 256);
  return s;
}

// x [T,H] times a stack of PL bf16 planes [PL][N][H] -> partial [ks][T][N] fp32
template <int PL>
static void launch_gate_gemm(const RouteShape& sh, hipStream_t st, const bf16_t* x, const bf16_t* planes, int T,
                             int H, int N, float* partial, int32_t* zero0 = nullptr, int32_t* zero1 = nullptr,
                             int n_zero = 0) {
  if (sh.dma) {
    const int lds = 2 * (sh.bm + 128 * PL) * 128;
    if (sh.bm == 256)
      hipLaunchKernelGGL((gate_gemm_dma_kernel<4, PL>), dim3(sh.mt, sh.nt, sh.ks), dim3(512), lds, st, x, planes, T,
                         H, N, sh.k_chunk, partial, zero0, zero1, n_zero);
    else
      hipLaunchKernelGGL((gate_gemm_dma_kernel<2, PL>), dim3(sh.mt, sh.nt, sh.ks), dim3(512), lds, st, x, planes, T,
                         H, N, sh.k_chunk, partial, zero0, zero1, n_zero);
  } else {
    hipLaunchKernelGGL(gate_gemm_kernel<PL>, dim3(sh.mt, sh.nt, sh.ks), dim3(256), 0, st, x, planes, T, H, N,
                       sh.k_chunk, partial, zero0, zero1, n_zero);
  }
}

// Workspace of a call: gate planes | logit partials (+ one plane for the residual) | u partials
struct RouteLayout {
  RouteShape gate, resid, resid2;  // gate GEMM; u = W1_hat h; r = W2_hat silu(u)
  size_t partial_bytes, upartial_bytes, a_bytes, b_bytes, total;
};

static RouteLayout route_layout(int T, int H, int E, int D, bool packed = false) {
  RouteLayout L;
  L.gate = route_shape(T, H, E);
  if (packed) L.gate.planes_bytes = 0;  // the caller holds the planes (probe_pack_gate)
  const size_t plane = static_cast<size_t>(T > 0 ? T : 1) * E * sizeof(float);
  L.upartial_bytes = L.a_bytes = L.b_bytes = 0;
  int extra = 0;
  if (D > 0) {
    L.resid = route_shape(T, H, D);
    L.resid2 = route_shape(T, 3 * D, E, 4);  // few slices: the softmax kernel reads every one of them
    L.upartial_bytes = L.resid.partial_bytes;
    L.a_bytes = align_up(static_cast<size_t>(T > 0 ? T : 1) * 3 * D * sizeof(bf16_t), 256);
    L.b_bytes = L.resid2.planes_bytes;
    extra = L.resid2.ks;
  }
  L.partial_bytes = align_up((L.gate.ks + extra) * plane, 256);
  L.total = L.gate.planes_bytes + L.partial_bytes + L.upartial_bytes + L.a_bytes + L.b_bytes;
  return L;
}

// Router (w1_hat == nullptr) or predictor with the residual MLP of Eq. 7 (w1_hat bf16 [D,H],
// w2_hat fp32 [E,D]).
static int route_impl(const char* name, const void* x_bf16, const float* w_gate, const float* bias,
                      int bias_groups, int tokens_per_group, const void* w1_hat, const float* w2_hat, int D,
                      int T, int H, int E, int k, int renormalize, int32_t* topk_idx, float* topk_w,
                      float* probs, int32_t* expert_counts, void* workspace, size_t workspace_bytes,
                      void* stream, const probe_gating* gating = nullptr, const float* select_bias = nullptr,
                      const void* packed = nullptr) {
  // w_gate (fp32, split into planes inside the call) or packed (planes made once by probe_pack_gate)
  PROBE_REQUIRE(T >= 0 && H > 0 && E > 0 && k > 0 && k <= E, PROBE_EINVAL,
                "%s: bad dims T=%d H=%d E=%d k=%d", name, T, H, E, k);
  PROBE_REQUIRE(bias == nullptr || (bias_groups >= 1 && tokens_per_group >= 1), PROBE_EINVAL,
                "%s: bias_groups=%d tokens_per_group=%d", name, bias_groups, tokens_per_group);
  PROBE_REQUIRE(E <= PROBE_MAX_EXPERTS && k <= PROBE_MAX_TOPK && H % 8 == 0, PROBE_EUNSUPPORTED,
                "%s: needs E <= %d, k <= %d, H %% 8 == 0 (E=%d k=%d H=%d)", name, PROBE_MAX_EXPERTS,
                PROBE_MAX_TOPK, E, k, H);
  if (gating) {
    const probe_gating& g = *gating;
    PROBE_REQUIRE(g.scoring == PROBE_SCORE_SOFTMAX || g.scoring == PROBE_SCORE_SIGMOID, PROBE_EINVAL,
                  "%s: scoring=%d", name, g.scoring);
    PROBE_REQUIRE(g.n_group >= 1 && E % g.n_group == 0 && g.topk_group >= 1 && g.topk_group <= g.n_group,
                  PROBE_EINVAL, "%s: n_group=%d must divide E=%d, topk_group=%d must be in 1..n_group", name,
                  g.n_group, E, g.topk_group);
    PROBE_REQUIRE(g.group_top >= 1 && g.group_top <= E / g.n_group && k <= g.topk_group * (E / g.n_group),
                  PROBE_EINVAL, "%s: group_top=%d and k=%d must fit %d groups of %d experts", name, g.group_top, k,
                  g.topk_group, E / g.n_group);
    PROBE_REQUIRE(g.n_group <= PROBE_MAX_GROUPS, PROBE_EUNSUPPORTED, "%s: needs n_group <= %d (n_group=%d)", name,
                  PROBE_MAX_GROUPS, g.n_group);
    PROBE_REQUIRE(aligned16(select_bias), PROBE_EALIGN, "%s: select_bias must be 16-byte aligned", name);
  }
  PROBE_REQUIRE(w_gate != nullptr || packed != nullptr, PROBE_EINVAL, "%s: the gate is NULL", name);
  PROBE_REQUIRE(T == 0 || (x_bf16 && topk_idx && topk_w), PROBE_EINVAL, "%s: null pointer", name);
  PROBE_REQUIRE(aligned16(x_bf16) && aligned16(w_gate) && aligned16(packed), PROBE_EALIGN,
                "%s: x and the gate must be 16-byte aligned", name);
  PROBE_REQUIRE(aligned16(bias) && aligned16(probs), PROBE_EALIGN,
                "%s: bias and probs must be 16-byte aligned", name);
  const bool resid = D > 0;
  if (resid) {
    PROBE_REQUIRE(w1_hat && w2_hat, PROBE_EINVAL, "%s: residual weights are NULL", name);
    PROBE_REQUIRE(D % 8 == 0 && D <= PROBE_MAX_RESIDUAL_WIDTH, PROBE_EUNSUPPORTED,
                  "%s: needs D %% 8 == 0 and D <= %d (D=%d)", name, PROBE_MAX_RESIDUAL_WIDTH, D);
    PROBE_REQUIRE(aligned16(w1_hat) && aligned16(w2_hat), PROBE_EALIGN,
                  "%s: w1_hat and w2_hat must be 16-byte aligned", name);
  }
  RouteLayout L = route_layout(T, H, E, resid ? D : 0, packed != nullptr);
  const RouteShape& sh = L.gate;
  PROBE_REQUIRE(workspace && aligned16(workspace) && workspace_bytes >= L.total, PROBE_EWORKSPACE,
                "%s: workspace too small or misaligned (%zu < %zu)", name, workspace_bytes, L.total);
  if (T > 0 && (sh.dma || (resid && (L.resid.dma || L.resid2.dma)))) {
    int rc = gate_prepare();
    if (rc != PROBE_OK) return rc;
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  const bf16_t* x = static_cast<const bf16_t*>(x_bf16);
  const bf16_t* planes = static_cast<const bf16_t*>(packed);
  float* partial = reinterpret_cast<float*>(static_cast<char*>(workspace) + sh.planes_bytes);
  float* upartial = reinterpret_cast<float*>(static_cast<char*>(workspace) + sh.planes_bytes + L.partial_bytes);
  const long n = static_cast<long>(E) * H;
  if (T == 0) {  // nothing to route: only the counts are cleared
    if (expert_counts)
      hipLaunchKernelGGL(gate_split_kernel, dim3((E + 255) / 256), dim3(256), 0, st, w_gate, 0l, nullptr, 0l,
                         expert_counts, E);
  } else if (packed == nullptr) {
    bf16_t* ws_planes = static_cast<bf16_t*>(workspace);
    hipLaunchKernelGGL(gate_split_kernel, dim3(static_cast<unsigned>((n + 255) / 256)), dim3(256), 0, st, w_gate, n,
                       ws_planes, n, nullptr, E);
    planes = ws_planes;
  }
  if (T > 0) {
    launch_gate_gemm<3>(sh, st, x, planes, T, H, E, partial, expert_counts, nullptr, expert_counts ? E : 0);
    int planes_to_sum = sh.ks;
    if (resid) {
      // u = W1_hat h (one bf16 plane); s = silu(u) and W2_hat split into planes; r = W2_hat s as
      // further slices of the logits
      char* base = static_cast<char*>(workspace) + sh.planes_bytes + L.partial_bytes + L.upartial_bytes;
      bf16_t* a_planes = reinterpret_cast<bf16_t*>(base);
      bf16_t* b_planes = reinterpret_cast<bf16_t*>(base + L.a_bytes);
      launch_gate_gemm<1>(L.resid, st, x, static_cast<const bf16_t*>(w1_hat), T, H, D, upartial);
      const long n_a = static_cast<long>(T) * (D / 8), n_b = static_cast<long>(E) * D;
      hipLaunchKernelGGL(resid_silu_split_kernel, dim3(static_cast<unsigned>((n_a + 255) / 256)), dim3(256), 0, st,
                         upartial, L.resid.ks, T, D, a_planes);
      hipLaunchKernelGGL(resid_w2_split_kernel, dim3(static_cast<unsigned>((n_b + 255) / 256)), dim3(256), 0, st,
                         w2_hat, E, D, b_planes);
      launch_gate_gemm<3>(L.resid2, st, a_planes, b_planes, T, 3 * D, E, partial + static_cast<size_t>(sh.ks) * T * E);
      planes_to_sum = sh.ks + L.resid2.ks;
    }
    int grid = (T + 31) / 32;
    if (grid > 4096) grid = 4096;
    int G = bias ? bias_groups : 1, tpg = bias ? tokens_per_group : 1;
#define PROBE_TOPK_LAUNCH(V)                                                                               \
  hipLaunchKernelGGL(gate_softmax_topk_kernel<V>, dim3(grid), dim3(256), 0, st, partial, E, planes_to_sum, bias, \
                     G, tpg, T, E, k, renormalize ? 1 : 0, topk_idx, topk_w, probs, expert_counts)
#define PROBE_GROUPED_LAUNCH(V)                                                                              \
  hipLaunchKernelGGL(gate_grouped_topk_kernel<V>, dim3(grid), dim3(256), 0, st, partial, E, planes_to_sum, bias, \
                     G, tpg, select_bias, T, E, k, gating->scoring, gating->n_group, gating->topk_group,         \
                     gating->group_top, gating->renormalize ? 1 : 0, gating->routed_scale, topk_idx, topk_w,     \
                     probs, expert_counts)
    if (gating) {
      if (E <= 64) {
        PROBE_GROUPED_LAUNCH(1);
      } else if (E <= 128) {
        PROBE_GROUPED_LAUNCH(2);
      } else {
        PROBE_GROUPED_LAUNCH(4);
      }
    } else if (E <= 64) {
      PROBE_TOPK_LAUNCH(1);
    } else {
      // small batches (decode): one token per row in flight and all split-K slices loaded at once give twice
      // the waves per SIMD to hide the loads behind; large batches are bound by reading the partial sums
      // either way (measured at 8192 and 16384 tokens: no difference)
#define PROBE_TOPK_LAUNCH_SMALL(V)                                                                              \
  hipLaunchKernelGGL((gate_softmax_topk_kernel<V, 1, 4>), dim3((T + 15) / 16), dim3(256), 0, st, partial, E,     \
                     planes_to_sum, bias, G, tpg, T, E, k, renormalize ? 1 : 0, topk_idx, topk_w, probs,        \
                     expert_counts)
      const bool small = T <= 2048;
      if (E <= 128) {
        if (small) PROBE_TOPK_LAUNCH_SMALL(2); else PROBE_TOPK_LAUNCH(2);
      } else {
        if (small) PROBE_TOPK_LAUNCH_SMALL(4); else PROBE_TOPK_LAUNCH(4);
      }
#undef PROBE_TOPK_LAUNCH_SMALL
    }
#undef PROBE_TOPK_LAUNCH
#undef PROBE_GROUPED_LAUNCH
  }
  return check_launch(name);
}

// Router of layer L-1 and zero-residual predictor of layer L on the same hidden states in one pass:
// the two gates are stacked into one operand of 2E rows per plane, one GEMM produces both sets of
// logits (x is read once, half as many split-K slices), the softmax / top-k kernel runs once per
// gate on its half of the columns.
static int route_predict_impl(const void* x_bf16, const float* w_gate, const float* bias,
                              const float* w_gate_next, const float* bias_next, int bias_groups,
                              int tokens_per_group, int T, int H, int E, int k, int renormalize,
                              int32_t* topk_idx, float* topk_w, float* probs, int32_t* expert_counts,
                              int32_t* pred_idx, float* pred_w, float* pred_probs, int32_t* pred_counts,
                              void* workspace, size_t workspace_bytes, void* stream,
                              const void* packed_stack = nullptr) {
  // (w_gate, w_gate_next) in fp32, or packed_stack: both gates packed into one stack of 2E rows
  const char* name = packed_stack ? "probe_route_predict_topk_packed" : "probe_route_predict_topk";
  PROBE_REQUIRE(T >= 0 && H > 0 && E > 0 && k > 0 && k <= E, PROBE_EINVAL,
                "%s: bad dims T=%d H=%d E=%d k=%d", name, T, H, E, k);
  PROBE_REQUIRE((bias == nullptr && bias_next == nullptr) || (bias_groups >= 1 && tokens_per_group >= 1),
                PROBE_EINVAL, "%s: bias_groups=%d tokens_per_group=%d", name, bias_groups, tokens_per_group);
  PROBE_REQUIRE(E <= PROBE_MAX_EXPERTS && k <= PROBE_MAX_TOPK && H % 8 == 0, PROBE_EUNSUPPORTED,
                "%s: needs E <= %d, k <= %d, H %% 8 == 0 (E=%d k=%d H=%d)", name, PROBE_MAX_EXPERTS,
                PROBE_MAX_TOPK, E, k, H);
  PROBE_REQUIRE(packed_stack != nullptr || (w_gate != nullptr && w_gate_next != nullptr), PROBE_EINVAL,
                "%s: a gate is NULL", name);
  PROBE_REQUIRE(T == 0 || (x_bf16 && topk_idx && topk_w && pred_idx && pred_w), PROBE_EINVAL,
                "%s: null pointer", name);
  PROBE_REQUIRE(aligned16(x_bf16) && aligned16(w_gate) && aligned16(w_gate_next) && aligned16(packed_stack),
                PROBE_EALIGN, "%s: x and the gates must be 16-byte aligned", name);
  PROBE_REQUIRE(aligned16(bias) && aligned16(bias_next) && aligned16(probs) && aligned16(pred_probs), PROBE_EALIGN,
                "%s: biases and probability outputs must be 16-byte aligned", name);
  RouteLayout L = route_layout(T, H, 2 * E, 0, packed_stack != nullptr);
  const RouteShape& sh = L.gate;
  PROBE_REQUIRE(workspace && aligned16(workspace) && workspace_bytes >= L.total, PROBE_EWORKSPACE,
                "%s: workspace too small or misaligned (%zu < %zu)", name, workspace_bytes, L.total);
  if (T > 0 && sh.dma) {
    int rc = gate_prepare();
    if (rc != PROBE_OK) return rc;
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  // planes [3][2E][H]: rows 0..E-1 this layer's gate, E..2E-1 the next
  const bf16_t* planes = static_cast<const bf16_t*>(packed_stack);
  float* partial = reinterpret_cast<float*>(static_cast<char*>(workspace) + sh.planes_bytes);
  const long n = static_cast<long>(E) * H;
  if (T == 0) {  // nothing to route: only the counts are cleared
    if (expert_counts)
      hipLaunchKernelGGL(gate_split_kernel, dim3((E + 255) / 256), dim3(256), 0, st, w_gate, 0l, nullptr, 0l,
                         expert_counts, E);
    if (pred_counts)
      hipLaunchKernelGGL(gate_split_kernel, dim3((E + 255) / 256), dim3(256), 0, st, w_gate, 0l, nullptr, 0l,
                         pred_counts, E);
  } else if (packed_stack == nullptr) {
    bf16_t* ws_planes = static_cast<bf16_t*>(workspace);
    const unsigned split_grid = static_cast<unsigned>((n + 255) / 256);
    hipLaunchKernelGGL(gate_split_kernel, dim3(split_grid), dim3(256), 0, st, w_gate, n, ws_planes, 2 * n, nullptr, E);
    hipLaunchKernelGGL(gate_split_kernel, dim3(split_grid), dim3(256), 0, st, w_gate_next, n, ws_planes + n, 2 * n,
                       nullptr, E);
    planes = ws_planes;
  }
  if (T > 0) {
    launch_gate_gemm<3>(sh, st, static_cast<const bf16_t*>(x_bf16), planes, T, H, 2 * E, partial, expert_counts,
                        pred_counts, E);
    int grid = (T + 31) / 32;
    if (grid > 4096) grid = 4096;
    const int G1 = bias ? bias_groups : 1, tpg1 = bias ? tokens_per_group : 1;
    const int G2 = bias_next ? bias_groups : 1, tpg2 = bias_next ? tokens_per_group : 1;
    const int rn = renormalize ? 1 : 0;
#define PROBE_TOPK_LAUNCH2(V)                                                                                     \
  do {                                                                                                            \
    hipLaunchKernelGGL(gate_softmax_topk_kernel<V>, dim3(grid), dim3(256), 0, st, partial, 2 * E, sh.ks, bias, G1, \
                       tpg1, T, E, k, rn, topk_idx, topk_w, probs, expert_counts);                                \
    hipLaunchKernelGGL(gate_softmax_topk_kernel<V>, dim3(grid), dim3(256), 0, st, partial + E, 2 * E, sh.ks,      \
                       bias_next, G2, tpg2, T, E, k, rn, pred_idx, pred_w, pred_probs, pred_counts);              \
  } while (0)
    if (E <= 64) {
      PROBE_TOPK_LAUNCH2(1);
    } else if (E <= 128) {
      PROBE_TOPK_LAUNCH2(2);
    } else {
      PROBE_TOPK_LAUNCH2(4);
    }
#undef PROBE_TOPK_LAUNCH2
  }
  return check_launch(name);
}

}  // namespace probe

extern "C" size_t probe_route_topk_workspace_bytes(int T, int H, int E, int k) {
  (void)k;
  if (T < 0 || H <= 0 || E <= 0) return 0;
  return probe::route_layout(T, H, E, 0).total;
}

extern "C" size_t probe_predict_topk_workspace_bytes(int T, int H, int E, int k) {
  return probe_route_topk_workspace_bytes(T, H, E, k);
}

extern "C" size_t probe_predict_topk_residual_workspace_bytes(int T, int H, int E, int k, int D) {
  (void)k;
  if (T < 0 || H <= 0 || E <= 0 || D <= 0) return 0;
  return probe::route_layout(T, H, E, D).total;
}

extern "C" int probe_route_topk(const void* x_bf16, const float* w_gate, const float* bias,
                                int bias_groups, int tokens_per_group, int T, int H, int E, int k,
                                int renormalize, int32_t* topk_idx, float* topk_w, float* probs,
                                int32_t* expert_counts, void* workspace, size_t workspace_bytes,
                                void* stream) {
  return probe::route_impl("probe_route_topk", x_bf16, w_gate, bias, bias_groups, tokens_per_group, nullptr,
                           nullptr, 0, T, H, E, k, renormalize, topk_idx, topk_w, probs, expert_counts,
                           workspace, workspace_bytes, stream);
}

extern "C" size_t probe_route_grouped_workspace_bytes(int T, int H, int E, int k) {
  return probe_route_topk_workspace_bytes(T, H, E, k);
}

// The router with a model's own gate: same GEMM, group-limited selection in place of the plain top-k.
extern "C" int probe_route_grouped(const void* x_bf16, const float* w_gate, const float* bias, int bias_groups,
                                   int tokens_per_group, const float* select_bias, const probe_gating* gating,
                                   int T, int H, int E, int k, int32_t* topk_idx, float* topk_w, float* scores,
                                   int32_t* expert_counts, void* workspace, size_t workspace_bytes,
                                   void* stream) {
  PROBE_REQUIRE(gating != nullptr, PROBE_EINVAL, "probe_route_grouped: gating is NULL");
  return probe::route_impl("probe_route_grouped", x_bf16, w_gate, bias, bias_groups, tokens_per_group, nullptr,
                           nullptr, 0, T, H, E, k, gating->renormalize, topk_idx, topk_w, scores, expert_counts,
                           workspace, workspace_bytes, stream, gating, select_bias);
}

// Eq. 7 with the residual at its zero initialisation is the cloned router applied to the
// previous layer's hidden states: the same kernels, fed with (h_{L-1}, W_L, b_L).
extern "C" int probe_predict_topk(const void* h_prev_bf16, const float* w_gate_next,
                                  const float* bias_next, int bias_groups, int tokens_per_group,
                                  int T, int H, int E, int k, int renormalize, int32_t* pred_idx,
                                  float* pred_w, float* probs, int32_t* pred_counts, void* workspace,
                                  size_t workspace_bytes, void* stream) {
  return probe::route_impl("probe_predict_topk", h_prev_bf16, w_gate_next, bias_next, bias_groups,
                           tokens_per_group, nullptr, nullptr, 0, T, H, E, k, renormalize, pred_idx, pred_w,
                           probs, pred_counts, workspace, workspace_bytes, stream);
}

// Eq. 7 in full: the frozen prior plus W2_hat silu(W1_hat h).
extern "C" int probe_predict_topk_residual(const void* h_prev_bf16, const float* w_gate_next,
                                           const float* bias_next, int bias_groups, int tokens_per_group,
                                           const void* w1_hat_bf16, const float* w2_hat, int D, int T, int H,
                                           int E, int k, int renormalize, int32_t* pred_idx, float* pred_w,
                                           float* probs, int32_t* pred_counts, void* workspace,
                                           size_t workspace_bytes, void* stream) {
  PROBE_REQUIRE(D > 0, PROBE_EINVAL, "probe_predict_topk_residual: D=%d", D);
  return probe::route_impl("probe_predict_topk_residual", h_prev_bf16, w_gate_next, bias_next, bias_groups,
                           tokens_per_group, w1_hat_bf16, w2_hat, D, T, H, E, k, renormalize, pred_idx, pred_w,
                           probs, pred_counts, workspace, workspace_bytes, stream);
}

extern "C" size_t probe_route_predict_topk_workspace_bytes(int T, int H, int E, int k) {
  (void)k;
  if (T < 0 || H <= 0 || E <= 0) return 0;
  return probe::route_layout(T, H, 2 * E, 0).total;
}

extern "C" int probe_route_predict_topk(const void* x_bf16, const float* w_gate, const float* bias,
                                        const float* w_gate_next, const float* bias_next, int bias_groups,
                                        int tokens_per_group, int T, int H, int E, int k, int renormalize,
                                        int32_t* topk_idx, float* topk_w, float* probs, int32_t* expert_counts,
                                        int32_t* pred_idx, float* pred_w, float* pred_probs,
                                        int32_t* pred_counts, void* workspace, size_t workspace_bytes,
                                        void* stream) {
  return probe::route_predict_impl(x_bf16, w_gate, bias, w_gate_next, bias_next, bias_groups, tokens_per_group, T,
                                   H, E, k, renormalize, topk_idx, topk_w, probs, expert_counts, pred_idx, pred_w,
                                   pred_probs, pred_counts, workspace, workspace_bytes, stream);
}

// ---- the gate packed once -------------------------------------------------------------------
// The router's (W_L, b_L) are frozen (Sec. 4.2), so the split of the fp32 gate into three bf16 planes
// need not be repeated on every call: probe_pack_gate writes the planes once, the *_packed entry points
// take them in place of the fp32 matrix.
extern "C" size_t probe_pack_gate_bytes(int H, int E_stack) {
  if (H <= 0 || E_stack <= 0) return 0;
  return probe::align_up(static_cast<size_t>(3) * E_stack * H * sizeof(probe::bf16_t), 256);
}

extern "C" int probe_pack_gate(const float* w_gate, int H, int E, int stack_rows, int row_offset,
                               void* packed, void* stream) {
  using namespace probe;
  PROBE_REQUIRE(H > 0 && E > 0 && stack_rows >= E && row_offset >= 0 && row_offset + E <= stack_rows, PROBE_EINVAL,
                "probe_pack_gate: bad dims H=%d E=%d stack_rows=%d row_offset=%d", H, E, stack_rows, row_offset);
  PROBE_REQUIRE(H % 8 == 0, PROBE_EUNSUPPORTED, "probe_pack_gate: needs H %% 8 == 0 (H=%d)", H);
  PROBE_REQUIRE(w_gate && packed, PROBE_EINVAL, "probe_pack_gate: null pointer");
  PROBE_REQUIRE(aligned16(w_gate) && aligned16(packed), PROBE_EALIGN,
                "probe_pack_gate: w_gate and packed must be 16-byte aligned");
  const long n = static_cast<long>(E) * H;
  hipLaunchKernelGGL(gate_split_kernel, dim3(static_cast<unsigned>((n + 255) / 256)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), w_gate, n,
                     static_cast<bf16_t*>(packed) + static_cast<long>(row_offset) * H,
                     static_cast<long>(stack_rows) * H, nullptr, E);
  return check_launch("probe_pack_gate");
}

extern "C" size_t probe_route_topk_packed_workspace_bytes(int T, int H, int E, int k) {
  (void)k;
  if (T < 0 || H <= 0 || E <= 0) return 0;
  return probe::route_layout(T, H, E, 0, true).total;
}

extern "C" int probe_route_topk_packed(const void* x_bf16, const void* packed_gate, const float* bias,
                                       int bias_groups, int tokens_per_group, int T, int H, int E, int k,
                                       int renormalize, int32_t* topk_idx, float* topk_w, float* probs,
                                       int32_t* expert_counts, void* workspace, size_t workspace_bytes,
                                       void* stream) {
  PROBE_REQUIRE(packed_gate != nullptr, PROBE_EINVAL, "probe_route_topk_packed: packed_gate is NULL");
  return probe::route_impl("probe_route_topk_packed", x_bf16, nullptr, bias, bias_groups, tokens_per_group, nullptr,
                           nullptr, 0, T, H, E, k, renormalize, topk_idx, topk_w, probs, expert_counts, workspace,
                           workspace_bytes, stream, nullptr, nullptr, packed_gate);
}

extern "C" int probe_predict_topk_packed(const void* h_prev_bf16, const void* packed_gate_next,
                                         const float* bias_next, int bias_groups, int tokens_per_group, int T,
                                         int H, int E, int k, int renormalize, int32_t* pred_idx, float* pred_w,
                                         float* probs, int32_t* pred_counts, void* workspace,
                                         size_t workspace_bytes, void* stream) {
  PROBE_REQUIRE(packed_gate_next != nullptr, PROBE_EINVAL, "probe_predict_topk_packed: packed_gate_next is NULL");
  return probe::route_impl("probe_predict_topk_packed", h_prev_bf16, nullptr, bias_next, bias_groups,
                           tokens_per_group, nullptr, nullptr, 0, T, H, E, k, renormalize, pred_idx, pred_w, probs,
                           pred_counts, workspace, workspace_bytes, stream, nullptr, nullptr, packed_gate_next);
}

extern "C" int probe_route_grouped_packed(const void* x_bf16, const void* packed_gate, const float* bias,
                                          int bias_groups, int tokens_per_group, const float* select_bias,
                                          const probe_gating* gating, int T, int H, int E, int k,
                                          int32_t* topk_idx, float* topk_w, float* scores,
                                          int32_t* expert_counts, void* workspace, size_t workspace_bytes,
                                          void* stream) {
  PROBE_REQUIRE(gating != nullptr, PROBE_EINVAL, "probe_route_grouped_packed: gating is NULL");
  PROBE_REQUIRE(packed_gate != nullptr, PROBE_EINVAL, "probe_route_grouped_packed: packed_gate is NULL");
  return probe::route_impl("probe_route_grouped_packed", x_bf16, nullptr, bias, bias_groups, tokens_per_group,
                           nullptr, nullptr, 0, T, H, E, k, gating->renormalize, topk_idx, topk_w, scores,
                           expert_counts, workspace, workspace_bytes, stream, gating, select_bias, packed_gate);
}

extern "C" size_t probe_route_predict_topk_packed_workspace_bytes(int T, int H, int E, int k) {
  (void)k;
  if (T < 0 || H <= 0 || E <= 0) return 0;
  return probe::route_layout(T, H, 2 * E, 0, true).total;
}

extern "C" int probe_route_predict_topk_packed(const void* x_bf16, const void* packed_stack, const float* bias,
                                               const float* bias_next, int bias_groups, int tokens_per_group,
                                               int T, int H, int E, int k, int renormalize, int32_t* topk_idx,
                                               float* topk_w, float* probs, int32_t* expert_counts,
                                               int32_t* pred_idx, float* pred_w, float* pred_probs,
                                               int32_t* pred_counts, void* workspace, size_t workspace_bytes,
                                               void* stream) {
  PROBE_REQUIRE(packed_stack != nullptr, PROBE_EINVAL, "probe_route_predict_topk_packed: packed_stack is NULL");
  return probe::route_predict_impl(x_bf16, nullptr, bias, nullptr, bias_next, bias_groups, tokens_per_group, T, H, E,
                                   k, renormalize, topk_idx, topk_w, probs, expert_counts, pred_idx, pred_w,
                                   pred_probs, pred_counts, workspace, workspace_bytes, stream, packed_stack);
}
