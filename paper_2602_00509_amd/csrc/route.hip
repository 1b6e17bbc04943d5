// probe_route_topk / probe_predict_topk: gate logits on the matrix cores, softmax, top-k.
//
// The gate is x[T,H] (bf16) times w_gate[E,H] (fp32).  At E = 128..256 this is far above the
// fp32 vector ridge of the chip, so the product runs on the bf16 MFMA units without giving up
// fp32 weights: every weight is split once per call into three bf16 planes hi + mid + lo
// (each the round-to-nearest bf16 of what the previous planes left over), which together
// carry all 24 significand bits.  x is bf16 already, every bf16 x bf16 product is exact in
// fp32, and the MFMA accumulates in fp32.
//
//   1. split    w_gate -> planes[3][E][H] bf16 in the workspace; zero the expert counts
//   2. gemm     split-K tiled GEMM (128 tokens x 128 experts x 64 k per step, 4 waves of
//               64x64, LDS-staged with register prefetch), three MFMAs per operand pair
//               (one per plane) into one accumulator               -> partial[KS][T][E] fp32
//   3. softmax  one wave per token: sum the KS partials in fixed order, add the bias, softmax
//               over E, k rounds of wave arg-max (ties to the lower index), weights, counts
#include <limits.h>

#include "common.hpp"

namespace probe {

constexpr int GBM = 128, GBN = 128, GBK = 64;

// ---- 1. split -------------------------------------------------------------------------
__global__ __launch_bounds__(256) void gate_split_kernel(const float* __restrict__ w, long n,
                                                         bf16_t* __restrict__ planes,
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
  planes[n + gid] = mid;
  planes[2 * n + gid] = lo;
}

// ---- 2. gemm --------------------------------------------------------------------------
__global__ __launch_bounds__(256, 2) void gate_gemm_kernel(const bf16_t* __restrict__ x,
                                                           const bf16_t* __restrict__ planes,
                                                           int T, int H, int E, int k_chunk,
                                                           float* __restrict__ partial) {
  __shared__ u32x4 sA[GBM * 8];
  __shared__ u32x4 sB[3][GBN * 8];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int wm = wv >> 1, wn = wv & 1;
  const int m0 = blockIdx.x * GBM, n0 = blockIdx.y * GBN, ks = blockIdx.z;
  const int kbeg = ks * k_chunk, kend = min(H, kbeg + k_chunk);
  const long plane_elems = static_cast<long>(E) * H;

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  u32x4 ra[4], rb[3][4];
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
      for (int p = 0; p < 3; ++p) {
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
      for (int p = 0; p < 3; ++p) sB[p][lds_chunk_off(row, c)] = rb[p][j];
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
      for (int p = 2; p >= 0; --p) {
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

// ---- 3. softmax + top-k ---------------------------------------------------------------
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// VPT = experts per lane (lane owns experts lane, lane+64, ...), E <= 64*VPT.
template <int VPT>
__global__ __launch_bounds__(256) void gate_softmax_topk_kernel(
    const float* __restrict__ partial, int KS, const float* __restrict__ bias, int G, int tpg, int T,
    int E, int k, int renorm, int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
    float* __restrict__ probs, int32_t* __restrict__ counts) {
  __shared__ int32_t hist[PROBE_MAX_EXPERTS];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  hist[tid] = 0;
  __syncthreads();
  const float ninf = -__builtin_inff();
  for (int t = blockIdx.x * 4 + wv; t < T; t += gridDim.x * 4) {
    int g = 0;
    if (bias) g = min(t / tpg, G - 1);
    float l[VPT], p[VPT];
    float mx = ninf;
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
      int e = lane + 64 * i;
      l[i] = ninf;
      if (e < E) {
        float s = 0.f;
        for (int q = 0; q < KS; ++q) s += partial[(static_cast<long>(q) * T + t) * E + e];
        if (bias) s += bias[static_cast<long>(g) * E + e];
        l[i] = s;
      }
      mx = fmaxf(mx, l[i]);
    }
    mx = wave_max(mx);
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
      p[i] = (lane + 64 * i < E) ? expf(l[i] - mx) : 0.f;
      sum += p[i];
    }
    sum = wave_sum(sum);
    const float inv = 1.f / sum;
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
      p[i] *= inv;
      if (probs && lane + 64 * i < E) probs[static_cast<long>(t) * E + lane + 64 * i] = p[i];
    }
    unsigned taken = 0;
    int isel = 0;
    float wsel = 0.f, wtot = 0.f;
    for (int s = 0; s < k; ++s) {
      float bv = ninf;
      int be = INT_MAX;
#pragma unroll
      for (int i = 0; i < VPT; ++i) {
        int e = lane + 64 * i;
        if (e < E && !((taken >> i) & 1u) && (be == INT_MAX || l[i] > bv)) {
          bv = l[i];
          be = e;
        }
      }
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) {
        float ov = __shfl_xor(bv, o, kWave);
        int oe = __shfl_xor(be, o, kWave);
        if (oe != INT_MAX && (be == INT_MAX || ov > bv || (ov == bv && oe < be))) {
          bv = ov;
          be = oe;
        }
      }
      float pv = 0.f;
#pragma unroll
      for (int i = 0; i < VPT; ++i)
        if (i == (be >> 6)) pv = p[i];
      float pw = __shfl(pv, be & 63, kWave);
      if (lane == (be & 63)) taken |= 1u << (be >> 6);
      wtot += pw;
      if (lane == s) {
        isel = be;
        wsel = pw;
      }
    }
    if (renorm) wsel /= wtot;
    if (lane < k) {
      topk_idx[static_cast<long>(t) * k + lane] = isel;
      topk_w[static_cast<long>(t) * k + lane] = wsel;
      if (counts) atomicAdd(&hist[isel], 1);
    }
  }
  __syncthreads();
  if (counts && tid < E && hist[tid] != 0) atomicAdd(&counts[tid], hist[tid]);
}

struct RouteShape {
  int mt, nt, ks, k_chunk;
  size_t planes_bytes, partial_bytes;
};

static RouteShape route_shape(int T, int H, int E) {
  RouteShape s;
  s.mt = (T + GBM - 1) / GBM;
  s.nt = (E + GBN - 1) / GBN;
  int tiles = s.mt * s.nt;
  int ksteps = (H + GBK - 1) / GBK;
  int want = tiles > 0 ? (512 + tiles - 1) / tiles : 1;
  if (want < 1) want = 1;
  if (want > ksteps) want = ksteps;
  int steps_per = (ksteps + want - 1) / want;
  s.k_chunk = steps_per * GBK;
  s.ks = (ksteps + steps_per - 1) / steps_per;
  s.planes_bytes = align_up(static_cast<size_t>(3) * E * H * sizeof(bf16_t), 256);
  s.partial_bytes = align_up(static_cast<size_t>(s.ks) * (T > 0 ? T : 1) * E * sizeof(float), 256);
  return s;
}

static int route_impl(const char* name, const void* x_bf16, const float* w_gate, const float* bias,
                      int bias_groups, int tokens_per_group, int T, int H, int E, int k,
                      int renormalize, int32_t* topk_idx, float* topk_w, float* probs,
                      int32_t* expert_counts, void* workspace, size_t workspace_bytes, void* stream) {
  PROBE_REQUIRE(T >= 0 && H > 0 && E > 0 && k > 0 && k <= E, PROBE_EINVAL,
                "%s: bad dims T=%d H=%d E=%d k=%d", name, T, H, E, k);
  PROBE_REQUIRE(bias == nullptr || (bias_groups >= 1 && tokens_per_group >= 1), PROBE_EINVAL,
                "%s: bias_groups=%d tokens_per_group=%d", name, bias_groups, tokens_per_group);
  PROBE_REQUIRE(E <= PROBE_MAX_EXPERTS && k <= PROBE_MAX_TOPK && H % 8 == 0, PROBE_EUNSUPPORTED,
                "%s: needs E <= %d, k <= %d, H %% 8 == 0 (E=%d k=%d H=%d)", name, PROBE_MAX_EXPERTS,
                PROBE_MAX_TOPK, E, k, H);
  PROBE_REQUIRE(w_gate != nullptr, PROBE_EINVAL, "%s: w_gate is NULL", name);
  PROBE_REQUIRE(T == 0 || (x_bf16 && topk_idx && topk_w), PROBE_EINVAL, "%s: null pointer", name);
  PROBE_REQUIRE(aligned16(x_bf16) && aligned16(w_gate), PROBE_EALIGN,
                "%s: x and w_gate must be 16-byte aligned", name);
  RouteShape sh = route_shape(T, H, E);
  PROBE_REQUIRE(workspace && aligned16(workspace) && workspace_bytes >= sh.planes_bytes + sh.partial_bytes,
                PROBE_EWORKSPACE, "%s: workspace too small or misaligned (%zu < %zu)", name,
                workspace_bytes, sh.planes_bytes + sh.partial_bytes);
  hipStream_t st = static_cast<hipStream_t>(stream);
  bf16_t* planes = static_cast<bf16_t*>(workspace);
  float* partial = reinterpret_cast<float*>(static_cast<char*>(workspace) + sh.planes_bytes);
  long n = static_cast<long>(E) * H;
  if (T == 0) n = 0;  // nothing to route: only the counts are cleared
  long split_threads = n > E ? n : E;
  hipLaunchKernelGGL(gate_split_kernel, dim3(static_cast<unsigned>((split_threads + 255) / 256)), dim3(256),
                     0, st, w_gate, n, planes, expert_counts, E);
  if (T > 0) {
    hipLaunchKernelGGL(gate_gemm_kernel, dim3(sh.mt, sh.nt, sh.ks), dim3(256), 0, st,
                       static_cast<const bf16_t*>(x_bf16), planes, T, H, E, sh.k_chunk, partial);
    int grid = (T + 3) / 4;
    if (grid > 2048) grid = 2048;
    int G = bias ? bias_groups : 1, tpg = bias ? tokens_per_group : 1;
#define PROBE_TOPK_LAUNCH(V)                                                                           \
  hipLaunchKernelGGL(gate_softmax_topk_kernel<V>, dim3(grid), dim3(256), 0, st, partial, sh.ks, bias, \
                     G, tpg, T, E, k, renormalize ? 1 : 0, topk_idx, topk_w, probs, expert_counts)
    if (E <= 64) {
      PROBE_TOPK_LAUNCH(1);
    } else if (E <= 128) {
      PROBE_TOPK_LAUNCH(2);
    } else {
      PROBE_TOPK_LAUNCH(4);
    }
#undef PROBE_TOPK_LAUNCH
  }
  return check_launch(name);
}

}  // namespace probe

extern "C" size_t probe_route_topk_workspace_bytes(int T, int H, int E, int k) {
  (void)k;
  if (T < 0 || H <= 0 || E <= 0) return 0;
  probe::RouteShape s = probe::route_shape(T, H, E);
  return s.planes_bytes + s.partial_bytes;
}

extern "C" size_t probe_predict_topk_workspace_bytes(int T, int H, int E, int k) {
  return probe_route_topk_workspace_bytes(T, H, E, k);
}

extern "C" int probe_route_topk(const void* x_bf16, const float* w_gate, const float* bias,
                                int bias_groups, int tokens_per_group, int T, int H, int E, int k,
                                int renormalize, int32_t* topk_idx, float* topk_w, float* probs,
                                int32_t* expert_counts, void* workspace, size_t workspace_bytes,
                                void* stream) {
  return probe::route_impl("probe_route_topk", x_bf16, w_gate, bias, bias_groups, tokens_per_group, T,
                           H, E, k, renormalize, topk_idx, topk_w, probs, expert_counts, workspace,
                           workspace_bytes, stream);
}

// Eq. 7 with the residual at its zero initialisation is the cloned router applied to the
// previous layer's hidden states: the same kernels, fed with (h_{L-1}, W_L, b_L).
extern "C" int probe_predict_topk(const void* h_prev_bf16, const float* w_gate_next,
                                  const float* bias_next, int bias_groups, int tokens_per_group,
                                  int T, int H, int E, int k, int renormalize, int32_t* pred_idx,
                                  float* pred_w, float* probs, int32_t* pred_counts, void* workspace,
                                  size_t workspace_bytes, void* stream) {
  return probe::route_impl("probe_predict_topk", h_prev_bf16, w_gate_next, bias_next, bias_groups,
                           tokens_per_group, T, H, E, k, renormalize, pred_idx, pred_w, probs,
                           pred_counts, workspace, workspace_bytes, stream);
}
