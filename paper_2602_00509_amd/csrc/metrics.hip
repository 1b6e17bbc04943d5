// probe_predictor_metrics: how well the lookahead predictor forecasts the router (Sec. 4.2, Sec. 6.4).
// Evaluation only - never on the serving path.
//
//   hits = sum over tokens of |{pred_idx[t, 0..kp)} intersect {true_idx[t, 0..kt)}|
//       kp = kt = k        -> hits / (T k)      is the paper's top-k accuracy
//       kt = k / 2         -> hits / (T k / 2)  is its top-half-k hit rate (true_idx is ordered by logit)
//   ce   = sum over tokens of - sum_e true_probs[t,e] * log(pred_probs[t,e])
//       the cross-entropy that the online distillation of Sec. 4.2 minimises (reported, not trained)
//
// One workgroup, fixed summation order (a thread's tokens in ascending order, then a tree over the
// threads): the integer is exact and the fp64 sum is reproducible.
#include "common.hpp"

namespace probe {

__global__ __launch_bounds__(1024) void predictor_metrics_kernel(const int32_t* __restrict__ pred_idx,
                                                                 int pred_stride, int kp,
                                                                 const int32_t* __restrict__ true_idx,
                                                                 int true_stride, int kt, int T,
                                                                 const float* __restrict__ pred_probs,
                                                                 const float* __restrict__ true_probs, int E,
                                                                 long long* __restrict__ hits,
                                                                 double* __restrict__ ce_sum) {
  __shared__ long long s_hits[1024];
  __shared__ double s_ce[1024];
  const int tid = threadIdx.x;
  long long h = 0;
  double ce = 0.0;
  for (int t = tid; t < T; t += 1024) {
    const int32_t* p = pred_idx + static_cast<long>(t) * pred_stride;
    const int32_t* q = true_idx + static_cast<long>(t) * true_stride;
    for (int i = 0; i < kt; ++i) {
      const int e = q[i];
      bool found = false;
      for (int j = 0; j < kp; ++j) found |= (p[j] == e);
      h += found ? 1 : 0;
    }
    if (ce_sum) {
      const float* pp = pred_probs + static_cast<long>(t) * E;
      const float* tp = true_probs + static_cast<long>(t) * E;
      double acc = 0.0;
      for (int e = 0; e < E; ++e) {
        const float w = tp[e];
        if (w > 0.f) acc -= static_cast<double>(w) * log(static_cast<double>(pp[e]));
      }
      ce += acc;
    }
  }
  s_hits[tid] = h;
  s_ce[tid] = ce;
  __syncthreads();
  for (int d = 512; d > 0; d >>= 1) {
    if (tid < d) {
      s_hits[tid] += s_hits[tid + d];
      s_ce[tid] += s_ce[tid + d];
    }
    __syncthreads();
  }
  if (tid == 0) {
    hits[0] = s_hits[0];
    if (ce_sum) ce_sum[0] = s_ce[0];
  }
}

}  // namespace probe

extern "C" int probe_predictor_metrics(const int32_t* pred_idx, int pred_stride, int kp,
                                       const int32_t* true_idx, int true_stride, int kt, int T,
                                       const float* pred_probs, const float* true_probs, int E,
                                       int64_t* hits, double* cross_entropy_sum, void* stream) {
  using namespace probe;
  PROBE_REQUIRE(T >= 0 && kp >= 1 && kt >= 1 && pred_stride >= kp && true_stride >= kt, PROBE_EINVAL,
                "probe_predictor_metrics: bad dims T=%d kp=%d kt=%d strides %d %d", T, kp, kt, pred_stride,
                true_stride);
  PROBE_REQUIRE(hits != nullptr && (T == 0 || (pred_idx && true_idx)), PROBE_EINVAL,
                "probe_predictor_metrics: null pointer");
  PROBE_REQUIRE(cross_entropy_sum == nullptr || (E >= 1 && (T == 0 || (pred_probs && true_probs))), PROBE_EINVAL,
                "probe_predictor_metrics: the cross-entropy needs both probability tensors");
  hipLaunchKernelGGL(predictor_metrics_kernel, dim3(1), dim3(1024), 0, static_cast<hipStream_t>(stream), pred_idx,
                     pred_stride, kp, true_idx, true_stride, kt, T, pred_probs, true_probs, E,
                     reinterpret_cast<long long*>(hits), cross_entropy_sum);
  return check_launch("probe_predictor_metrics");
}
