// probe_combine: out[t] = sum_s w[t,s] * y[pair_row[t,s]] (gather form, no atomics).
//
// HBM-bound streaming kernel.  One thread owns one 16-byte chunk (8 bf16) of one output row:
// it issues up to k independent 16-byte loads from the k source rows, accumulates in fp32 in
// ascending s and stores 16 bytes.  Adjacent threads own adjacent chunks, so every load and
// store instruction of a wave covers 1 KiB of contiguous memory.
// probe_combine_shared adds shared_scale * shared[t] (a shared expert's output, one more 16-byte
// load per thread) after the k routed terms.
#include "common.hpp"

namespace probe {

template <int K, bool SHARED>
__global__ __launch_bounds__(256) void combine_kernel(const u32x4* __restrict__ y,
                                                      const int32_t* __restrict__ pair_row,
                                                      const float* __restrict__ topk_w,
                                                      const u32x4* __restrict__ shared, float shared_scale,
                                                      long total_chunks, int chunks_per_row,
                                                      u32x4* __restrict__ out) {
  long gid = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (gid >= total_chunks) return;
  int t = static_cast<int>(gid / chunks_per_row);
  int c = static_cast<int>(gid - static_cast<long>(t) * chunks_per_row);
  int rows[K];
  float w[K];
#pragma unroll
  for (int s = 0; s < K; ++s) {
    rows[s] = pair_row[static_cast<long>(t) * K + s];
    w[s] = topk_w[static_cast<long>(t) * K + s];
  }
  u32x4 v[K];
#pragma unroll
  for (int s = 0; s < K; ++s) {
    v[s] = u32x4{0u, 0u, 0u, 0u};
    if (rows[s] >= 0) v[s] = __builtin_nontemporal_load(&y[static_cast<long>(rows[s]) * chunks_per_row + c]);
  }
  u32x4 sv = u32x4{0u, 0u, 0u, 0u};
  if constexpr (SHARED) sv = __builtin_nontemporal_load(&shared[gid]);
  float acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.f;
#pragma unroll
  for (int s = 0; s < K; ++s) {
    if (rows[s] >= 0) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        acc[2 * i] = fmaf(w[s], __uint_as_float(v[s][i] << 16), acc[2 * i]);
        acc[2 * i + 1] = fmaf(w[s], __uint_as_float(v[s][i] & 0xffff0000u), acc[2 * i + 1]);
      }
    }
  }
  if constexpr (SHARED) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      acc[2 * i] = fmaf(shared_scale, __uint_as_float(sv[i] << 16), acc[2 * i]);
      acc[2 * i + 1] = fmaf(shared_scale, __uint_as_float(sv[i] & 0xffff0000u), acc[2 * i + 1]);
    }
  }
  u32x4 o;
#pragma unroll
  for (int i = 0; i < 4; ++i) o[i] = pack_bf16x2(acc[2 * i], acc[2 * i + 1]);
  __builtin_nontemporal_store(o, &out[gid]);
}

}  // namespace probe

namespace probe {

static int combine_impl(const char* name, const void* y_bf16, const int32_t* pair_row, const float* topk_w,
                        const void* shared_bf16, bool with_shared, float shared_scale, int T, int H, int k,
                        void* out_bf16, void* stream) {
  PROBE_REQUIRE(T >= 0 && H > 0 && k > 0, PROBE_EINVAL, "%s: bad dims T=%d H=%d k=%d", name, T, H, k);
  PROBE_REQUIRE(k <= PROBE_MAX_TOPK && H % 8 == 0, PROBE_EUNSUPPORTED,
                "%s: needs k <= %d and H %% 8 == 0 (k=%d H=%d)", name, PROBE_MAX_TOPK, k, H);
  if (T == 0) return PROBE_OK;
  PROBE_REQUIRE(y_bf16 && pair_row && topk_w && out_bf16 && (!with_shared || shared_bf16), PROBE_EINVAL,
                "%s: null pointer", name);
  PROBE_REQUIRE(aligned16(y_bf16) && aligned16(out_bf16) && aligned16(shared_bf16), PROBE_EALIGN,
                "%s: y/shared/out must be 16-byte aligned", name);
  hipStream_t st = static_cast<hipStream_t>(stream);
  int cpr = H / 8;
  long total = static_cast<long>(T) * cpr;
  unsigned grid = static_cast<unsigned>((total + 255) / 256);
  const u32x4* y = static_cast<const u32x4*>(y_bf16);
  const u32x4* sh = static_cast<const u32x4*>(shared_bf16);
  u32x4* out = static_cast<u32x4*>(out_bf16);
#define PROBE_COMBINE_CASE(K)                                                                                  \
  case K:                                                                                                      \
    if (with_shared)                                                                                           \
      hipLaunchKernelGGL((combine_kernel<K, true>), dim3(grid), dim3(256), 0, st, y, pair_row, topk_w, sh,      \
                         shared_scale, total, cpr, out);                                                       \
    else                                                                                                       \
      hipLaunchKernelGGL((combine_kernel<K, false>), dim3(grid), dim3(256), 0, st, y, pair_row, topk_w, sh,     \
                         0.f, total, cpr, out);                                                                \
    break;
  switch (k) {
    PROBE_COMBINE_CASE(1) PROBE_COMBINE_CASE(2) PROBE_COMBINE_CASE(3) PROBE_COMBINE_CASE(4)
    PROBE_COMBINE_CASE(5) PROBE_COMBINE_CASE(6) PROBE_COMBINE_CASE(7) PROBE_COMBINE_CASE(8)
  }
#undef PROBE_COMBINE_CASE
  return check_launch(name);
}

}  // namespace probe

extern "C" int probe_combine(const void* y_bf16, const int32_t* pair_row, const float* topk_w,
                             int T, int H, int k, void* out_bf16, void* stream) {
  return probe::combine_impl("probe_combine", y_bf16, pair_row, topk_w, nullptr, false, 0.f, T, H, k, out_bf16,
                             stream);
}

extern "C" int probe_combine_shared(const void* y_bf16, const int32_t* pair_row, const float* topk_w,
                                    const void* shared_y_bf16, float shared_scale, int T, int H, int k,
                                    void* out_bf16, void* stream) {
  return probe::combine_impl("probe_combine_shared", y_bf16, pair_row, topk_w, shared_y_bf16, true, shared_scale,
                             T, H, k, out_bf16, stream);
}
