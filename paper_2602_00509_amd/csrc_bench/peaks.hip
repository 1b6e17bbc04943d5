// Measurement aid of bench.py, built into its own library (libprobe_peaks.so) and not part of libprobe:
// an MFMA-only loop with its operands in registers.  bench.py times it to report what the matrix cores of
// the box sustain with no memory instruction in flight, for zero operands and for random bf16 operands
// (the chip is power-limited under matrix work and the operand bits decide how far).
//
//   double peaks_mfma_flops_per_launch(int workgroups, int iters)      flops of one launch (host arithmetic)
//   int    peaks_mfma(float* out, int workgroups, int iters, int random_operands, void* stream)
//          out: device, fp32 [workgroups * 512] (one checksum per thread; keeps the loop alive);
//          returns 0, -1 for bad arguments, -5 if the launch was rejected
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace peaks {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

__device__ __forceinline__ f32x16 mfma_32x32x16(u32x4 a, u32x4 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c,
                                                 0, 0, 0);
}

__device__ __forceinline__ uint32_t xorshift(uint32_t& s) {
  s ^= s << 13;
  s ^= s >> 17;
  s ^= s << 5;
  return s;
}

// two bf16 values with random sign and mantissa and one of four exponents (|v| in [1/8, 2))
__device__ __forceinline__ uint32_t random_bf16x2(uint32_t& s) {
  const uint32_t r = xorshift(s);
  const uint32_t e1 = 0x3c + ((r >> 8) & 3), e2 = 0x3c + ((r >> 24) & 3);
  return (r & 0x807f807fu) | (e1 << 7) | (e2 << 23);
}

// 8 waves per workgroup, each with a 4 x 2 grid of 32x32 accumulators as in the GEMM main loop.
__global__ __launch_bounds__(512, 2) void mfma_peak_kernel(float* __restrict__ out, int iters, int random) {
  uint32_t s = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
  u32x4 a[4], b[2];
  for (int i = 0; i < 4; ++i)
    for (int j = 0; j < 4; ++j) a[i][j] = random ? random_bf16x2(s) : 0u;
  for (int i = 0; i < 2; ++i)
    for (int j = 0; j < 4; ++j) b[i][j] = random ? random_bf16x2(s) : 0u;
  f32x16 acc[4][2];
  for (int i = 0; i < 4; ++i)
    for (int j = 0; j < 2; ++j)
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) acc[i][j] = mfma_32x32x16(a[i], b[j], acc[i][j]);
    if (random) a[it & 3][it & 3] ^= 0x00150015u;  // keep the operand bits moving
  }
  float sum = 0.f;
  for (int i = 0; i < 4; ++i)
    for (int j = 0; j < 2; ++j)
      for (int r = 0; r < 16; ++r) sum += acc[i][j][r];
  out[blockIdx.x * blockDim.x + threadIdx.x] = sum;
}

}  // namespace peaks

extern "C" double peaks_mfma_flops_per_launch(int workgroups, int iters) {
  // 8 waves x 8 MFMAs per iteration x 2 * 32 * 32 * 16 flops
  return static_cast<double>(workgroups) * 8.0 * iters * 8.0 * 32768.0;
}

extern "C" int peaks_mfma(float* out, int workgroups, int iters, int random_operands, void* stream) {
  if (out == nullptr || workgroups <= 0 || workgroups > 65536 || iters <= 0) return -1;
  hipLaunchKernelGGL(peaks::mfma_peak_kernel, dim3(workgroups), dim3(512), 0, static_cast<hipStream_t>(stream), out,
                     iters, random_operands);
  return hipGetLastError() == hipSuccess ? 0 : -5;
}
