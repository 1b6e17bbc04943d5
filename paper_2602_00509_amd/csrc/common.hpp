// Shared device/host helpers of libprobe (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "probe.h"

namespace probe {

typedef uint16_t bf16_t;  // raw bf16 bit pattern
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;  // one 16-byte chunk = 8 bf16

constexpr int kWave = 64;

// ---- host side ------------------------------------------------------------------------
void set_error(const char* fmt, ...);
int check_launch(const char* what);

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

#define PROBE_REQUIRE(cond, code, ...) \
  do {                                 \
    if (!(cond)) {                     \
      ::probe::set_error(__VA_ARGS__); \
      return (code);                   \
    }                                  \
  } while (0)

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- device side ----------------------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(bf16_t v) {
  return __uint_as_float(static_cast<uint32_t>(v) << 16);
}

// fp32 -> bf16, round to nearest, ties to even; NaN stays a quiet NaN.  gfx950 converts in
// hardware (v_cvt_pk_bf16_f32, two values per instruction); the compiler selects it for these casts.
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  return __builtin_bit_cast(bf16_t, static_cast<__bf16>(f));
}

// lo in bits 0..15, hi in bits 16..31
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

// D = A(32x16) * B(16x32) + C on the matrix cores.  Lane l supplies A[l%32][8*(l/32)..+8] and
// B[8*(l/32)..+8][l%32]; it receives D[(r/4)*8 + (l/32)*4 + r%4][l%32] in c[r], r = 0..15.
__device__ __forceinline__ f32x16 mfma_32x32x16(u32x4 a, u32x4 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                 __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// Row/column of accumulator register r of a 32x32 MFMA tile for this lane.
__device__ __forceinline__ int mfma32_row(int r, int lane) { return (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3); }
__device__ __forceinline__ int mfma32_col(int lane) { return lane & 31; }

// LDS tile of ROWS x 64 bf16 (128 bytes per row, eight 16-byte chunks).  Chunk c of row r is
// stored at chunk position c ^ (r & 7) so that eight consecutive rows reading the same
// logical chunk touch all 32 banks once.
__device__ __forceinline__ int lds_chunk_off(int row, int chunk) {
  return row * 8 + (chunk ^ (row & 7));  // in units of 16 bytes
}

}  // namespace probe
