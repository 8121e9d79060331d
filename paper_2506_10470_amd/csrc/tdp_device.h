// Device-side helpers shared by the HIP kernels of the stage library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tdp {

typedef __bf16 bf16;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int kWave = 64;

// D(32x32) += A(32x16) * B(16x32).  Lane l supplies A[row = l%32][k = (l/32)*8 .. +8] and
// B[k = (l/32)*8 .. +8][col = l%32]; it receives D[row = (i/4)*8 + (l/32)*4 + i%4][col = l%32]
// in element i of the accumulator.
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
// D(16x16) += A(16x32) * B(32x16).  Lane l supplies A[row = l%16][k = (l/16)*8 .. +8] and
// B[k = (l/16)*8 .. +8][col = l%16]; it receives D[row = (l/16)*4 + i][col = l%16].
__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ bf16x8 ld_bf16x8(const bf16* p) {
  return *reinterpret_cast<const bf16x8*>(p);
}
__device__ __forceinline__ void st_bf16x8(bf16* p, bf16x8 v) {
  *reinterpret_cast<bf16x8*>(p) = v;
}
__device__ __forceinline__ bf16x8 zero_bf16x8() {
  bf16x8 z;
#pragma unroll
  for (int i = 0; i < 8; ++i) z[i] = (bf16)0.0f;
  return z;
}

// Offset of element (r, k) in an operand laid out as (r>>1)*pair + (k>>5)*kb + (r&1)*par + (k&31).
template <typename L>
__device__ __forceinline__ int64_t operand_offset(const L& lay, int r, int k) {
  return (int64_t)(r >> 1) * lay.pair + (int64_t)(k >> 5) * lay.kb + (int64_t)(r & 1) * lay.par + (k & 31);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

}  // namespace tdp
