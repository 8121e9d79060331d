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
// The same load marked non-temporal: for data a launch reads exactly once (a request's keys and values in
// decode), so that it does not displace what other workgroups share in L2.
__device__ __forceinline__ bf16x8 ld_bf16x8_nt(const bf16* p) {
  typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned u32x4_t;
  const u32x4_t raw = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return __builtin_bit_cast(bf16x8, raw);
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

// Offset of element (r, k) in an operand laid out as
// (r >> shift)*group + (k>>5)*kb + (r & (2^shift - 1))*par + (k&31).
template <typename L>
__device__ __forceinline__ int64_t operand_offset(const L& lay, int r, int k) {
  return (int64_t)(r >> lay.shift) * lay.group + (int64_t)(k >> 5) * lay.kb +
         (int64_t)(r & ((1 << lay.shift) - 1)) * lay.par + (k & 31);
}
// the row part of that offset alone
template <typename L>
__device__ __forceinline__ int64_t operand_row_offset(const L& lay, int r) {
  return (int64_t)(r >> lay.shift) * lay.group + (int64_t)(r & ((1 << lay.shift) - 1)) * lay.par;
}

// ---- 8-bit KV cache: OCP E4M3 (sign, 4 exponent bits with bias 7, 3 mantissa bits; exponent field
// 0 is subnormal, no infinities, S.1111.111 is NaN, largest finite magnitude 448) -------------------
// fp32 -> code: round to nearest, ties to the even code; magnitudes from 448 up (infinity included)
// saturate to +-448; NaN -> 0x7f | sign.  Integer arithmetic only, so the result does not depend on
// any conversion mode of the hardware.
__device__ __forceinline__ uint32_t f32_to_e4m3(float x) {
  const uint32_t u = __float_as_uint(x);
  const uint32_t sign = (u >> 24) & 0x80u;
  const uint32_t a = u & 0x7fffffffu;
  if (a > 0x7f800000u) return sign | 0x7fu;
  if (a >= 0x43e00000u) return sign | 0x7eu;                  // |x| >= 448
  if (a < 0x3c800000u)                                        // |x| < 2^-6: multiples of 2^-9
    return sign | (uint32_t)__float2int_rn(__uint_as_float(a) * 512.0f);  // 8 is the code of 2^-6 itself
  const uint32_t r = a + 0x7ffffu + ((a >> 20) & 1u);         // nearest even at mantissa bit 20
  return sign | ((r >> 20) - (120u << 3));                    // exponent bias 127 -> 7
}
// code -> fp32, exact (not used on the hot path, which converts with the hardware instruction)
__device__ __forceinline__ float e4m3_to_f32(uint32_t c) {
  const uint32_t sign = (c & 0x80u) << 24, e = (c >> 3) & 15u, m = c & 7u;
  if (e == 15u && m == 7u) return __uint_as_float(sign | 0x7fc00000u);
  if (e == 0u) return __uint_as_float(sign | __float_as_uint((float)m * 0.001953125f));
  return __uint_as_float(sign | ((e + 120u) << 23) | (m << 20));
}
// Four codes (one dword, lowest byte first) -> four bf16 as two dwords.  v_cvt_pk_f32_fp8 decodes
// E4M3 on gfx950; every E4M3 value is a bf16 value, so keeping the upper halves is exact.
__device__ __forceinline__ void e4m3x4_to_bf16x4(uint32_t w, uint32_t& lo, uint32_t& hi) {
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t a = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, false);
  const f32x2_t b = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, true);
  lo = __builtin_amdgcn_perm(__float_as_uint(a.y), __float_as_uint(a.x), 0x07060302u);
  hi = __builtin_amdgcn_perm(__float_as_uint(b.y), __float_as_uint(b.x), 0x07060302u);
}
// 16 codes -> the two MFMA operands they make (codes 0..7 and 8..15)
__device__ __forceinline__ void e4m3x16_to_bf16x8x2(uint4 raw, bf16x8& first, bf16x8& second) {
  union {
    uint32_t u[4];
    bf16x8 v;
  } f, g;
  e4m3x4_to_bf16x4(raw.x, f.u[0], f.u[1]);
  e4m3x4_to_bf16x4(raw.y, f.u[2], f.u[3]);
  e4m3x4_to_bf16x4(raw.z, g.u[0], g.u[1]);
  e4m3x4_to_bf16x4(raw.w, g.u[2], g.u[3]);
  first = f.v;
  second = g.v;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

}  // namespace tdp
