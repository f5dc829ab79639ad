// Device-side building blocks shared by the gfx950 kernels: bf16 conversion,
// the Philox4x32-10 counter RNG and the 32-bit-word -> N(0,1) pair recipe that
// regenerates the perturbation z of Q-SPSA (paper Def. 3.3, Algorithm 1) from
// (seed, row, group) instead of storing it.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace qzo {

typedef unsigned short bf16_t;   // raw bf16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t b) {
  return __uint_as_float(((uint32_t)b) << 16);
}
// round-to-nearest-even; inputs are finite in every use here.
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
// A stored group scale (16 bits: bf16, or fp16 when the arena is fp16) as fp32.
__device__ __forceinline__ float scale_to_f32(uint32_t bits16, bool fp16) {
  return fp16 ? (float)__builtin_bit_cast(_Float16, (uint16_t)bits16) : __uint_as_float(bits16 << 16);
}
// fp32 -> the scale's storage type, round-to-nearest-even, as 16 bits.
__device__ __forceinline__ uint32_t f32_to_scale(float f, bool fp16);
// two floats -> packed pair of bf16 (lo in the low half).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
  typedef float f2 __attribute__((ext_vector_type(2)));
  f2 v = {lo, hi};
  bf2 r = __builtin_convertvector(v, bf2);   // v_cvt_pk_bf16_f32, RNE
  return __builtin_bit_cast(uint32_t, r);
}

// two floats -> packed pair in the scale's storage type.
__device__ __forceinline__ uint32_t pack_scale_x2(float lo, float hi, bool fp16) {
  if (fp16) {
    const _Float16 a = (_Float16)lo, b = (_Float16)hi;      // v_cvt_f16_f32, RNE
    return (uint32_t)__builtin_bit_cast(uint16_t, a) | ((uint32_t)__builtin_bit_cast(uint16_t, b) << 16);
  }
  return pack_bf16x2(lo, hi);
}
__device__ __forceinline__ uint32_t f32_to_scale(float f, bool fp16) { return pack_scale_x2(f, 0.0f, fp16) & 0xffffu; }

struct u32x4_t { uint32_t x, y, z, w; };

// Philox4x32 with 10 rounds (Salmon et al., SC'11).
__device__ __forceinline__ u32x4_t philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return {c0, c1, c2, c3};
}

// One 32-bit word -> two N(0,1) variates (Box-Muller):
//   bits 31..16 h: u1 = (2h+1)/2^17; bit 15 / 14: signs; bits 13..0 k:
//   first-quadrant angle (k+1/2)(pi/2)/2^14.
// Built only from exact integer/exponent steps and fp32 mul/add/fma so that
// any IEEE machine gives the same bits (the file is compiled with
// -ffp-contract=off; every fused step is an explicit fma).
// The radius sqrt(-ln u1) depends on h only and the two angle factors on k only; the variates are
// one IEEE product of the two each, so the factors may be computed apart (or looked up).
__device__ __forceinline__ float normal_radius(uint32_t w) {
  const float QL0 = 0x1.fffffap-1f, QL1 = 0x1.000586p-1f, QL2 = 0x1.53a4dcp-2f,
              QL3 = 0x1.18fbf0p-2f, QL4 = 0x1.a5d4cap-6f, QL5 = 0x1.a4912ap-1f,
              QL6 = -0x1.2245dap+0f, QL7 = 0x1.36ff60p+0f;
  const float LN2 = 0x1.62e430p-1f;
  // -ln(u1) = (17-E) ln2 + (1-m) Q(1-m), with 2h+1 = m 2^E, m in [1/2,1)
  float a = (float)((w >> 15) | 1u);
  float m = __builtin_amdgcn_frexp_mantf(a);
  int E = __builtin_amdgcn_frexp_expf(a);
  float f = 1.0f - m;
  float q = QL7;
  q = __builtin_fmaf(q, f, QL6); q = __builtin_fmaf(q, f, QL5); q = __builtin_fmaf(q, f, QL4);
  q = __builtin_fmaf(q, f, QL3); q = __builtin_fmaf(q, f, QL2); q = __builtin_fmaf(q, f, QL1);
  q = __builtin_fmaf(q, f, QL0);
  float fq = f * q;
  float t = __builtin_fmaf((float)(17 - E), LN2, fq);
  // sqrt(t) = t * rsqrt(t): integer seed + three Newton steps
  float y = __int_as_float(0x5f3759df - (__float_as_int(t) >> 1));
  float ht = 0.5f * t;
#pragma unroll
  for (int it = 0; it < 3; ++it) {
    float hy = ht * y;
    float c = __builtin_fmaf(-hy, y, 1.5f);
    y = y * c;
  }
  return t * y;
}
// k = 0 .. 16383 -> (cos x - sin x, cos x + sin x) = sqrt2 (cos phi, sin phi), x = phi - pi/4
__device__ __forceinline__ float2 normal_angle(uint32_t k) {
  const float ANG_STEP = 0x1.921fb6p-14f, ANG_OFF = -0x1.92196cp-1f;
  const float S0 = -0x1.555552p-3f, S1 = 0x1.110c2cp-7f, S2 = -0x1.9acab0p-13f;
  const float C0 = -0x1.000000p-1f, C1 = 0x1.55555ep-5f, C2 = -0x1.6c16a2p-10f,
              C3 = 0x1.9ca594p-16f;
  float x = __builtin_fmaf((float)k, ANG_STEP, ANG_OFF);
  float x2 = x * x;
  float sp = __builtin_fmaf(x2, S2, S1);
  sp = __builtin_fmaf(x2, sp, S0);
  float sx = __builtin_fmaf(x2 * sp, x, x);
  float cp = __builtin_fmaf(x2, C3, C2);
  cp = __builtin_fmaf(x2, cp, C1);
  cp = __builtin_fmaf(x2, cp, C0);
  float cx = __builtin_fmaf(x2, cp, 1.0f);
  return make_float2(cx - sx, cx + sx);
}
__device__ __forceinline__ void normal_from_factors(uint32_t w, float r, float2 cs, float& z0, float& z1) {
  float a0 = r * cs.x;
  float a1 = r * cs.y;
  z0 = __uint_as_float(__float_as_uint(a0) | ((w & 0x8000u) << 16));
  z1 = __uint_as_float(__float_as_uint(a1) | ((w & 0x4000u) << 17));
}
__device__ __forceinline__ void normal_pair(uint32_t w, float& z0, float& z1) {
  normal_from_factors(w, normal_radius(w), normal_angle(w & 0x3fffu), z0, z1);
}

// The eight variates z(row, 8*gblock .. 8*gblock+7) of one Philox counter.
__device__ __forceinline__ void scale_normals8(uint32_t seed_lo, uint32_t seed_hi, uint32_t stream,
                                               uint32_t row, uint32_t gblock, float z[8]) {
  u32x4_t w = philox4x32_10(row, gblock, stream, 0u, seed_lo, seed_hi);
  normal_pair(w.x, z[0], z[1]);
  normal_pair(w.y, z[2], z[3]);
  normal_pair(w.z, z[4], z[5]);
  normal_pair(w.w, z[6], z[7]);
}

// z for entry i of a flat vector (per-output-channel scales): counter (i/8, 0, stream, 0),
// word (i%8)/2, variate i%2.
__device__ __forceinline__ float flat_normal(uint32_t seed_lo, uint32_t seed_hi, uint32_t stream,
                                             uint32_t i) {
  const u32x4_t w = philox4x32_10(i >> 3, 0u, stream, 0u, seed_lo, seed_hi);
  const uint32_t p = (i & 7u) >> 1;
  const uint32_t word = p == 0 ? w.x : (p == 1 ? w.y : (p == 2 ? w.z : w.w));
  float z0, z1;
  normal_pair(word, z0, z1);
  return (i & 1u) ? z1 : z0;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

}  // namespace qzo
