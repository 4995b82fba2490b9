// Device-side helpers shared by the gfx950 kernels: bf16 widening, the pinned binary32
// quantizer arithmetic (Eq. 1-2 of the paper plus the NVFP4 two-level scales), E4M3 / E2M1
// rounding, and wavefront (64-lane) reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pq {

constexpr int kWave = 64;

enum Fmt : int { kNvfp4 = 0, kInt4 = 1, kInt3 = 2 };

__host__ __device__ constexpr float qmax_of(int fmt) { return fmt == kInt4 ? 7.0f : 3.0f; }

// ---------------------------------------------------------------- bit casts / bf16
__device__ __forceinline__ float as_f32(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t as_u32(float f) { return __builtin_bit_cast(uint32_t, f); }

// two bf16 packed in a dword -> the two floats (exact)
__device__ __forceinline__ float bf16_lo(uint32_t p) { return as_f32(p << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t p) { return as_f32(p & 0xFFFF0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return as_f32(uint32_t(b) << 16); }

// fp32 -> bf16 bits, round-to-nearest-even (finite inputs)
__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
  uint32_t u = as_u32(f);
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

__device__ __forceinline__ bool is_normal32(float v) {
  // v >= 0 finite: normal iff exponent field non-zero
  return (as_u32(v) & 0x7F800000u) != 0u && (as_u32(v) & 0x7F800000u) != 0x7F800000u;
}

// ---------------------------------------------------------------- E4M3 (scales, >= 0)
// round-to-nearest-even with saturation to 448 (byte 0x7E); t >= 0, may be +inf
__device__ __forceinline__ uint32_t e4m3_rne_sat(float t) {
  t = fminf(t, 448.0f);
  uint32_t r;
  if (t < 0.015625f) {                 // below the smallest normal 2^-6: fixed step 2^-9
    r = (uint32_t)(int)rintf(t * 512.0f);   // 0..8; 8 is the byte of 2^-6
  } else {
    uint32_t b = as_u32(t);
    b = b + 0x7FFFFu + ((b >> 20) & 1u);    // RNE to 3 mantissa bits
    r = (b >> 20) - ((127u - 7u) << 3);
  }
  return r;
}

__device__ __forceinline__ float e4m3_decode(uint32_t byte) {
  uint32_t e = (byte >> 3) & 0xFu, m = byte & 7u;
  if (e == 0) return float(m) * 0.001953125f;          // m * 2^-9
  return as_f32(((e + 120u) << 23) | (m << 20));       // 2^(e-7) * (1 + m/8)
}

// ---------------------------------------------------------------- E2M1 (element codes)
// index 0..7 of the nearest E2M1 magnitude, ties to the even index, saturating at 6; a >= 0.
// Adding 2^(e+22), e = exponent of max(a, 1), rounds a to a multiple of 2^(e-1) (one mantissa
// bit, fixed step 0.5 below 1) in the adder's nearest-even mode; the low bits of the sum then
// count those steps.
__device__ __forceinline__ uint32_t e2m1_rne_sat(float a) {
  a = fminf(a, 6.0f);
  uint32_t eb = as_u32(fmaxf(a, 1.0f)) & 0x7F800000u;       // (127 + e) << 23, e in {0,1,2}
  uint32_t mb = eb + (22u << 23);
  uint32_t steps = as_u32(a + as_f32(mb)) - mb;              // a / 2^(e-1), rounded
  return steps + (eb >> 22) - 254u;                          // + 2e
}

// ---------------------------------------------------------------- lane reductions
// max over aligned blocks of LANES consecutive lanes (LANES power of two <= 64)
template <int LANES>
__device__ __forceinline__ float group_max(float v) {
#pragma unroll
  for (int off = 1; off < LANES; off <<= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
  return v;
}

__device__ __forceinline__ float wave_max(float v) { return group_max<64>(v); }

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

// ---------------------------------------------------------------- quantizer steps
struct IntScale {
  float s, inv;
};
__device__ __forceinline__ IntScale int_scale(float amax, float Q) {
  IntScale r;
  r.s = amax / Q;
  r.inv = is_normal32(r.s) ? 1.0f / r.s : 0.0f;
  return r;
}
// 4-bit two's complement container of clip(rint(x * inv), -Q, Q)
__device__ __forceinline__ uint32_t int_code(float x, float inv, float Q) {
  float v = x * inv;
  v = fminf(fmaxf(v, -Q), Q);            // clipping before rounding is the same for integer Q
  return (uint32_t)(int)rintf(v) & 0xFu;
}

struct Nv4Scale {
  uint32_t byte;
  float inv;
};
__device__ __forceinline__ float nv4_enc_scale(float T) { return is_normal32(T) ? 1.0f / T : 0.0f; }
__device__ __forceinline__ Nv4Scale nv4_scale(float amax, float T, float encT) {
  Nv4Scale r;
  float t = (amax * encT) / 6.0f;
  r.byte = e4m3_rne_sat(t);
  float d = e4m3_decode(r.byte) * T;
  r.inv = is_normal32(d) ? 1.0f / d : 0.0f;
  return r;
}
__device__ __forceinline__ uint32_t nv4_code(float x, float inv) {
  float v = x * inv;
  return ((as_u32(x) >> 28) & 8u) | e2m1_rne_sat(fabsf(v));
}

}  // namespace pq
