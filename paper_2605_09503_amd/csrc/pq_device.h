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

// The same rounding without branches, with the rounded value itself: the step of the E4M3 grid at t
// is max(2^(e-3), 2^-9), e the exponent of t.  Adding M = max(2^(e+20), 2^14) makes that step the last
// place of the sum, so the adder rounds t onto the grid (nearest, ties to even); sum - M is the grid
// value, exactly, and the sum's mantissa field counts the steps: m in 8..16 of a normal result (16 is the
// next binade's first value -- the carry lands in the exponent field), or 0..8 steps of 2^-9 below 2^-6,
// which is the subnormal byte itself.  byte = m + 8 (e + 6) for normals, with (e + 6) = field(M) - 141.
__device__ __forceinline__ void e4m3_round(float t, uint32_t& byte, float& value) {
  t = fminf(t, 448.0f);
  const uint32_t eb = as_u32(t) & 0x7F800000u;
  const uint32_t mb = max(eb + (20u << 23), 141u << 23);       // bits of M; 2^14 has the exponent field 141
  const float sum = t + as_f32(mb);
  value = sum - as_f32(mb);
  byte = (as_u32(sum) - mb) + ((mb >> 20) - (141u << 3));
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
// value of the lane selected by a DPP control word (invalid source lanes read 0)
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
  return as_f32(dpp_u32<CTRL>(as_u32(v)));
}

// max over aligned blocks of LANES consecutive lanes (LANES power of two <= 64) of a
// non-negative, non-NaN value.  Such floats order like their bit patterns, so the maximum is an
// unsigned integer max, which takes the DPP lane exchange as an operand modifier (quad permutes,
// then mirrors inside 8 and 16 lanes: one instruction per step); wider groups finish with lane
// shuffles.
template <int LANES>
__device__ __forceinline__ float group_max(float v) {
  uint32_t u = as_u32(v);
  if constexpr (LANES >= 2) u = max(u, dpp_u32<0xB1>(u));    // quad_perm [1,0,3,2]
  if constexpr (LANES >= 4) u = max(u, dpp_u32<0x4E>(u));    // quad_perm [2,3,0,1]
  if constexpr (LANES >= 8) u = max(u, dpp_u32<0x141>(u));   // row_half_mirror
  if constexpr (LANES >= 16) u = max(u, dpp_u32<0x140>(u));  // row_mirror
#pragma unroll
  for (int off = 16; off < LANES; off <<= 1) u = max(u, (uint32_t)__shfl_xor((int)u, off, kWave));
  return as_f32(u);
}

__device__ __forceinline__ float wave_max(float v) { return group_max<64>(v); }

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

// ---------------------------------------------------------------- exact divisions, cheaply
// x / Q for a constant Q with c = RN(1 / Q): one multiply and two fused multiply-adds
// (quotient, exact remainder, correction).  Checked against IEEE division for every
// non-negative finite binary32 x: identical for Q = 3 and 7 everywhere, and for Q = 6 whenever
// the exponent field of x is at least 3.
__device__ __forceinline__ float div_const(float x, float Q, float c) {
  const float q0 = x * c;
  const float r = __builtin_fmaf(-Q, q0, x);
  return __builtin_fmaf(r, c, q0);
}

// 1 / s: hardware reciprocal plus one Newton step equals the IEEE quotient for every s whose
// exponent field lies in [3, 251] (checked exhaustively); outside that window (s >= 2^125; zero
// and subnormal s never get here) the whole wave takes the IEEE division.
__device__ __forceinline__ float recip_exact(float s, bool needed) {
  const bool fast = !needed || ((as_u32(s) >> 23) - 3u) <= 248u;
  if (__builtin_expect(__all(fast), 1)) {
    const float r = __builtin_amdgcn_rcpf(s);
    const float e = __builtin_fmaf(-s, r, 1.0f);
    return __builtin_fmaf(e, r, r);
  }
  return 1.0f / s;
}

// ---------------------------------------------------------------- quantizer steps
struct IntScale {
  float s, inv;
};
template <int FMT>
__device__ __forceinline__ IntScale int_scale(float amax) {
  constexpr float Q = qmax_of(FMT);
  IntScale r;
  r.s = div_const(amax, Q, 1.0f / Q);
  const bool normal = is_normal32(r.s);
  const float inv = recip_exact(r.s, normal);
  r.inv = normal ? inv : 0.0f;
  return r;
}
// the same for R independent maxima at once: one wave-wide window test for all of them
template <int FMT, int R>
__device__ __forceinline__ void int_scales(const float (&amax)[R], IntScale (&out)[R]) {
  constexpr float Q = qmax_of(FMT);
  bool normal[R];
  bool fast = true;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    out[r].s = div_const(amax[r], Q, 1.0f / Q);
    normal[r] = is_normal32(out[r].s);
    fast = fast && (!normal[r] || ((as_u32(out[r].s) >> 23) - 3u) <= 248u);
  }
  if (__builtin_expect(__all(fast), 1)) {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const float q = __builtin_amdgcn_rcpf(out[r].s);
      const float e = __builtin_fmaf(-out[r].s, q, 1.0f);
      out[r].inv = normal[r] ? __builtin_fmaf(e, q, q) : 0.0f;
    }
  } else {
#pragma unroll
    for (int r = 0; r < R; ++r) out[r].inv = normal[r] ? 1.0f / out[r].s : 0.0f;
  }
}
// Scales of four rows at once, for groups of LANES >= 4 lanes (a quad of lanes then lies inside one
// group).  a[r]: this lane's maximum over its own channels of row r.  The maxima are first combined
// across the quads of the group (mirror exchanges keep all four values per lane), then inside the
// quad by a transposing reduction: after two exchange steps lane l holds the group maximum of row
// l & 3 only.  Each lane derives the scale of its row -- a quarter of the arithmetic of doing all
// four in every lane -- and the quad broadcasts the four results.  Same values as int_scale.
template <int FMT, int LANES>
__device__ __forceinline__ void int_scales_rows4(const float (&a)[4], int lane, IntScale (&out)[4]) {
  static_assert(LANES >= 4, "a quad must lie inside a group");
  uint32_t u[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    u[r] = as_u32(a[r]);
    if constexpr (LANES >= 8) u[r] = max(u[r], dpp_u32<0x141>(u[r]));    // row_half_mirror
    if constexpr (LANES >= 16) u[r] = max(u[r], dpp_u32<0x140>(u[r]));   // row_mirror
#pragma unroll
    for (int off = 16; off < LANES; off <<= 1) u[r] = max(u[r], (uint32_t)__shfl_xor((int)u[r], off, kWave));
  }
  const bool odd = lane & 1, upper = lane & 2;
  uint32_t k01 = odd ? u[1] : u[0], g01 = odd ? u[0] : u[1];
  uint32_t k23 = odd ? u[3] : u[2], g23 = odd ? u[2] : u[3];
  k01 = max(k01, dpp_u32<0xB1>(g01));                                    // quad_perm [1,0,3,2]
  k23 = max(k23, dpp_u32<0xB1>(g23));
  uint32_t k = upper ? k23 : k01;
  const uint32_t g = upper ? k01 : k23;
  k = max(k, dpp_u32<0x4E>(g));                                          // quad_perm [2,3,0,1]
  const IntScale mine = int_scale<FMT>(as_f32(k));
  out[0].s = dpp_f32<0x00>(mine.s);                                      // quad_perm [r,r,r,r]
  out[1].s = dpp_f32<0x55>(mine.s);
  out[2].s = dpp_f32<0xAA>(mine.s);
  out[3].s = dpp_f32<0xFF>(mine.s);
  out[0].inv = dpp_f32<0x00>(mine.inv);
  out[1].inv = dpp_f32<0x55>(mine.inv);
  out[2].inv = dpp_f32<0xAA>(mine.inv);
  out[3].inv = dpp_f32<0xFF>(mine.inv);
}
// clip(rint(x * inv), -Q, Q) as a float: clipping first is the same for integer Q, and adding
// 1.5 * 2^23 rounds to the nearest integer (ties to even) in the adder; the low mantissa bits of
// the sum are then the two's complement integer.
__device__ __forceinline__ uint32_t int_code_bits(float x, float inv, float Q) {
  const float v = __builtin_amdgcn_fmed3f(x * inv, -Q, Q);
  return as_u32(v + 12582912.0f);
}
__device__ __forceinline__ uint32_t int_code(float x, float inv, float Q) {
  return int_code_bits(x, inv, Q) & 0xFu;
}
// Eight codes of one chunk, packed (element j at bits 4j, two's complement nibbles), for values
// whose group maximum produced `inv`: then |x * inv| <= Q (1 + 3 * 2^-24) < Q + 1/2, the rounding
// already lands inside [-Q, Q] and the clip is a no-op (inv = 0 gives 0).  Adding 1.5 * 2^23 + 8
// rounds to the nearest integer (ties to even) and leaves z + 8, in 1..15, in the low nibble under
// constant upper bits; the eight words are summed at nibble offsets (one shift-add each, carries
// into the discarded upper bits only), the constant part is subtracted once and bit 3 of every
// nibble flipped, which turns z + 8 into the two's complement of z.
__device__ __forceinline__ uint32_t int_codes8(const float (&x)[8], float inv) {
  constexpr uint32_t kBase = 0x4B400000u;                 // bits of 1.5 * 2^23
  constexpr uint32_t kConst = kBase * 0x11111111u;        // sum of kBase << 4j, modulo 2^32
  uint32_t acc = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) acc = (as_u32(x[j] * inv + 12582920.0f) << (4 * j)) + acc;
  return (acc - kConst) ^ 0x88888888u;
}
// Dense 3-bit storage of INT3 codes: code k of a row sits in bits 3k..3k+2 of the row's bit stream
// (z mod 8, least significant bit first), so eight codes -- one word of two's complement nibbles,
// element j at bits 4j -- make one 24-bit word.  The squeeze drops bit 3 of every nibble (for codes
// in -4..3 it repeats bit 2) and closes the gaps in three steps: nibble pairs to 6 bits per byte,
// byte pairs to 12 bits per half word, the two halves to 24 bits.  The spread is the inverse and
// restores bit 3 from bit 2.
__device__ __forceinline__ uint32_t int3_squeeze8(uint32_t nibbles) {
  const uint32_t a = (nibbles & 0x07070707u) | ((nibbles & 0x70707070u) >> 1);
  const uint32_t b = (a & 0x003F003Fu) | ((a & 0x3F003F00u) >> 2);
  return (b & 0x00000FFFu) | ((b & 0x0FFF0000u) >> 4);
}
__device__ __forceinline__ uint32_t int3_spread8(uint32_t w24) {
  const uint32_t b = (w24 & 0x00000FFFu) | ((w24 & 0x00FFF000u) << 4);
  const uint32_t a = (b & 0x003F003Fu) | ((b << 2) & 0x3F003F00u);
  const uint32_t n = (a & 0x07070707u) | ((a << 1) & 0x70707070u);
  return n | ((n & 0x44444444u) << 1);
}
// 32 codes: four nibble words <-> twelve bytes (three little-endian words)
__device__ __forceinline__ void int3_squeeze32(const uint4& n, uint32_t (&o)[3]) {
  const uint32_t w0 = int3_squeeze8(n.x), w1 = int3_squeeze8(n.y), w2 = int3_squeeze8(n.z), w3 = int3_squeeze8(n.w);
  o[0] = w0 | (w1 << 24);
  o[1] = (w1 >> 8) | (w2 << 16);
  o[2] = (w2 >> 16) | (w3 << 8);
}
__device__ __forceinline__ uint4 int3_spread32(uint32_t o0, uint32_t o1, uint32_t o2) {
  return make_uint4(int3_spread8(o0 & 0x00FFFFFFu), int3_spread8((o0 >> 24) | ((o1 & 0x0000FFFFu) << 8)),
                    int3_spread8((o1 >> 16) | ((o2 & 0x000000FFu) << 16)), int3_spread8(o2 >> 8));
}
// the same integer as a float (for the error evaluation)
__device__ __forceinline__ float int_code_value(float x, float inv, float Q) {
  const float v = __builtin_amdgcn_fmed3f(x * inv, -Q, Q);
  return (v + 12582912.0f) - 12582912.0f;
}

struct Nv4Scale {
  uint32_t byte;
  float inv;
  float d;       // decoded block scale times the tensor scale, rounded to binary32
  float value;   // decoded block scale (exact)
};
__device__ __forceinline__ float nv4_enc_scale(float T) { return is_normal32(T) ? 1.0f / T : 0.0f; }
// A tensor scale T with an exponent field in [13, 241] keeps every non-zero d = value(s_b) * T (values
// from 2^-9 to 448) a normal number with an exponent field in [4, 250], inside the window in which the
// hardware reciprocal plus one Newton step is the IEEE quotient: no per-group test is needed then.  T is
// the same for a whole launch, so the test is scalar and leaves the loops.
__device__ __forceinline__ bool nv4_tensor_scale_is_tame(float T) { return ((as_u32(T) >> 23) - 13u) <= 228u; }
__device__ __forceinline__ Nv4Scale nv4_scale(float amax, float T, float encT) {
  Nv4Scale r;
  // division by 6: the cheap sequence differs from IEEE only below 2^-124, far under the
  // smallest E4M3 value, where the byte is 0 either way
  const float t = div_const(amax * encT, 6.0f, 1.0f / 6.0f);
  e4m3_round(t, r.byte, r.value);
  const float value = r.value;
  r.d = value * T;
  if (__builtin_expect(nv4_tensor_scale_is_tame(T), 1)) {
    const float q = __builtin_amdgcn_rcpf(r.d);
    const float e = __builtin_fmaf(-r.d, q, 1.0f);
    r.inv = value != 0.0f ? __builtin_fmaf(e, q, q) : 0.0f;
  } else {
    const bool normal = is_normal32(r.d);
    const float inv = recip_exact(r.d, normal);
    r.inv = normal ? inv : 0.0f;
  }
  return r;
}
template <int R>
__device__ __forceinline__ void nv4_scales(const float (&amax)[R], float T, float encT, Nv4Scale (&out)[R]) {
#pragma unroll
  for (int r = 0; r < R; ++r) out[r] = nv4_scale(amax[r], T, encT);
}
__device__ __forceinline__ uint32_t nv4_code(float x, float inv) {
  float v = x * inv;
  return ((as_u32(x) >> 28) & 8u) | e2m1_rne_sat(fabsf(v));
}
// two elements at once on the conversion unit: byte = code(x1) << 4 | code(x0).  The
// instruction rounds to nearest even, saturates at +-6 and keeps the sign of a zero result
// (checked against nv4_code for all 2^32 inputs); the sign of x * inv is the sign of x.
__device__ __forceinline__ uint32_t nv4_code_pair(float x0, float x1, float inv) {
  return __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(0u, x0 * inv, x1 * inv, 1.0f, 0) & 0xFFu;
}

}  // namespace pq
