// Operand slices of the qgemm kernel, their loading and exact unpacking to scaled fp16 (see
// pq_qgemm.hip for why fp16 operands carry the per-group scales exactly).
#pragma once
#include "pq_device.h"
#include "pq_host.h"

namespace pq {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));

constexpr int kBK = 64;                 // K elements per step
constexpr int kRowBytes = kBK * 2 + 16; // fp16 row in LDS, padded by one 16-byte piece: with 144-byte
                                        // rows both the 16-byte fragment reads (rows 0..31 of a
                                        // piece) and the unpack writes spread over all banks

__device__ __forceinline__ half2_t as_h2(uint32_t u) { return __builtin_bit_cast(half2_t, u); }
__device__ __forceinline__ uint32_t h2_bits(half2_t h) { return __builtin_bit_cast(uint32_t, h); }

// ------------------------------------------------------------------------ operand unpack
// Per-thread slice of a tile row: 32 consecutive k (16 bytes of codes) plus its scales.
struct Slice {
  uint4 codes;
  uint32_t sc;      // NVFP4: two E4M3 bytes (k 0-15, 16-31); INT: one fp16 in the low half
};

// Where a quantized operand lives.  One description covers both layouts the kernel reads:
//   codes of (row, K step, half)  at codes  + row * code_row + step * code_step + half * 16
//   scale unit u of a row         at scales + row * sc_row   + u * sc_step          (2 bytes)
// where a scale unit is the pair of E4M3 bytes of 32 consecutive k (NVFP4, u = k / 32) or the
// fp16 normalised maximum of a group (INT, u = k / G).
//   row-major (as the quantizers store it): code_row = K / 2, code_step = 32;
//                                           sc_row = K / 16 (NVFP4) or 2 K / G, sc_step = 2
//   panel (K-step-major, see pq_pack.hip):  code_row = 32, code_step = 32 * rows;
//                                           sc_row = 2, sc_step = 2 * rows
// mul: per-row epilogue factor (stride 1) or a single factor (stride 0).
// bias: bf16 value per row of this operand added to the product in the epilogue (used for the
// weight operand, whose rows are the output columns), or null.
struct OperandView {
  const uint8_t* codes;
  int64_t code_row;
  int code_step;
  const uint8_t* scales;
  int64_t sc_row;
  int sc_step;
  const float* mul;
  int mul_stride;
  const uint16_t* bias = nullptr;
};

// Branch-free load of one slice.  `codes_row` / `sc_row` point at a valid row (the caller
// clamps the row index) and a k beyond K is redirected to the row start, so the address is
// always valid.  The loaded registers are not touched here (a use would make the wave wait for
// the load at once); a slice that is out of range is neutralised when it is unpacked, by
// zeroing its scale (see slice_scales).
template <int FMT, int G>
__device__ __forceinline__ Slice load_slice(const uint8_t* __restrict__ codes_row, int code_step,
                                            const uint8_t* __restrict__ sc_row, int sc_step, int K,
                                            int step, int half) {
  const int k0 = step * kBK + half * 32;
  const bool ok = k0 < K;
  const int unit = FMT == kNvfp4 ? k0 >> 5 : k0 / G;
  Slice s;
  s.codes = *reinterpret_cast<const uint4*>(codes_row + (ok ? (int64_t)step * code_step + half * 16 : 0));
  s.sc = *reinterpret_cast<const uint16_t*>(sc_row + (ok ? (int64_t)unit * sc_step : 0));
  return s;
}

// Scale pair(s) handed to unpack_pair.  INT carries {h, h} and {-24 h, -24 h} (see below).
struct PairScale {
  half2_t mul, add;
};

// {s, s} pairs of the two group scales a slice can touch; all zero when the slice is out of
// range (row beyond the matrix or k beyond K), so that whatever codes were loaded contribute 0
template <int FMT>
__device__ __forceinline__ void slice_scales(const Slice& s, bool ok, PairScale& p0, PairScale& p1) {
  if constexpr (FMT == kNvfp4) {
    // E4M3 byte b -> fp16: bits (b << 7) read as fp16 are value * 2^-8, subnormals included
    uint32_t two = ((s.sc & 0xFFu) << 7) | ((s.sc & 0xFF00u) << 15);
    two = ok ? two : 0u;
    half2_t v = as_h2(two) * (half2_t){(_Float16)256.0f, (_Float16)256.0f};
    p0.mul = (half2_t){v.x, v.x};
    p1.mul = (half2_t){v.y, v.y};
    p0.add = p1.add = (half2_t){(_Float16)0.0f, (_Float16)0.0f};
  } else {
    uint32_t b = (s.sc & 0xFFFFu) | (s.sc << 16);
    half2_t v = as_h2(ok ? b : 0u);
    p0.mul = p1.mul = v;
    p0.add = p1.add = v * (half2_t){(_Float16)-24.0f, (_Float16)-24.0f};   // exact: 2 + 8 bits
  }
}

// two codes of dword d (pair j of four: nibbles j and j + 4 for INT, byte j for NVFP4) -> two
// scaled fp16 values.  Which two elements form a pair only has to be the same for A and W.
//
// INT: the two's complement nibble z becomes offset binary u = z + 8 (flip bit 3), is placed
// at mantissa bits 6..9 of an fp16 with exponent field 0x4C00, which reads 16 + u = 24 + z, and
// one fused multiply-add forms (24 + z) * h - 24 * h = z * h.  The product has at most 13
// significant bits, 24 * h has 10, the result 11: every step is exact in the fma.
template <int FMT, int J>
__device__ __forceinline__ uint32_t unpack_pair(uint32_t d, const PairScale& sc) {
  if constexpr (FMT == kNvfp4) {
    return h2_bits(__builtin_amdgcn_cvt_scalef32_pk_f16_fp4(d, 1.0f, J) * sc.mul);
  } else {
    constexpr int SH = 4 * J - 6;                       // nibble J from bit 4J to bit 6
    const uint32_t x = SH < 0 ? (d << -SH) : (d >> SH);
    const half2_t t = as_h2((x & 0x03C003C0u) ^ 0x4E004E00u);   // exponent 0x4C00, bit 9 flipped
    return h2_bits(__builtin_elementwise_fma(t, sc.mul, sc.add));
  }
}

// tile row `r`, 16-byte piece `piece` (0..7) -> byte offset inside one LDS operand tile
__device__ __forceinline__ int lds_off(int r, int piece) { return r * kRowBytes + (piece << 4); }

template <int V>
struct IntC {
  static constexpr int value = V;
};

// view of an operand in the panel layout (pq_pack.hip)
inline OperandView panel_view(pq_format fmt, int group, const void* operand, int64_t rows, int64_t K,
                              const float* tensor_scale) {
  const OperandLayout L = operand_layout(fmt, group, rows, K);
  const uint8_t* o = (const uint8_t*)operand;
  OperandView v;
  v.codes = o + L.codes;
  v.code_row = 32;
  v.code_step = (int)(rows * 32);
  v.scales = o + L.scales;
  v.sc_row = 2;
  v.sc_step = (int)(rows * 2);
  if (fmt == PQ_FMT_NVFP4) {
    v.mul = tensor_scale;
    v.mul_stride = 0;
  } else {
    v.mul = (const float*)(o + L.mul);
    v.mul_stride = 1;
  }
  return v;
}

// the product kernel on two operand views (pq_qgemm.hip)
int launch_qgemm_views(pq_format fmt, int group, const OperandView& A, const OperandView& W, int64_t M,
                       int64_t N, int64_t K, void* y, int64_t ldy, bool out_f32, hipStream_t st);

}  // namespace pq
