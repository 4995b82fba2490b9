// Panel layout of a quantized operand for the GEMM, and the kernel that builds it from the
// row-major output of the quantizers.
//
// Why: the GEMM reads 64 k of every tile row per step, which is 32 bytes of codes and a 2-byte
// scale unit per row.  In the row-major layout those are 512 scattered pieces per step and
// workgroup: every 128-byte line of codes is fetched four times and every line of scales up to
// 32 times (the per-step footprint, 128 KB, does not fit the 32 KB vector cache), and the
// texture addresser, which works line by line, is busy half of the kernel time.  In the panel
// layout the pieces of consecutive rows are adjacent for a given step:
//     codes   [ceil(K / 64)][rows][32 bytes]
//     scales  [units][rows][2 bytes]   units: pairs of E4M3 bytes per 32 k (NVFP4), or the fp16
//                                      normalised group maximum per group (INT)
//     mul     [rows] fp32              INT only: 2^E(row) / Q
// so a wave reads whole lines.  For INT the scale normalisation of pq_qgemm.hip (recover the
// group's bf16 maximum h = bf16_rne(s * Q), divide by a per-row power of two that puts the row
// maximum in [2^10, 2^11)) happens here, once, instead of in a pass of its own.
// Weights are packed once offline; activations once per forward.
#include "pq_qgemm_common.h"

namespace pq {

size_t operand_bytes(pq_format fmt, int group, int64_t rows, int64_t K) {
  return operand_layout(fmt, group, rows, K).total;
}

constexpr int kPackRows = 8;      // rows per workgroup

// One workgroup of 256 threads moves kPackRows consecutive rows.
//   codes:  a wave covers 8 rows x 4 steps per trip -- it reads 128 contiguous bytes of each row
//           and writes four runs of 256 bytes.
//   scales: a wave covers 8 rows x 8 units per trip.
// DENSE3: the codes come from the dense 3-bit storage of INT3 (pq_int3.hip), rows of 3 K / 8 bytes;
// 32 codes are twelve bytes there and are widened to nibbles on the way.
template <int FMT, int G, bool DENSE3>
__global__ __launch_bounds__(256) void pack_operand_kernel(const uint8_t* __restrict__ codes,
                                                           const void* __restrict__ scales,
                                                           int64_t rows, int64_t K, int64_t steps,
                                                           int64_t units, uint8_t* __restrict__ p_codes,
                                                           uint16_t* __restrict__ p_scales,
                                                           float* __restrict__ p_mul) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t r0 = (int64_t)blockIdx.x * kPackRows;
  {
    const int s_local = lane >> 4, r_local = (lane & 15) >> 1, half = lane & 1;
    const int64_t r = r0 + r_local;
    // four trips' loads in flight before the first store
    for (int64_t s0 = 0; s0 < steps; s0 += 64) {
      uint4 v[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int64_t step = s0 + t * 16 + wave * 4 + s_local;
        const int64_t k0 = step * 64 + half * 32;
        v[t] = make_uint4(0u, 0u, 0u, 0u);
        if (r < rows && k0 < K) {
          if constexpr (DENSE3) {
            const uint32_t* d = reinterpret_cast<const uint32_t*>(codes + r * (K / 8 * 3) + k0 / 8 * 3);
            v[t] = int3_spread32(d[0], d[1], d[2]);
          } else {
            v[t] = *reinterpret_cast<const uint4*>(codes + r * (K / 2) + k0 / 2);
          }
        }
      }
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int64_t step = s0 + t * 16 + wave * 4 + s_local;
        if (r < rows && step < steps) *reinterpret_cast<uint4*>(p_codes + (step * rows + r) * 32 + half * 16) = v[t];
      }
    }
  }
  const int r_local = lane & 7, u_local = lane >> 3;
  const int64_t r = r0 + r_local;
  if constexpr (FMT == kNvfp4) {
    const uint8_t* sc = reinterpret_cast<const uint8_t*>(scales);
    for (int64_t u0 = 0; u0 < units; u0 += 32) {
      const int64_t u = u0 + wave * 8 + u_local;
      if (r < rows && u < units) {
        // K is a multiple of 32, so a unit is whole
        p_scales[u * rows + r] = *reinterpret_cast<const uint16_t*>(sc + r * (K / 16) + u * 2);
      }
    }
  } else {
    constexpr float Q = qmax_of(FMT);
    const float* sc = reinterpret_cast<const float*>(scales);
    __shared__ float row_down[kPackRows];
    // row maximum of the recovered group maxima: wave w takes rows 2 w and 2 w + 1, 32 lanes each
    {
      const int rr = wave * 2 + (lane >> 5);
      const int64_t row = r0 + rr;
      float mx = 0.0f;
      if (row < rows)
        for (int64_t g = lane & 31; g < units; g += 32)
          mx = fmaxf(mx, as_f32(f32_to_bf16_rne(sc[row * units + g] * Q) << 16));
      mx = group_max<32>(mx);
      // E = exponent(mx) - 10: the row maximum lands in [2^10, 2^11), so that the addend 24 * h
      // of the unpack fma stays below the fp16 maximum; clamped so that 2^E and 2^-E are normal
      int e = (int)((as_u32(mx) >> 23) & 0xFF) - 127;
      if (mx == 0.0f) e = 0;
      const int E = max(-120, min(120, e - 10));
      if ((lane & 31) == 0) {
        row_down[rr] = as_f32((uint32_t)(127 - E) << 23);                            // 2^-E
        if (row < rows) p_mul[row] = as_f32((uint32_t)(127 + E) << 23) / Q;          // 2^E / Q
      }
    }
    __syncthreads();
    const float down = row_down[r_local];
    for (int64_t u0 = 0; u0 < units; u0 += 32) {
      const int64_t u = u0 + wave * 8 + u_local;
      if (r < rows && u < units) {
        const float h = as_f32(f32_to_bf16_rne(sc[r * units + u] * Q) << 16);
        const _Float16 hn = (_Float16)(h * down);           // exact unless far below the row maximum
        p_scales[u * rows + r] = __builtin_bit_cast(uint16_t, hn);
      }
    }
  }
}

template <int FMT, int G, bool DENSE3 = false>
static int launch_pack(const uint8_t* codes, const void* scales, int64_t rows, int64_t K,
                       const OperandLayout& L, uint8_t* operand, hipStream_t st) {
  const int64_t blocks = (rows + kPackRows - 1) / kPackRows;
  hipLaunchKernelGGL((pack_operand_kernel<FMT, G, DENSE3>), dim3((unsigned)blocks), dim3(256), 0, st, codes, scales,
                     rows, K, L.steps, L.units, operand + L.codes, (uint16_t*)(operand + L.scales),
                     (float*)(operand + L.mul));
  return check_hip(hipGetLastError(), "pack_operand_kernel");
}

int run_pack_operand(pq_format fmt, int group, const uint8_t* codes, const void* scales, int64_t rows,
                     int64_t K, void* operand, bool dense3, hipStream_t st) {
  if (rows > 0x7FFFFFF0) return fail(PQ_ERR_SHAPE, "too many rows");
  const OperandLayout L = operand_layout(fmt, group, rows, K);
  uint8_t* o = (uint8_t*)operand;
  if (dense3) {
    if (fmt != PQ_FMT_INT3) return fail(PQ_ERR_FORMAT, "dense 3-bit codes are INT3 only");
    switch (group) {
      case 32: return launch_pack<kInt3, 32, true>(codes, scales, rows, K, L, o, st);
      case 64: return launch_pack<kInt3, 64, true>(codes, scales, rows, K, L, o, st);
      case 128: return launch_pack<kInt3, 128, true>(codes, scales, rows, K, L, o, st);
      case 256: return launch_pack<kInt3, 256, true>(codes, scales, rows, K, L, o, st);
    }
    return fail(PQ_ERR_FORMAT, "unsupported (format, group) = (%d, %d)", (int)fmt, group);
  }
  if (fmt == PQ_FMT_NVFP4) return launch_pack<kNvfp4, 16>(codes, scales, rows, K, L, o, st);
#define PQ_INT_CASE(F, FE)                                                \
  if (fmt == F) {                                                         \
    switch (group) {                                                      \
      case 32: return launch_pack<FE, 32>(codes, scales, rows, K, L, o, st);   \
      case 64: return launch_pack<FE, 64>(codes, scales, rows, K, L, o, st);   \
      case 128: return launch_pack<FE, 128>(codes, scales, rows, K, L, o, st); \
      case 256: return launch_pack<FE, 256>(codes, scales, rows, K, L, o, st); \
    }                                                                     \
  }
  PQ_INT_CASE(PQ_FMT_INT4, kInt4)
  PQ_INT_CASE(PQ_FMT_INT3, kInt3)
#undef PQ_INT_CASE
  return fail(PQ_ERR_FORMAT, "unsupported (format, group) = (%d, %d)", (int)fmt, group);
}

int run_qgemm_packed(pq_format fmt, int group, const void* a_operand, const float* a_ts,
                     const void* w_operand, const float* w_ts, int64_t M, int64_t N, int64_t K,
                     const void* bias, void* y, int64_t ldy, bool out_f32, hipStream_t st) {
  if (M * 32 > 0x7FFFFFFF || N * 32 > 0x7FFFFFFF) return fail(PQ_ERR_SHAPE, "too many rows for the panel layout");
  const OperandView A = panel_view(fmt, group, a_operand, M, K, a_ts);
  OperandView W = panel_view(fmt, group, w_operand, N, K, w_ts);
  W.bias = (const uint16_t*)bias;
  return launch_qgemm_views(fmt, group, A, W, M, N, K, y, ldy, out_f32, st);
}

}  // namespace pq
