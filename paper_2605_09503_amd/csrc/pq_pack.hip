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

struct OperandLayout {
  size_t codes, scales, mul, total;     // byte offsets and total size
  int64_t steps, units;
};

static OperandLayout operand_layout(pq_format fmt, int group, int64_t rows, int64_t K) {
  OperandLayout L;
  L.steps = (K + 63) / 64;
  L.units = fmt == PQ_FMT_NVFP4 ? (K + 31) / 32 : K / group;
  L.codes = 0;
  L.scales = align_up((size_t)L.steps * rows * 32, 256);
  L.mul = L.scales + align_up((size_t)L.units * rows * 2, 256);
  L.total = L.mul + (fmt == PQ_FMT_NVFP4 ? 0 : align_up((size_t)rows * 4, 256));
  return L;
}

size_t operand_bytes(pq_format fmt, int group, int64_t rows, int64_t K) {
  return operand_layout(fmt, group, rows, K).total;
}

constexpr int kPackRows = 8;      // rows per workgroup

// One workgroup of 256 threads moves kPackRows consecutive rows.
//   codes:  a wave covers 8 rows x 4 steps per trip -- it reads 128 contiguous bytes of each row
//           and writes four runs of 256 bytes.
//   scales: a wave covers 8 rows x 8 units per trip.
template <int FMT, int G>
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
        if (r < rows && k0 < K) v[t] = *reinterpret_cast<const uint4*>(codes + r * (K / 2) + k0 / 2);
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

template <int FMT, int G>
static int launch_pack(const uint8_t* codes, const void* scales, int64_t rows, int64_t K,
                       const OperandLayout& L, uint8_t* operand, hipStream_t st) {
  const int64_t blocks = (rows + kPackRows - 1) / kPackRows;
  hipLaunchKernelGGL((pack_operand_kernel<FMT, G>), dim3((unsigned)blocks), dim3(256), 0, st, codes, scales,
                     rows, K, L.steps, L.units, operand + L.codes, (uint16_t*)(operand + L.scales),
                     (float*)(operand + L.mul));
  return check_hip(hipGetLastError(), "pack_operand_kernel");
}

int run_pack_operand(pq_format fmt, int group, const uint8_t* codes, const void* scales, int64_t rows,
                     int64_t K, void* operand, hipStream_t st) {
  if (rows > 0x7FFFFFF0) return fail(PQ_ERR_SHAPE, "too many rows");
  const OperandLayout L = operand_layout(fmt, group, rows, K);
  uint8_t* o = (uint8_t*)operand;
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

// ------------------------------------------------------------------ fused quantizer -> panel
// Dynamic activation quantization (paper Eq. 1-2, the contract of pq_quantize.hip) that stores
// its result directly in the panel layout, so that the forward path needs no packing pass.
// A workgroup of up to sixteen waves owns kPackRows rows; a wave works on one 64-wide K step (or, for
// groups wider than 64, on the G / 64 steps of a group) of all eight rows at a time: lane
// 8 r + c holds chunk c (8 channels) of row r, loads whole 128-byte lines and stores the eight
// rows' codes of a step as one contiguous 256-byte run.  INT: the group maxima of the rows are
// kept in LDS until the row maximum, and with it the per-row power of two, is known.
constexpr int kQuantPanelMaxWaves = 16;

template <int FMT, int G>
__global__ __launch_bounds__(64 * kQuantPanelMaxWaves) void quantize_panel_kernel(const uint16_t* __restrict__ x, int64_t rows,
                                                             int64_t K, int64_t ld,
                                                             const float* __restrict__ tensor_scale,
                                                             int64_t steps, int64_t units,
                                                             uint8_t* __restrict__ p_codes,
                                                             uint16_t* __restrict__ p_scales,
                                                             float* __restrict__ p_mul,
                                                             uint32_t* __restrict__ c_codes,
                                                             void* __restrict__ c_scales) {
  constexpr int SPG = G > 64 ? G / 64 : 1;          // steps a group spans
  constexpr int LPG = G >= 64 ? 8 : G / 8;          // lanes of a row-step that share a group
  extern __shared__ float h_lds[];                  // INT: [kPackRows][units] group maxima
  __shared__ float wave_rowmax[kQuantPanelMaxWaves][kPackRows];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n_waves = blockDim.x >> 6;
  const int r_local = lane >> 3, c_local = lane & 7;
  const int64_t r0 = (int64_t)blockIdx.x * kPackRows;
  const int64_t r = r0 + r_local;
  const bool r_ok = r < rows;
  float T = 0.0f, encT = 0.0f;
  if constexpr (FMT == kNvfp4) {
    T = *tensor_scale;
    encT = nv4_enc_scale(T);
  }
  float row_max = 0.0f;
  const int64_t blocks = (steps + SPG - 1) / SPG;   // group blocks along K (whole: K % G == 0)
  // one group block: quantize, store codes and scales
  auto process = [&](int64_t b, const uint4 (&raw)[SPG]) {
    float v[SPG][8];
    bool k_ok[SPG];
#pragma unroll
    for (int t = 0; t < SPG; ++t) {
      const int64_t k0 = (b * SPG + t) * 64 + c_local * 8;
      k_ok[t] = k0 < K;
      const uint4 p = raw[t];
      v[t][0] = bf16_lo(p.x); v[t][1] = bf16_hi(p.x); v[t][2] = bf16_lo(p.y); v[t][3] = bf16_hi(p.y);
      v[t][4] = bf16_lo(p.z); v[t][5] = bf16_hi(p.z); v[t][6] = bf16_lo(p.w); v[t][7] = bf16_hi(p.w);
    }
    float a = 0.0f;
#pragma unroll
    for (int t = 0; t < SPG; ++t)
#pragma unroll
      for (int j = 0; j < 8; ++j) a = fmaxf(a, fabsf(v[t][j]));
    a = group_max<LPG>(a);
    uint32_t codes[SPG];
    uint32_t sc_bits;                               // NVFP4: E4M3 byte; INT: fp32 bits of the scale
    if constexpr (FMT == kNvfp4) {
      const Nv4Scale sc = nv4_scale(a, T, encT);
#pragma unroll
      for (int t = 0; t < SPG; ++t) {
        uint32_t c = 0;
        c = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(c, v[t][0] * sc.inv, v[t][1] * sc.inv, 1.0f, 0);
        c = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(c, v[t][2] * sc.inv, v[t][3] * sc.inv, 1.0f, 1);
        c = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(c, v[t][4] * sc.inv, v[t][5] * sc.inv, 1.0f, 2);
        c = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(c, v[t][6] * sc.inv, v[t][7] * sc.inv, 1.0f, 3);
        codes[t] = c;
      }
      sc_bits = sc.byte;
    } else {
      constexpr float Q = qmax_of(FMT);
      const IntScale sc = int_scale<FMT>(a);
#pragma unroll
      for (int t = 0; t < SPG; ++t) {
        uint32_t c = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) c |= int_code(v[t][j], sc.inv, Q) << (4 * j);
        codes[t] = c;
      }
      sc_bits = as_u32(sc.s);
      row_max = fmaxf(row_max, a);
    }
    // codes: the panel takes every chunk of the step (a half step past K holds zeros), the
    // row-major copy only what exists
#pragma unroll
    for (int t = 0; t < SPG; ++t) {
      const int64_t step = b * SPG + t;
      if (r_ok && step < steps)
        *reinterpret_cast<uint32_t*>(p_codes + (step * rows + r) * 32 + c_local * 4) = codes[t];
      if (c_codes && r_ok && k_ok[t]) c_codes[r * (K / 8) + step * 8 + c_local] = codes[t];
    }
    // scales
    if constexpr (FMT == kNvfp4) {
      // a unit is the two bytes of 32 k = four lanes; the first lane of the quad collects the byte
      // of the second pair
      const uint32_t other = dpp_u32<0x4E>(sc_bits);            // lane ^ 2
      const int64_t u = b * 2 + (c_local >> 2);
      if ((c_local & 3) == 0 && r_ok && u < units) {
        const uint16_t two = (uint16_t)(sc_bits | (other << 8));
        p_scales[u * rows + r] = two;
        if (c_scales) reinterpret_cast<uint16_t*>(c_scales)[r * (K / 32) + u] = two;
      }
    } else {
      // group index of this lane's chunk; its first lane stores
      const int64_t g = G >= 64 ? b : b * (64 / G) + c_local / LPG;
      const bool leader = G >= 64 ? c_local == 0 : c_local % LPG == 0;
      if (leader && r_ok && g < units) {
        h_lds[r_local * units + g] = a;
        if (c_scales) reinterpret_cast<uint32_t*>(c_scales)[r * units + g] = sc_bits;
      }
    }
  };
  // U group blocks per trip: their loads are all issued before the first is processed, so that a
  // wave keeps several lines in flight
  constexpr int U = SPG == 1 ? 3 : 1;
  for (int64_t b0 = wave; b0 < blocks; b0 += (int64_t)U * n_waves) {
    uint4 raw[U][SPG];
#pragma unroll
    for (int q = 0; q < U; ++q)
#pragma unroll
      for (int t = 0; t < SPG; ++t) {
        const int64_t k0 = ((b0 + (int64_t)q * n_waves) * SPG + t) * 64 + c_local * 8;
        raw[q][t] = make_uint4(0u, 0u, 0u, 0u);
        if (r_ok && k0 < K) raw[q][t] = *reinterpret_cast<const uint4*>(x + r * ld + k0);
      }
#pragma unroll
    for (int q = 0; q < U; ++q) {
      const int64_t b = b0 + (int64_t)q * n_waves;
      if (b < blocks) process(b, raw[q]);              // wave-uniform
    }
  }
  if constexpr (FMT != kNvfp4) {
    constexpr float Q = qmax_of(FMT);
    row_max = group_max<8>(row_max);                 // the eight lanes of a row
    if (c_local == 0) wave_rowmax[wave][r_local] = row_max;
    __syncthreads();
    // every thread recomputes the factor of the row it will write below
    const int wr = lane & 7;                         // row of the write mapping
    float mx = 0.0f;
    for (int w = 0; w < n_waves; ++w) mx = fmaxf(mx, wave_rowmax[w][wr]);
    // E = exponent(mx) - 10: the row maximum lands in [2^10, 2^11) (see pack_operand_kernel)
    int e = (int)((as_u32(mx) >> 23) & 0xFF) - 127;
    if (mx == 0.0f) e = 0;
    const int E = max(-120, min(120, e - 10));
    const float down = as_f32((uint32_t)(127 - E) << 23);
    const int64_t row = r0 + wr;
    if (wave == 0 && lane < kPackRows && row < rows) p_mul[row] = as_f32((uint32_t)(127 + E) << 23) / Q;
    for (int64_t u0 = 0; u0 < units; u0 += 8 * n_waves) {
      const int64_t u = u0 + wave * 8 + (lane >> 3);
      if (row < rows && u < units) {
        const _Float16 hn = (_Float16)(h_lds[wr * units + u] * down);
        p_scales[u * rows + row] = __builtin_bit_cast(uint16_t, hn);
      }
    }
  }
}

template <int FMT, int G>
static int launch_qpanel(const void* x, int64_t rows, int64_t K, int64_t ld, const float* ts,
                         const OperandLayout& L, uint8_t* operand, uint8_t* codes, void* scales,
                         hipStream_t st) {
  const int64_t blocks = (rows + kPackRows - 1) / kPackRows;
  const size_t shmem = FMT == kNvfp4 ? 0 : (size_t)kPackRows * L.units * sizeof(float);
  auto kern = quantize_panel_kernel<FMT, G>;
  if (shmem > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
    if (e != hipSuccess) return check_hip(e, "hipFuncSetAttribute(quantize_panel_kernel)");
  }
  // one wave per group block along K, up to sixteen
  constexpr int SPG = G > 64 ? G / 64 : 1;
  const int64_t k_blocks = (L.steps + SPG - 1) / SPG;
  int n_waves = 1;
  while (n_waves < 8 && n_waves * 3 <= k_blocks) n_waves *= 2;   // >= 2-3 trips per wave, four workgroups per compute unit
  hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(64 * n_waves), shmem, st, (const uint16_t*)x, rows, K, ld, ts,
                     L.steps, L.units, operand + L.codes, (uint16_t*)(operand + L.scales),
                     (float*)(operand + L.mul), (uint32_t*)codes, scales);
  return check_hip(hipGetLastError(), "quantize_panel_kernel");
}

int run_quantize_packed(pq_format fmt, int group, const void* x, int64_t rows, int64_t K, int64_t ld,
                        const float* ts, void* operand, uint8_t* codes, void* scales, hipStream_t st) {
  if (rows > 0x7FFFFFF0) return fail(PQ_ERR_SHAPE, "too many rows");
  const OperandLayout L = operand_layout(fmt, group, rows, K);
  if (fmt != PQ_FMT_NVFP4 && (size_t)kPackRows * L.units * 4 > 150 * 1024)
    return fail(PQ_ERR_SHAPE, "K=%lld has too many groups for the fused quantizer", (long long)K);
  uint8_t* o = (uint8_t*)operand;
  if (fmt == PQ_FMT_NVFP4) return launch_qpanel<kNvfp4, 16>(x, rows, K, ld, ts, L, o, codes, scales, st);
#define PQ_INT_CASE(F, FE)                                                                  \
  if (fmt == F) {                                                                           \
    switch (group) {                                                                        \
      case 32: return launch_qpanel<FE, 32>(x, rows, K, ld, ts, L, o, codes, scales, st);   \
      case 64: return launch_qpanel<FE, 64>(x, rows, K, ld, ts, L, o, codes, scales, st);   \
      case 128: return launch_qpanel<FE, 128>(x, rows, K, ld, ts, L, o, codes, scales, st); \
      case 256: return launch_qpanel<FE, 256>(x, rows, K, ld, ts, L, o, codes, scales, st); \
    }                                                                                       \
  }
  PQ_INT_CASE(PQ_FMT_INT4, kInt4)
  PQ_INT_CASE(PQ_FMT_INT3, kInt3)
#undef PQ_INT_CASE
  return fail(PQ_ERR_FORMAT, "unsupported (format, group) = (%d, %d)", (int)fmt, group);
}

static OperandView panel_view(pq_format fmt, int group, const void* operand, int64_t rows, int64_t K,
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

int run_qgemm_packed(pq_format fmt, int group, const void* a_operand, const float* a_ts,
                     const void* w_operand, const float* w_ts, int64_t M, int64_t N, int64_t K, void* y,
                     int64_t ldy, bool out_f32, hipStream_t st) {
  if (M * 32 > 0x7FFFFFFF || N * 32 > 0x7FFFFFFF) return fail(PQ_ERR_SHAPE, "too many rows for the panel layout");
  const OperandView A = panel_view(fmt, group, a_operand, M, K, a_ts);
  const OperandView W = panel_view(fmt, group, w_operand, N, K, w_ts);
  return launch_qgemm_views(fmt, group, A, W, M, N, K, y, ldy, out_f32, st);
}

}  // namespace pq
