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

// ------------------------------------------------------------------ fused quantizer -> panel
// Dynamic activation quantization (paper Eq. 1-2, the contract of pq_quantize.hip) that stores
// its result directly in the panel layout, so that the forward path needs no packing pass.
// A workgroup of up to sixteen waves owns RPW rows (8 or 4); a wave works on 64 / RPW chunks (one
// or two 64-wide K steps) of all its rows at a time: lane (64 / RPW) r + c holds chunk c (8
// channels) of row r, the wave loads whole 128-byte lines and stores the rows' codes of a step as
// one contiguous run of 32 RPW bytes.  Groups wider than what a wave covers per trip take
// several trips' chunks at once.  INT: the group maxima of the rows are kept in LDS until the row
// maximum, and with it the per-row power of two, is known.
constexpr int kQuantPanelMaxWaves = 16;

template <int FMT, int G, int RPW>
__global__ __launch_bounds__(64 * kQuantPanelMaxWaves) void quantize_panel_kernel(
    const uint16_t* __restrict__ x, int64_t rows, int64_t K, int64_t ld, const float* __restrict__ tensor_scale,
    int64_t steps, int64_t units, uint8_t* __restrict__ p_codes, uint16_t* __restrict__ p_scales,
    float* __restrict__ p_mul, uint32_t* __restrict__ c_codes, void* __restrict__ c_scales) {
  constexpr int LPR = 64 / RPW;                             // lanes (= chunks per trip) of a row
  constexpr int SPG = G > LPR * 8 ? G / (LPR * 8) : 1;      // trips' worth of chunks a group spans
  constexpr int LPG = G / 8 < LPR ? G / 8 : LPR;            // lanes of a row that share a group
  extern __shared__ float h_lds[];                          // INT: [RPW][units] group maxima
  __shared__ float wave_rowmax[kQuantPanelMaxWaves][RPW];
  // the wave index is uniform over a wave: held in a scalar register, so is every address part
  // that depends only on the group block
  const int tid = threadIdx.x, lane = tid & 63, n_waves = blockDim.x >> 6;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r_local = lane / LPR, c_local = lane % LPR;
  const int64_t r0 = (int64_t)blockIdx.x * RPW;
  const int64_t r = r0 + r_local;
  const bool r_ok = r < rows;
  const int n_chunks = (int)steps * 8;                      // chunks per row, a half step past K included
  const int k_chunks = (int)(K / 8);                        // chunks that exist
  const int n_units = (int)units;
  float T = 0.0f, encT = 0.0f;
  if constexpr (FMT == kNvfp4) {
    T = *tensor_scale;
    encT = nv4_enc_scale(T);
  }
  float row_max = 0.0f;
  const int blocks = (n_chunks + SPG * LPR - 1) / (SPG * LPR);       // group blocks along K
  // per-lane parts of the addresses; chunk cb + c_local (cb a multiple of LPR, uniform) lives at
  //   x_lane + 8 cb,   pc_lane + 32 rows (cb / 8),   ps_lane + rows (cb / 4)   (NVFP4 unit)
  const uint16_t* x_lane = x + (r_ok ? r : 0) * ld + c_local * 8;
  uint8_t* pc_lane = p_codes + ((int64_t)(c_local >> 3) * rows + r) * 32 + (c_local & 7) * 4;
  uint16_t* ps_lane = p_scales + (int64_t)(c_local >> 2) * rows + r;
  uint32_t* cc_lane = c_codes ? c_codes + r * k_chunks + c_local : nullptr;
  // one group block: quantize, store codes and scales
  auto process = [&](int b, const uint4 (&raw)[SPG]) {
    float v[SPG][8];
#pragma unroll
    for (int t = 0; t < SPG; ++t) {
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
      const IntScale sc = int_scale<FMT>(a);
#pragma unroll
      for (int t = 0; t < SPG; ++t) codes[t] = int_codes8(v[t], sc.inv);
      sc_bits = as_u32(sc.s);
      row_max = fmaxf(row_max, a);
    }
    // codes: the panel takes every chunk of a step (a half step past K holds zeros), the
    // row-major copy only what exists
#pragma unroll
    for (int t = 0; t < SPG; ++t) {
      const int cb = (b * SPG + t) * LPR;           // uniform
      if (r_ok && cb + c_local < n_chunks)
        *reinterpret_cast<uint32_t*>(pc_lane + (int64_t)(cb >> 3) * rows * 32) = codes[t];
      if (c_codes && r_ok && cb + c_local < k_chunks) cc_lane[cb] = codes[t];
    }
    // scales
    const int cb0 = b * SPG * LPR;
    if constexpr (FMT == kNvfp4) {
      // a unit is the two bytes of 32 k = four lanes; the first lane of the quad collects the byte
      // of the second pair
      const uint32_t other = dpp_u32<0x4E>(sc_bits);            // lane ^ 2
      const int u = (cb0 + c_local) >> 2;
      if ((c_local & 3) == 0 && r_ok && u < n_units) {
        const uint16_t two = (uint16_t)(sc_bits | (other << 8));
        ps_lane[(int64_t)(cb0 >> 2) * rows] = two;
        if (c_scales) reinterpret_cast<uint16_t*>(c_scales)[r * (K / 32) + u] = two;
      }
    } else {
      // group of this lane's chunk; its first lane stores
      const int g = SPG > 1 ? b : (cb0 + c_local) / (G / 8);
      if (c_local % LPG == 0 && r_ok && g < n_units) {
        h_lds[r_local * n_units + g] = a;
        if (c_scales) reinterpret_cast<uint32_t*>(c_scales)[r * units + g] = sc_bits;
      }
    }
  };
  // U group blocks per trip: their loads are all issued before the first is processed, so that a
  // wave keeps several lines in flight
  constexpr int U = SPG == 1 ? 3 : 1;
  for (int b0 = wave; b0 < blocks; b0 += U * n_waves) {
    uint4 raw[U][SPG];
#pragma unroll
    for (int q = 0; q < U; ++q)
#pragma unroll
      for (int t = 0; t < SPG; ++t) {
        const int cb = ((b0 + q * n_waves) * SPG + t) * LPR;          // uniform
        raw[q][t] = make_uint4(0u, 0u, 0u, 0u);
        if (r_ok && cb + c_local < k_chunks) raw[q][t] = *reinterpret_cast<const uint4*>(x_lane + (int64_t)cb * 8);
      }
#pragma unroll
    for (int q = 0; q < U; ++q) {
      const int b = b0 + q * n_waves;
      if (b < blocks) process(b, raw[q]);              // wave-uniform
    }
  }
  if constexpr (FMT != kNvfp4) {
    constexpr float Q = qmax_of(FMT);
    row_max = group_max<LPR>(row_max);               // the lanes of a row
    if (c_local == 0) wave_rowmax[wave][r_local] = row_max;
    __syncthreads();
    // every thread recomputes the factor of the row it will write below
    const int wr = lane % RPW;                       // row of the write mapping
    float mx = 0.0f;
    for (int w = 0; w < n_waves; ++w) mx = fmaxf(mx, wave_rowmax[w][wr]);
    // E = exponent(mx) - 10: the row maximum lands in [2^10, 2^11) (see pack_operand_kernel)
    int e = (int)((as_u32(mx) >> 23) & 0xFF) - 127;
    if (mx == 0.0f) e = 0;
    const int E = max(-120, min(120, e - 10));
    const float down = as_f32((uint32_t)(127 - E) << 23);
    const int64_t row = r0 + wr;
    if (wave == 0 && lane < RPW && row < rows) p_mul[row] = as_f32((uint32_t)(127 + E) << 23) / Q;
    for (int u0 = 0; u0 < n_units; u0 += LPR * n_waves) {
      const int u = u0 + wave * LPR + lane / RPW;
      if (row < rows && u < n_units) {
        const _Float16 hn = (_Float16)(h_lds[wr * n_units + u] * down);
        p_scales[(int64_t)u * rows + row] = __builtin_bit_cast(uint16_t, hn);
      }
    }
  }
}

template <int FMT, int G, int RPW>
static int launch_qpanel_r(const void* x, int64_t rows, int64_t K, int64_t ld, const float* ts,
                           const OperandLayout& L, uint8_t* operand, uint8_t* codes, void* scales,
                           hipStream_t st) {
  const int64_t blocks = (rows + RPW - 1) / RPW;
  const size_t shmem = FMT == kNvfp4 ? 0 : (size_t)RPW * L.units * sizeof(float);
  auto kern = quantize_panel_kernel<FMT, G, RPW>;
  if (shmem > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
    if (e != hipSuccess) return check_hip(e, "hipFuncSetAttribute(quantize_panel_kernel)");
  }
  // one wave per group block along K, up to eight (four workgroups per compute unit)
  constexpr int LPR = 64 / RPW;
  constexpr int SPG = G > LPR * 8 ? G / (LPR * 8) : 1;
  const int64_t k_blocks = (L.steps * 8 + SPG * LPR - 1) / (SPG * LPR);
  int n_waves = 1;
  while (n_waves < 8 && n_waves * 3 <= k_blocks) n_waves *= 2;   // >= 2-3 trips per wave
  hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(64 * n_waves), shmem, st, (const uint16_t*)x, rows, K, ld, ts,
                     L.steps, L.units, operand + L.codes, (uint16_t*)(operand + L.scales),
                     (float*)(operand + L.mul), (uint32_t*)codes, scales);
  return check_hip(hipGetLastError(), "quantize_panel_kernel");
}

// Eight rows per workgroup: four rows (twice the workgroups, spread more evenly over the compute
// units when rows / 8 is a little above a multiple of 256) measured the same within 2 % on
// 4608 x 3072 with either four or eight waves, so the template is instantiated for 8 only.
template <int FMT, int G>
static int launch_qpanel(const void* x, int64_t rows, int64_t K, int64_t ld, const float* ts,
                         const OperandLayout& L, uint8_t* operand, uint8_t* codes, void* scales,
                         hipStream_t st) {
  return launch_qpanel_r<FMT, G, 8>(x, rows, K, ld, ts, L, operand, codes, scales, st);
}

int run_quantize_packed(pq_format fmt, int group, const void* x, int64_t rows, int64_t K, int64_t ld,
                        const float* ts, void* operand, uint8_t* codes, void* scales, hipStream_t st) {
  if (rows > 0x7FFFFFF0) return fail(PQ_ERR_SHAPE, "too many rows");
  const OperandLayout L = operand_layout(fmt, group, rows, K);
  if (fmt != PQ_FMT_NVFP4 && (size_t)8 * L.units * 4 > 150 * 1024)
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
