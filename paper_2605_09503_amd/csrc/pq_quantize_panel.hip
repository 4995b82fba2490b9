// Dynamic activation quantization (paper Eq. 1-2, applied online per token row; the arithmetic is the
// contract of pq_quantize.hip) that stores its result directly in the GEMM's panel layout
// (pq_pack.hip), so that the forward path needs no packing pass.  Two kernels:
//
// quantize_panel_kernel (every format).  A workgroup of up to sixteen waves owns RPW rows; a wave works on
// 64 / RPW chunks (one 64-wide K step for RPW = 8) of eight rows at a time: lane (64 / RPW) r + c holds
// chunk c (8 channels) of row r, the wave loads whole 128-byte lines and stores the rows' codes of a step
// as one contiguous run of 32 RPW bytes.  INT: the waves share the workgroup's rows and take the group
// blocks along K in turn; the group maxima are kept in LDS until the row maximum, and with it the per-row
// power of two of the operand, is known.  NVFP4: nothing links the blocks of a row, so every wave takes
// rows of its own and the blocks along K are shared out over several workgroups.
//
// quantize_panel_nv4_kernel (NVFP4, large tensors).  Reads and writes want different shapes.  The input is
// read fastest as it lies -- a wave takes 1 KB of one row per load instruction, like a plain streaming
// kernel; eight rows x 128 bytes per instruction put all eight requests on one L2 channel (rows are a
// multiple of 2 KB apart).  The panel, [K step][row][32 bytes] and [scale unit][row][2 bytes], is written
// fastest in long runs over consecutive rows: with eight rows per workgroup the 16-byte pieces of eight
// workgroups share every 128-byte line of the scale panel, and at 4608 x 12288 those 3.5 MB of partial-line
// writes cost 2.5 us of 30, half as much as the 28 MB of codes.  So a workgroup takes a block of 512
// columns of 64 rows (eight rows per wave, their loads all in flight together); codes (4 bytes per lane)
// and scale units cross through LDS, and after one barrier the threads store 16-byte pieces: 2 KB of
// contiguous codes per K step, one whole line per scale unit.  4608 x 12288, cold: 30.3 -> 28.6 us (the
// streaming reference with the same footprint: 24.6 us).  On the 28 MB tensors of the other layers the
// barrier and the short life of a workgroup cost more than the access pattern gains (10.3 against 9.0 us
// for 4608 x 3072), so those keep the first kernel.
#include "pq_qgemm_common.h"

namespace pq {

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
  // INT: the waves of a workgroup share its RPW rows and take the group blocks along K in turn (the row
  // maximum is needed before the scale units can be written).  NVFP4: nothing links the blocks of a row,
  // so every wave takes RPW rows of its own and walks consecutive blocks -- at any moment the waves of a
  // workgroup write one run of n_waves * RPW * 32 bytes of the panel (1 KB with four waves) instead of
  // 256-byte pieces a whole panel step apart, and a wave's loads in flight are consecutive pieces of its rows.
  constexpr bool kWaveRows = FMT == kNvfp4;
  const int64_t r0 = kWaveRows ? ((int64_t)blockIdx.x * n_waves + wave) * RPW : (int64_t)blockIdx.x * RPW;
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
  // FULL (compile-time): every row of the workgroup exists and K is a whole number of group blocks, so no
  // access needs a bounds test
  auto process = [&](auto fullc, int b, const uint4 (&raw)[SPG]) {
    constexpr bool FULL = decltype(fullc)::value;
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
      if (FULL || (r_ok && cb + c_local < n_chunks))
        *reinterpret_cast<uint32_t*>(pc_lane + (int64_t)(cb >> 3) * rows * 32) = codes[t];
      if (c_codes && (FULL || (r_ok && cb + c_local < k_chunks))) cc_lane[cb] = codes[t];
    }
    // scales
    const int cb0 = b * SPG * LPR;
    if constexpr (FMT == kNvfp4) {
      // a unit is the two bytes of 32 k = four lanes; the first lane of the quad collects the byte
      // of the second pair
      const uint32_t other = dpp_u32<0x4E>(sc_bits);            // lane ^ 2
      const int u = (cb0 + c_local) >> 2;
      if ((c_local & 3) == 0 && (FULL || (r_ok && u < n_units))) {
        const uint16_t two = (uint16_t)(sc_bits | (other << 8));
        ps_lane[(int64_t)(cb0 >> 2) * rows] = two;
        if (c_scales) reinterpret_cast<uint16_t*>(c_scales)[r * (K / 32) + u] = two;
      }
    } else {
      // group of this lane's chunk; its first lane stores
      const int g = SPG > 1 ? b : (cb0 + c_local) / (G / 8);
      if (c_local % LPG == 0 && (FULL || (r_ok && g < n_units))) {
        h_lds[r_local * n_units + g] = a;
        if (c_scales) reinterpret_cast<uint32_t*>(c_scales)[r * units + g] = sc_bits;
      }
    }
  };
  // U group blocks per trip: their loads are all issued before the first is processed, so that a
  // wave keeps several lines in flight
  // gridDim.y workgroups share the group blocks of a row set (NVFP4 only: nothing links the blocks of a
  // row there; the INT formats need the row maximum and keep a row set in one workgroup)
  constexpr int U = SPG == 1 ? 3 : 1;
  const int per_split = (blocks + (int)gridDim.y - 1) / (int)gridDim.y;
  const int b_begin = (int)blockIdx.y * per_split, b_end = min(blocks, b_begin + per_split);
  auto run = [&](auto fullc) {
    constexpr bool FULL = decltype(fullc)::value;
    const int b_first = kWaveRows ? b_begin : b_begin + wave;
    const int b_step = kWaveRows ? 1 : n_waves;           // distance of the blocks of one trip
    for (int b0 = b_first; b0 < b_end; b0 += U * b_step) {
      uint4 raw[U][SPG];
#pragma unroll
      for (int q = 0; q < U; ++q)
#pragma unroll
        for (int t = 0; t < SPG; ++t) {
          const int cb = ((b0 + q * b_step) * SPG + t) * LPR;           // uniform
          raw[q][t] = make_uint4(0u, 0u, 0u, 0u);
          if (b0 + q * b_step < b_end && (FULL || (r_ok && cb + c_local < k_chunks)))
            raw[q][t] = *reinterpret_cast<const uint4*>(x_lane + (int64_t)cb * 8);
        }
#pragma unroll
      for (int q = 0; q < U; ++q) {
        const int b = b0 + q * b_step;
        if (b < b_end) process(fullc, b, raw[q]);        // wave-uniform
      }
    }
  };
  if (r0 + RPW <= rows && k_chunks == n_chunks && k_chunks % (SPG * LPR) == 0) run(IntC<1>{});     // wave-uniform
  else run(IntC<0>{});
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
  // NVFP4: four waves with RPW rows each; the group blocks along K are shared out over several workgroups
  // until there are enough of them (some eight per compute unit) for the dispatcher to even out the load
  // (one workgroup per row set of 4608 rows gave 576 workgroups, 2.25 per unit: some units got three)
  int k_split = 1;
  int64_t wgs = blocks;
  if (FMT == kNvfp4) {
    n_waves = 32 / RPW;                                            // 32 rows per workgroup
    wgs = (rows + RPW * n_waves - 1) / (RPW * n_waves);
    while (wgs * k_split < 2048 && k_blocks / (k_split * 2) >= 3) k_split *= 2;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)wgs, (unsigned)k_split), dim3(64 * n_waves), shmem, st, (const uint16_t*)x, rows, K, ld, ts,
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

// NVFP4.  RW rows per wave, NW waves: a workgroup covers WR = RW * NW rows and walks column blocks of 512
// channels; per block a lane loads one 16-byte chunk of each of its wave's rows.
template <int RW, int NW>
__global__ __launch_bounds__(64 * NW) void quantize_panel_nv4_kernel(
    const uint16_t* __restrict__ x, int64_t rows, int64_t K, int64_t ld, const float* __restrict__ tensor_scale,
    int64_t steps, int64_t units, uint8_t* __restrict__ p_codes, uint16_t* __restrict__ p_scales,
    uint32_t* __restrict__ c_codes, uint16_t* __restrict__ c_scales, int blocks_per_wg) {
  constexpr int WR = RW * NW;
  constexpr int kStepWords = WR * 8 + 8;          // one spare 32-byte slot per K step spreads the steps over the banks
  __shared__ __attribute__((aligned(16))) uint32_t code_lds[2][8][kStepWords];   // [buffer][step][row][chunk]
  __shared__ __attribute__((aligned(16))) uint16_t unit_lds[2][16][WR];          // [buffer][unit][row]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t r0 = (int64_t)blockIdx.x * WR;
  const int k_chunks = (int)(K / 8);
  const int n_steps = (int)steps, n_units = (int)units;
  const int n_blocks = (n_steps + 7) / 8;
  const int b_begin = (int)blockIdx.y * blocks_per_wg;
  const int b_end = min(n_blocks, b_begin + blocks_per_wg);
  const float T = *tensor_scale;
  const float encT = nv4_enc_scale(T);
  int buf = 0;
  for (int blk = b_begin; blk < b_end; ++blk, buf ^= 1) {
    const int kc = blk * 64 + lane;
    uint4 raw[RW];
#pragma unroll
    for (int i = 0; i < RW; ++i) {
      const int64_t r = r0 + wave * RW + i;
      raw[i] = make_uint4(0u, 0u, 0u, 0u);
      if (r < rows && kc < k_chunks) raw[i] = *reinterpret_cast<const uint4*>(x + r * ld + (int64_t)kc * 8);
    }
#pragma unroll
    for (int i = 0; i < RW; ++i) {
      const int row_l = wave * RW + i;
      const int64_t r = r0 + row_l;
      const uint4 p = raw[i];
      float v[8];
      v[0] = bf16_lo(p.x); v[1] = bf16_hi(p.x); v[2] = bf16_lo(p.y); v[3] = bf16_hi(p.y);
      v[4] = bf16_lo(p.z); v[5] = bf16_hi(p.z); v[6] = bf16_lo(p.w); v[7] = bf16_hi(p.w);
      float a = 0.0f;
#pragma unroll
      for (int j = 0; j < 8; ++j) a = fmaxf(a, fabsf(v[j]));
      a = group_max<2>(a);
      const Nv4Scale sc = nv4_scale(a, T, encT);
      uint32_t code = 0;
      code = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(code, v[0] * sc.inv, v[1] * sc.inv, 1.0f, 0);
      code = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(code, v[2] * sc.inv, v[3] * sc.inv, 1.0f, 1);
      code = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(code, v[4] * sc.inv, v[5] * sc.inv, 1.0f, 2);
      code = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(code, v[6] * sc.inv, v[7] * sc.inv, 1.0f, 3);
      code_lds[buf][lane >> 3][row_l * 8 + (lane & 7)] = code;
      // a unit is the two scale bytes of 32 channels = four lanes; the first lane of the quad collects the
      // byte of the second pair
      const uint32_t other = dpp_u32<0x4E>(sc.byte);             // lane ^ 2
      if ((lane & 3) == 0) {
        const uint16_t two = (uint16_t)(sc.byte | (other << 8));
        unit_lds[buf][lane >> 2][row_l] = two;
        const int u = blk * 16 + (lane >> 2);
        if (c_scales && r < rows && u < n_units) c_scales[r * (K / 32) + u] = two;
      }
      if (c_codes && r < rows && kc < k_chunks) c_codes[r * k_chunks + kc] = code;
    }
    __syncthreads();
    // stores: 16-byte pieces; consecutive threads walk the rows of a K step, so a step's codes leave as one
    // run of 32 WR bytes and a unit's scales as one run of 2 WR bytes
    for (int idx = tid; idx < WR * 16; idx += 64 * NW) {
      const int step_l = idx / (2 * WR), piece = idx % (2 * WR);
      const int row_l = piece >> 1, half = piece & 1;
      const int64_t step = (int64_t)blk * 8 + step_l;
      if (step < n_steps && r0 + row_l < rows) {
        const uint4 c = *reinterpret_cast<const uint4*>(&code_lds[buf][step_l][row_l * 8 + half * 4]);
        *reinterpret_cast<uint4*>(p_codes + (step * rows + r0 + row_l) * 32 + half * 16) = c;
      }
    }
    if (tid < 2 * WR) {
      const int u_l = tid / (WR / 8), piece = tid % (WR / 8);
      const int64_t u = (int64_t)blk * 16 + u_l;
      const int64_t rr0 = r0 + piece * 8;
      if (u < n_units && rr0 < rows) {
        uint16_t* dst = p_scales + u * rows + rr0;
        if ((rows & 7) == 0) {                                   // eight whole rows, 16-byte aligned
          *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(&unit_lds[buf][u_l][piece * 8]);
        } else {
          for (int rr = 0; rr < 8 && rr0 + rr < rows; ++rr) dst[rr] = unit_lds[buf][u_l][piece * 8 + rr];
        }
      }
    }
  }
}

template <int RW>
static int launch_qpanel_nv4(const void* x, int64_t rows, int64_t K, int64_t ld, const float* ts,
                             const OperandLayout& L, uint8_t* operand, uint8_t* codes, void* scales, hipStream_t st) {
  constexpr int NW = 8;
  const int64_t row_sets = (rows + RW * NW - 1) / (RW * NW);
  const int n_blocks = (int)((L.steps + 7) / 8);
  // one column block per workgroup unless that makes more than some 16 workgroups per compute unit
  int per_wg = 1;
  while (row_sets * ((n_blocks + per_wg - 1) / per_wg) > 4096 && per_wg < n_blocks) per_wg *= 2;
  const int k_split = (n_blocks + per_wg - 1) / per_wg;
  hipLaunchKernelGGL((quantize_panel_nv4_kernel<RW, NW>), dim3((unsigned)row_sets, (unsigned)k_split), dim3(64 * NW), 0, st,
                     (const uint16_t*)x, rows, K, ld, ts, L.steps, L.units, operand + L.codes,
                     (uint16_t*)(operand + L.scales), (uint32_t*)codes, (uint16_t*)scales, per_wg);
  return check_hip(hipGetLastError(), "quantize_panel_nv4_kernel");
}

int run_quantize_packed(pq_format fmt, int group, const void* x, int64_t rows, int64_t K, int64_t ld,
                        const float* ts, void* operand, uint8_t* codes, void* scales, hipStream_t st) {
  if (rows > 0x7FFFFFF0) return fail(PQ_ERR_SHAPE, "too many rows");
  const OperandLayout L = operand_layout(fmt, group, rows, K);
  if (fmt != PQ_FMT_NVFP4 && (size_t)8 * L.units * 4 > 150 * 1024)
    return fail(PQ_ERR_SHAPE, "K=%lld has too many groups for the fused quantizer", (long long)K);
  uint8_t* o = (uint8_t*)operand;
  if (fmt == PQ_FMT_NVFP4) {
    // the 64-row kernel when that still leaves four workgroups per compute unit
    const int64_t n_blocks = (L.steps + 7) / 8;
    if ((rows + 63) / 64 * n_blocks >= 1024) return launch_qpanel_nv4<8>(x, rows, K, ld, ts, L, o, codes, scales, st);
    return launch_qpanel<kNvfp4, 16>(x, rows, K, ld, ts, L, o, codes, scales, st);
  }
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

}  // namespace pq
