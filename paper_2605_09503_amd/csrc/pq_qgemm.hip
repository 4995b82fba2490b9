// Low-bit GEMM of the reordered quantized layer (paper Eq. 8):
//     Y[m, n] = Ta Tw sum_g sa[m, g] sw[n, g] sum_{k in g} a[m, k] w[n, k]
//
// Design for gfx950.  The contraction runs on the fp16 MFMA (v_mfma_f32_32x32x16_f16, fp32
// accumulate).  Both operands stay 4-bit in HBM and L2; a workgroup unpacks its A and W tiles
// once per K step straight into fp16 values that already carry the per-group scale, and stages
// them in LDS:
//   NVFP4  value = E2M1 code * E4M3 block scale: 2 + 4 significant bits and an exponent range
//          of [2^-10, 2688] -- exact in fp16.  The two fp32 tensor scales go to the epilogue.
//   INT    the stored scale is s = fl32(h / Q) with h the group's bf16 maximum, so h is
//          recovered exactly as bf16_rne(s * Q) and the operand is z * h * 2^-E(row): 3 + 8
//          significant bits, exact in fp16; E(row) keeps the row's largest group below the
//          fp16 maximum.  2^E(row) / Q goes to the epilogue.
// The MFMA then forms exact products of the scaled operands and adds them in fp32, i.e. the
// per-group scale products are applied inside the K accumulation without any per-group pass
// over the accumulators on the vector ALU (that pass would cost 2 lane-ops per output per
// group and would bound the kernel well below the matrix pipe).
//
// Tiling: BM x BN output tile per workgroup, BK = 64 per step, double-buffered LDS, one
// barrier per step.  Waves form a WGM x WGN grid; each owns (BM/WGM) x (BN/WGN) outputs as
// 32x32 MFMA tiles.  The MFMA "A" operand is the weight tile and "B" the activation tile, so
// a lane ends up with 4 consecutive n for one m and stores 8 bytes of bf16 at once.
// LDS rows are 128 bytes (64 fp16) in 16-byte pieces, piece index XOR (row & 7): conflict-free
// for the 16-byte fragment reads and for the unpack writes.
#include "pq_device.h"
#include "pq_host.h"

namespace pq {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));

constexpr int kBK = 64;                 // K elements per step
constexpr int kRowBytes = kBK * 2;      // fp16 row in LDS

__device__ __forceinline__ half2_t as_h2(uint32_t u) { return __builtin_bit_cast(half2_t, u); }
__device__ __forceinline__ uint32_t h2_bits(half2_t h) { return __builtin_bit_cast(uint32_t, h); }

// ------------------------------------------------------------------------ operand unpack
// Eight 4-bit codes (one dword) -> eight fp16 values times the group scale (sc = {s, s}).
// The position of an element inside the group of eight only has to be the same for A and W.
template <int FMT>
__device__ __forceinline__ uint4 unpack8_scaled(uint32_t d, half2_t sc) {
  uint4 o;
  if constexpr (FMT == kNvfp4) {
    o.x = h2_bits(__builtin_amdgcn_cvt_scalef32_pk_f16_fp4(d, 1.0f, 0) * sc);
    o.y = h2_bits(__builtin_amdgcn_cvt_scalef32_pk_f16_fp4(d, 1.0f, 1) * sc);
    o.z = h2_bits(__builtin_amdgcn_cvt_scalef32_pk_f16_fp4(d, 1.0f, 2) * sc);
    o.w = h2_bits(__builtin_amdgcn_cvt_scalef32_pk_f16_fp4(d, 1.0f, 3) * sc);
  } else {
    // two's complement nibble z -> offset binary u = z + 8 -> fp16 1024 + u -> subtract 1032
    const uint32_t x = d ^ 0x88888888u;
    const half2_t off = {(_Float16)1032.0f, (_Float16)1032.0f};
    o.x = h2_bits((as_h2((x & 0x000F000Fu) | 0x64006400u) - off) * sc);
    o.y = h2_bits((as_h2(((x >> 4) & 0x000F000Fu) | 0x64006400u) - off) * sc);
    o.z = h2_bits((as_h2(((x >> 8) & 0x000F000Fu) | 0x64006400u) - off) * sc);
    o.w = h2_bits((as_h2(((x >> 12) & 0x000F000Fu) | 0x64006400u) - off) * sc);
  }
  return o;
}

// Per-thread slice of a tile row: 32 consecutive k (16 bytes of codes) plus its scales.
struct Slice {
  uint4 codes;
  uint32_t sc;      // NVFP4: two E4M3 bytes (k 0-15, 16-31); INT: one fp16 in the low half
};

// scale source for one operand
struct ScaleSrc {
  const uint8_t* e4m3;      // NVFP4: [rows, K/16]
  const uint16_t* f16;      // INT: normalised group maxima, [rows, K/G]
};

template <int FMT, int G>
__device__ __forceinline__ Slice load_slice(const uint8_t* __restrict__ codes, const ScaleSrc& sc,
                                            int row, int rows, int K, int k0) {
  Slice s;
  if (row < rows && k0 < K) {
    s.codes = *reinterpret_cast<const uint4*>(codes + (int64_t)row * (K / 2) + k0 / 2);
    if constexpr (FMT == kNvfp4) {
      s.sc = *reinterpret_cast<const uint16_t*>(sc.e4m3 + (int64_t)row * (K / 16) + k0 / 16);
    } else {
      s.sc = sc.f16[(int64_t)row * (K / G) + k0 / G];
    }
  } else {
    s.codes = make_uint4(0, 0, 0, 0);     // zero codes: contribute nothing
    s.sc = 0;
    if constexpr (FMT != kNvfp4) s.codes = make_uint4(0, 0, 0, 0);
  }
  return s;
}

template <int FMT>
__device__ __forceinline__ void unpack_slice(const Slice& s, uint4 (&out)[4]) {
  half2_t s0, s1;
  if constexpr (FMT == kNvfp4) {
    // E4M3 byte b -> fp16: bits (b << 7) read as fp16 are value * 2^-8, subnormals included
    uint32_t two = ((s.sc & 0xFFu) << 7) | ((s.sc & 0xFF00u) << 15);
    half2_t v = as_h2(two) * (half2_t){(_Float16)256.0f, (_Float16)256.0f};
    s0 = (half2_t){v.x, v.x};
    s1 = (half2_t){v.y, v.y};
  } else {
    half2_t v = as_h2((s.sc & 0xFFFFu) | (s.sc << 16));
    s0 = v;
    s1 = v;
  }
  out[0] = unpack8_scaled<FMT>(s.codes.x, s0);
  out[1] = unpack8_scaled<FMT>(s.codes.y, s0);
  out[2] = unpack8_scaled<FMT>(s.codes.z, s1);
  out[3] = unpack8_scaled<FMT>(s.codes.w, s1);
}

// tile row `r`, 16-byte piece `piece` (0..7) -> byte offset inside one LDS operand tile
__device__ __forceinline__ int lds_off(int r, int piece) {
  return r * kRowBytes + ((piece ^ (r & 7)) << 4);
}

template <int FMT, int G, int BM, int BN, int WGM, int WGN, bool OUT_F32>
__global__ __launch_bounds__(WGM* WGN * 64) void qgemm_kernel(
    const uint8_t* __restrict__ a_codes, ScaleSrc a_sc, const uint8_t* __restrict__ w_codes,
    ScaleSrc w_sc, const float* __restrict__ a_mul, int a_mul_stride,
    const float* __restrict__ w_mul, int w_mul_stride, int M, int N, int K, void* __restrict__ y,
    int64_t ldy, int tiles_m, int tiles_n) {
  constexpr int T = WGM * WGN * 64;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;      // wave tile
  constexpr int TM = WTM / 32, TN = WTN / 32;        // MFMA tiles per wave
  constexpr int A_SLOTS = BM * 2 / T, W_SLOTS = BN * 2 / T;
  static_assert(BM * 2 % T == 0 && BN * 2 % T == 0, "loader mapping");
  static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile");
  constexpr int A_TILE_BYTES = BM * kRowBytes, W_TILE_BYTES = BN * kRowBytes;
  constexpr int STAGE_BYTES = A_TILE_BYTES + W_TILE_BYTES;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  // ---- tile assignment: consecutive workgroup ids land on different XCDs (8 of them, each
  // with its own L2); give every XCD a contiguous range of tiles, and walk tiles in bands of
  // 8 along M so that concurrently running workgroups share A and W strips.
  const int n_tiles = tiles_m * tiles_n;
  int pid = blockIdx.x;
  {
    const int per_xcd = (n_tiles + 7) / 8;
    int xcd = pid & 7, local = pid >> 3;
    int remapped = xcd * per_xcd + local;
    // the last XCD ranges may be short when n_tiles % 8 != 0; fall back to the identity then
    if (n_tiles % 8 == 0) pid = remapped;
  }
  constexpr int BAND = 8;
  const int band_sz = BAND * tiles_n;
  const int band = pid / band_sz;
  const int band_m0 = band * BAND;
  const int band_h = min(BAND, tiles_m - band_m0);
  const int in_band = pid - band * band_sz;
  const int tile_m = band_m0 + in_band % band_h;
  const int tile_n = in_band / band_h;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave % WGM, wave_n = wave / WGM;

  // loader: slot s covers tile row (s*T + tid) / 2, half (tid & 1) -> k offset 32 * half
  const int ld_half = tid & 1;

  float16_t acc[TN][TM];
#pragma unroll
  for (int i = 0; i < TN; ++i)
#pragma unroll
    for (int j = 0; j < TM; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  Slice a_reg[A_SLOTS], w_reg[W_SLOTS];

  auto load_global = [&](int kstep) {
    const int k0 = kstep * kBK + ld_half * 32;
#pragma unroll
    for (int s = 0; s < A_SLOTS; ++s) {
      int r = (s * T + tid) >> 1;
      a_reg[s] = load_slice<FMT, G>(a_codes, a_sc, m0 + r, M, K, k0);
    }
#pragma unroll
    for (int s = 0; s < W_SLOTS; ++s) {
      int r = (s * T + tid) >> 1;
      w_reg[s] = load_slice<FMT, G>(w_codes, w_sc, n0 + r, N, K, k0);
    }
  };
  auto store_lds = [&](int stage) {
    unsigned char* a_t = smem + stage * STAGE_BYTES;
    unsigned char* w_t = a_t + A_TILE_BYTES;
#pragma unroll
    for (int s = 0; s < A_SLOTS; ++s) {
      int r = (s * T + tid) >> 1;
      uint4 v[4];
      unpack_slice<FMT>(a_reg[s], v);
#pragma unroll
      for (int q = 0; q < 4; ++q)
        *reinterpret_cast<uint4*>(a_t + lds_off(r, ld_half * 4 + q)) = v[q];
    }
#pragma unroll
    for (int s = 0; s < W_SLOTS; ++s) {
      int r = (s * T + tid) >> 1;
      uint4 v[4];
      unpack_slice<FMT>(w_reg[s], v);
#pragma unroll
      for (int q = 0; q < 4; ++q)
        *reinterpret_cast<uint4*>(w_t + lds_off(r, ld_half * 4 + q)) = v[q];
    }
  };

  const int ksteps = (K + kBK - 1) / kBK;
  load_global(0);
  store_lds(0);
  __syncthreads();

  const int frag_row = lane & 31, frag_half = lane >> 5;
  for (int ks = 0; ks < ksteps; ++ks) {
    const int stage = ks & 1;
    if (ks + 1 < ksteps) load_global(ks + 1);
    const unsigned char* a_t = smem + stage * STAGE_BYTES;
    const unsigned char* w_t = a_t + A_TILE_BYTES;
#pragma unroll
    for (int kk = 0; kk < kBK / 16; ++kk) {
      half8_t wf[TN], xf[TM];
      const int piece = kk * 2 + frag_half;
#pragma unroll
      for (int i = 0; i < TN; ++i) {
        int r = wave_n * WTN + i * 32 + frag_row;
        wf[i] = *reinterpret_cast<const half8_t*>(w_t + lds_off(r, piece));
      }
#pragma unroll
      for (int j = 0; j < TM; ++j) {
        int r = wave_m * WTM + j * 32 + frag_row;
        xf[j] = *reinterpret_cast<const half8_t*>(a_t + lds_off(r, piece));
      }
#pragma unroll
      for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wf[i], xf[j], acc[i][j], 0, 0, 0);
    }
    if (ks + 1 < ksteps) store_lds(stage ^ 1);
    __syncthreads();
  }

  // ---- epilogue: lane holds, per MFMA tile, column m = lane % 32 and rows
  // n = 8 * (r / 4) + 4 * (lane / 32) + r % 4
#pragma unroll
  for (int j = 0; j < TM; ++j) {
    const int m = m0 + wave_m * WTM + j * 32 + frag_row;
    if (m >= M) continue;
    const float am = a_mul[(int64_t)m * a_mul_stride];
#pragma unroll
    for (int i = 0; i < TN; ++i) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = n0 + wave_n * WTN + i * 32 + q * 8 + frag_half * 4;
        if (n >= N) continue;
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          int nn = n + e;
          float wm = (nn < N) ? w_mul[(int64_t)nn * w_mul_stride] : 0.0f;
          v[e] = acc[i][j][q * 4 + e] * (am * wm);
        }
        if constexpr (OUT_F32) {
          float* yo = reinterpret_cast<float*>(y) + (int64_t)m * ldy + n;
          if (n + 3 < N) {
            *reinterpret_cast<float4*>(yo) = make_float4(v[0], v[1], v[2], v[3]);
          } else {
            for (int e = 0; e < 4 && n + e < N; ++e) yo[e] = v[e];
          }
        } else {
          uint16_t* yo = reinterpret_cast<uint16_t*>(y) + (int64_t)m * ldy + n;
          uint32_t b0 = f32_to_bf16_rne(v[0]), b1 = f32_to_bf16_rne(v[1]);
          uint32_t b2 = f32_to_bf16_rne(v[2]), b3 = f32_to_bf16_rne(v[3]);
          if (n + 3 < N) {
            *reinterpret_cast<uint2*>(yo) = make_uint2(b0 | (b1 << 16), b2 | (b3 << 16));
          } else {
            uint32_t b[4] = {b0, b1, b2, b3};
            for (int e = 0; e < 4 && n + e < N; ++e) yo[e] = (uint16_t)b[e];
          }
        }
      }
    }
  }
}

// ------------------------------------------------------------------------ INT scale prepass
// One wave per row of scales: recover each group's bf16 maximum h = bf16_rne(s * Q), find the
// row's largest exponent, and emit fp16 h * 2^-E plus the fp32 epilogue factor 2^E / Q, with E
// chosen so that the largest Q * h * 2^-E stays below 2^15.
__global__ __launch_bounds__(256) void int_scale_prep_kernel(const float* __restrict__ s, int rows,
                                                             int groups, float Q,
                                                             uint16_t* __restrict__ h_out,
                                                             float* __restrict__ mul_out) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= rows) return;
  const float* sr = s + (int64_t)row * groups;
  float mx = 0.0f;
  for (int g = lane; g < groups; g += 64) {
    float h = as_f32(f32_to_bf16_rne(sr[g] * Q) << 16);
    mx = fmaxf(mx, h);
  }
  mx = wave_max(mx);
  // E = exponent(mx) - 11: the row maximum lands in [2^11, 2^12), times Q <= 7 stays < 2^15
  int e = (int)((as_u32(mx) >> 23) & 0xFF) - 127;
  if (mx == 0.0f) e = 0;
  int E = e - 11;
  // clamp so that both 2^-E and 2^E are normal fp32 numbers
  E = max(-120, min(120, E));
  const float down = as_f32((uint32_t)(127 - E) << 23);     // 2^-E
  const float up = as_f32((uint32_t)(127 + E) << 23);       // 2^E
  for (int g = lane; g < groups; g += 64) {
    float h = as_f32(f32_to_bf16_rne(sr[g] * Q) << 16);
    _Float16 hh = (_Float16)(h * down);                      // exact unless far below the row max
    h_out[(int64_t)row * groups + g] = __builtin_bit_cast(uint16_t, hh);
  }
  if (lane == 0) mul_out[row] = up / Q;
}

// ------------------------------------------------------------------------ host side
struct GemmWs {
  uint16_t* a_h;
  uint16_t* w_h;
  float* a_mul;
  float* w_mul;
};

static size_t carve_gemm(void* base, pq_format fmt, int group, int64_t M, int64_t N, int64_t K,
                         GemmWs* w) {
  if (fmt == PQ_FMT_NVFP4) return 0;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off = align_up(off + bytes, 256);
    return o;
  };
  size_t o_ah = take((size_t)M * (K / group) * 2);
  size_t o_wh = take((size_t)N * (K / group) * 2);
  size_t o_am = take((size_t)M * 4);
  size_t o_wm = take((size_t)N * 4);
  if (w) {
    char* b = (char*)base;
    w->a_h = (uint16_t*)(b + o_ah);
    w->w_h = (uint16_t*)(b + o_wh);
    w->a_mul = (float*)(b + o_am);
    w->w_mul = (float*)(b + o_wm);
  }
  return off;
}

size_t qgemm_workspace_bytes(pq_format fmt, int group, int64_t M, int64_t N, int64_t K) {
  return carve_gemm(nullptr, fmt, group, M, N, K, nullptr);
}

template <int FMT, int G, int BM, int BN, int WGM, int WGN, bool OUT_F32>
static int launch_gemm(const uint8_t* a_codes, ScaleSrc a_sc, const uint8_t* w_codes, ScaleSrc w_sc,
                       const float* a_mul, int a_stride, const float* w_mul, int w_stride, int M, int N,
                       int K, void* y, int64_t ldy, hipStream_t st) {
  constexpr int T = WGM * WGN * 64;
  constexpr size_t shmem = 2 * (size_t)(BM + BN) * kRowBytes;
  auto kern = qgemm_kernel<FMT, G, BM, BN, WGM, WGN, OUT_F32>;
  if (shmem > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
    if (e != hipSuccess) return check_hip(e, "hipFuncSetAttribute(qgemm_kernel)");
  }
  int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  int64_t n_tiles = (int64_t)tiles_m * tiles_n;
  if (n_tiles > 0x7FFFFFFF) return fail(PQ_ERR_SHAPE, "too many output tiles");
  hipLaunchKernelGGL(kern, dim3((unsigned)n_tiles), dim3(T), shmem, st, a_codes, a_sc, w_codes, w_sc, a_mul,
                     a_stride, w_mul, w_stride, M, N, K, y, ldy, tiles_m, tiles_n);
  return check_hip(hipGetLastError(), "qgemm_kernel");
}

template <int FMT, int G, bool OUT_F32>
static int pick_tile(const uint8_t* a_codes, ScaleSrc a_sc, const uint8_t* w_codes, ScaleSrc w_sc,
                     const float* a_mul, int a_stride, const float* w_mul, int w_stride, int M, int N,
                     int K, void* y, int64_t ldy, hipStream_t st) {
  // large tile when it still fills the 256 compute units, else the small one
  int64_t big_tiles = (int64_t)((M + 255) / 256) * ((N + 255) / 256);
  if (big_tiles >= 128)
    return launch_gemm<FMT, G, 256, 256, 2, 4, OUT_F32>(a_codes, a_sc, w_codes, w_sc, a_mul, a_stride,
                                                        w_mul, w_stride, M, N, K, y, ldy, st);
  return launch_gemm<FMT, G, 128, 128, 2, 2, OUT_F32>(a_codes, a_sc, w_codes, w_sc, a_mul, a_stride, w_mul,
                                                      w_stride, M, N, K, y, ldy, st);
}

template <int FMT, int G>
static int run_fmt(const uint8_t* a_codes, const void* a_scales, const float* a_ts,
                   const uint8_t* w_codes, const void* w_scales, const float* w_ts, int M, int N, int K,
                   void* y, int64_t ldy, bool out_f32, void* ws, hipStream_t st) {
  ScaleSrc a_sc{nullptr, nullptr}, w_sc{nullptr, nullptr};
  const float *a_mul, *w_mul;
  int a_stride, w_stride;
  if constexpr (FMT == kNvfp4) {
    a_sc.e4m3 = (const uint8_t*)a_scales;
    w_sc.e4m3 = (const uint8_t*)w_scales;
    a_mul = a_ts;
    w_mul = w_ts;
    a_stride = w_stride = 0;
  } else {
    GemmWs W;
    carve_gemm(ws, (pq_format)FMT, G, M, N, K, &W);
    const float Q = qmax_of(FMT);
    hipLaunchKernelGGL(int_scale_prep_kernel, dim3((unsigned)((M + 3) / 4)), dim3(256), 0, st,
                       (const float*)a_scales, M, K / G, Q, W.a_h, W.a_mul);
    hipLaunchKernelGGL(int_scale_prep_kernel, dim3((unsigned)((N + 3) / 4)), dim3(256), 0, st,
                       (const float*)w_scales, N, K / G, Q, W.w_h, W.w_mul);
    int rc = check_hip(hipGetLastError(), "int_scale_prep_kernel");
    if (rc) return rc;
    a_sc.f16 = W.a_h;
    w_sc.f16 = W.w_h;
    a_mul = W.a_mul;
    w_mul = W.w_mul;
    a_stride = w_stride = 1;
  }
  if (out_f32)
    return pick_tile<FMT, G, true>(a_codes, a_sc, w_codes, w_sc, a_mul, a_stride, w_mul, w_stride, M, N, K,
                                   y, ldy, st);
  return pick_tile<FMT, G, false>(a_codes, a_sc, w_codes, w_sc, a_mul, a_stride, w_mul, w_stride, M, N, K,
                                  y, ldy, st);
}

int run_qgemm(pq_format fmt, int group, const uint8_t* a_codes, const void* a_scales,
              const float* a_ts, const uint8_t* w_codes, const void* w_scales, const float* w_ts,
              int64_t M, int64_t N, int64_t K, void* y, int64_t ldy, bool out_f32, void* ws,
              hipStream_t st) {
#define PQ_ARGS a_codes, a_scales, a_ts, w_codes, w_scales, w_ts, (int)M, (int)N, (int)K, y, ldy, out_f32, ws, st
  if (fmt == PQ_FMT_NVFP4) return run_fmt<kNvfp4, 16>(PQ_ARGS);
  if (fmt == PQ_FMT_INT4) {
    switch (group) {
      case 32: return run_fmt<kInt4, 32>(PQ_ARGS);
      case 64: return run_fmt<kInt4, 64>(PQ_ARGS);
      case 128: return run_fmt<kInt4, 128>(PQ_ARGS);
      case 256: return run_fmt<kInt4, 256>(PQ_ARGS);
    }
  }
  if (fmt == PQ_FMT_INT3) {
    switch (group) {
      case 32: return run_fmt<kInt3, 32>(PQ_ARGS);
      case 64: return run_fmt<kInt3, 64>(PQ_ARGS);
      case 128: return run_fmt<kInt3, 128>(PQ_ARGS);
      case 256: return run_fmt<kInt3, 256>(PQ_ARGS);
    }
  }
#undef PQ_ARGS
  return fail(PQ_ERR_FORMAT, "unsupported (format, group) = (%d, %d)", (int)fmt, group);
}

}  // namespace pq
