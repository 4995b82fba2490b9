// The normalisation layer in front of a quantized linear layer with the channel reorder absorbed
// into it (paper App. C): RMSNorm, or LayerNorm followed by a per-sample scale and shift, emitting
// y_P[m, j] = y[m, pi(j)] as a bf16 tensor, as the activation operand of the GEMM (the dynamic
// quantizer of Eq. 1-2 applied to those bf16 values), or both.
//
// One wave owns one token row from load to store, so no step waits for another wave:
//   1. the row is read as it lies in memory (16 bytes per lane and access, whole lines), its sum
//      and sum of squares come from v_dot2c_f32_bf16 on the packed pairs, and it is parked in the
//      wave's own slab of LDS;
//   2. lane l then produces chunks l, l + 64, ... (8 consecutive positions j each) of the reordered
//      row: it loads pi(j) for its positions and gathers x[pi(j)] from the slab with 2-byte LDS
//      reads -- where the paper's kernel issues indexed global loads -- normalises, applies the
//      channel-wise vectors and rounds to bf16;
//   3. the bf16 chunk is stored (consecutive lanes, consecutive 16 bytes) and / or quantized: a
//      group of G positions is G / 8 consecutive lanes, so the group maximum is a lane reduction
//      and the per-row power of two of the INT operand layout a wave reduction.
// The channel-wise vectors are shared by the rows of a workgroup: they are staged in LDS already
// reordered (position j holds the value of channel pi(j)) once per workgroup, which is the only
// step all waves wait for.
//
// The same skeleton runs the Hadamard variant (paper App. D, x H P): step 1 becomes a fast
// Hadamard transform of the row in the wave's slab (fp32), steps 2 and 3 read the transformed
// row at pi(j) -- the reorder is the order in which the transform's output is consumed.
#include <math.h>

#include <algorithm>

#include "pq_qgemm_common.h"

namespace pq {

namespace {

enum Norm : int { kNormRms = 0, kNormAdaLn = 1, kHadamard = 2 };
constexpr int kFmtNone = -1;                  // normalise and reorder only, no quantization
constexpr int kNormMaxWaves = 8;

struct NormArgs {
  const int32_t* perm;          // pi, or null for the identity
  const uint16_t* gamma;        // RMSNorm: bf16 [K], or null for ones
  const uint16_t* mod_scale;    // AdaLN: bf16 [n_mod][K] s (the factor is 1 + s), or null for zeros
  const uint16_t* mod_shift;    // AdaLN: bf16 [n_mod][K] b, or null for zeros
  int64_t rows_per_mod;         // token row m uses modulation row m / rows_per_mod
  float eps;
  uint16_t* y;                  // bf16 [rows][ldy] normalised, reordered output, or null
  int64_t ldy;
  int rows_seq;                 // rows a team of waves takes one after the other (wide rows)
  int had_pow2, had_m;          // Hadamard: K = had_pow2 * had_m, had_m in {1, 12, 20}
  float had_scale;              // 1 / sqrt(K)
};

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float wave_sum_f32(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

__device__ __forceinline__ uint32_t pack_bf16_rne(float lo, float hi) {
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  return __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2_t){lo, hi}, bf16x2_t));
}

struct Idx8 {
  int4 lo, hi;
};


// ---- fast Hadamard transform of one row held in LDS as fp32, by one wave -------------------
// H = S_{2^k} (x) P_m / sqrt(K), channel i = a * m + b (a: Sylvester index, natural order; b: Paley
// index).  Kronecker factors act on separate index digits, so the transform is a sequence of
// passes, each applying a small matrix along one digit: every lane takes whole fibres (all elements
// that differ only in that digit), transforms them in registers and writes them back.

// between passes: the wave's LDS writes are complete and visible to its other lanes
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// A row is worked on by a team of TEAM waves: one wave, which only has to order its own LDS
// traffic, or (wide rows) all waves of the workgroup, which meet at a workgroup barrier.
template <int TEAM>
__device__ __forceinline__ void team_sync() {
  if constexpr (TEAM == 1) wave_lds_sync();
  else __syncthreads();
}

// Sylvester matrix of order R along a digit of weight `inner` elements; n_fibres = K / R
template <int R, int TEAM>
__device__ __forceinline__ void sylvester_pass(float* slab, int inner, int n_fibres, int lane) {
  // f / inner through a float reciprocal: f < 2^13 and the quotient's fractional part is at least
  // 1 / (2 inner) away from an integer, far more than the rounding error of the product
  const float inv_inner = 1.0f / (float)inner;
  for (int f = lane; f < n_fibres; f += 64 * TEAM) {
    const int hi = (int)(((float)f + 0.5f) * inv_inner), lo = f - hi * inner;
    float* base = slab + hi * (R * inner) + lo;
    float v[R];
#pragma unroll
    for (int t = 0; t < R; ++t) v[t] = base[t * inner];
#pragma unroll
    for (int h = 1; h < R; h <<= 1)
#pragma unroll
      for (int i = 0; i < R; i += 2 * h)
#pragma unroll
        for (int j = i; j < i + h; ++j) {
          const float a = v[j], b = v[j + h];
          v[j] = a + b;
          v[j + h] = a - b;
        }
#pragma unroll
    for (int t = 0; t < R; ++t) base[t * inner] = v[t];
  }
  team_sync<TEAM>();
}

// quadratic character mod Q (Q prime): +1 for a non-zero square, -1 otherwise, 0 for 0
template <int Q>
__host__ __device__ constexpr int legendre(int r) {
  r = ((r % Q) + Q) % Q;
  if (r == 0) return 0;
  for (int t = 1; t < Q; ++t)
    if ((t * t) % Q == r) return 1;
  return -1;
}

// entry (b, b2) of the Paley type I Hadamard matrix of order M = Q + 1:  I + [[0, 1^T], [-1, chi(i - j)]]
template <int M>
__host__ __device__ constexpr int paley_entry(int b, int b2) {
  if (b == b2) return 1;
  if (b == 0) return 1;
  if (b2 == 0) return -1;
  return legendre<M - 1>((b - 1) - (b2 - 1));
}

// y[b2] = sum_b x[b] P[b][b2] along the last digit (M contiguous elements per fibre)
template <int M, int TEAM>
__device__ __forceinline__ void paley_pass(float* slab, int n_fibres, int lane) {
  for (int f = lane; f < n_fibres; f += 64 * TEAM) {
    float* base = slab + f * M;
    float v[M], o[M];
#pragma unroll
    for (int b = 0; b < M; ++b) v[b] = base[b];
    // a pair of inputs enters every output as +-(v0 + v1) or +-(v0 - v1): form both once, then each
    // output is a signed sum of M / 2 terms instead of M
    float sum[M / 2], dif[M / 2];
#pragma unroll
    for (int j = 0; j < M / 2; ++j) {
      sum[j] = v[2 * j] + v[2 * j + 1];
      dif[j] = v[2 * j] - v[2 * j + 1];
    }
#pragma unroll
    for (int b2 = 0; b2 < M; ++b2) {
      float acc = 0.0f;
#pragma unroll
      for (int j = 0; j < M / 2; ++j) {
        const int s0 = paley_entry<M>(2 * j, b2), s1 = paley_entry<M>(2 * j + 1, b2);
        const float term = s0 == s1 ? sum[j] : dif[j];
        acc = s0 > 0 ? acc + term : acc - term;
      }
      o[b2] = acc;
    }
#pragma unroll
    for (int b = 0; b < M; ++b) base[b] = o[b];
  }
  team_sync<TEAM>();
}

// The Paley pass of order 12 on the matrix unit, straight from the bf16 row in memory into the fp32 slab:
// sixteen fibres (16 x 12 contiguous values) times P_12 padded to 16 x 16 is one v_mfma_f32_16x16x16_bf16.
// Inputs and the +-1 entries are exact in bf16 and the products are accumulated in fp32, as on the
// vector unit.  Operand layout of the instruction: lane l holds A[l % 16][4 (l / 16) + i] (a fibre's
// values 4j .. 4j + 3: eight contiguous bytes), B[4 (l / 16) + i][l % 16] and D[4 (l / 16) + i][l % 16].
// negative entries of rows 4j .. 4j + 3 of P_12: bit 16 i + n for entry (4j + i, n)
constexpr uint64_t paley12_negatives(int j) {
  uint64_t mask = 0;
  for (int i = 0; i < 4; ++i)
    for (int n = 0; n < 12; ++n)
      if (paley_entry<12>(4 * j + i, n) < 0) mask |= (uint64_t)1 << (16 * i + n);
  return mask;
}
template <int TEAM>
__device__ __forceinline__ void paley12_pass_from_memory(const uint16_t* __restrict__ xr, float* slab, int n_fibres,
                                                         int tl) {
  typedef short bf16x4_bits __attribute__((ext_vector_type(4)));
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  const int lane = tl & 63, wv = tl >> 6;
  const int n = lane & 15, j = lane >> 4;
  constexpr uint64_t kNeg0 = paley12_negatives(0), kNeg1 = paley12_negatives(1), kNeg2 = paley12_negatives(2);
  const uint64_t neg = j == 0 ? kNeg0 : j == 1 ? kNeg1 : kNeg2;
  const bool in_matrix = j < 3 && n < 12;                    // the padding rows and columns are zero
  uint32_t bw[2];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const uint32_t e0 = ((neg >> (32 * h + n)) & 1) ? 0xBF80u : 0x3F80u;
    const uint32_t e1 = ((neg >> (32 * h + 16 + n)) & 1) ? 0xBF80u : 0x3F80u;
    bw[h] = in_matrix ? (e0 | (e1 << 16)) : 0u;
  }
  const bf16x4_bits b = __builtin_bit_cast(bf16x4_bits, make_uint2(bw[0], bw[1]));
  const int groups = n_fibres / 16;
  constexpr int kInFlight = 8;
  for (int g0 = wv; g0 < groups; g0 += TEAM * kInFlight) {
    uint2 a[kInFlight];
#pragma unroll
    for (int t = 0; t < kInFlight; ++t) {
      const int g = g0 + t * TEAM;
      a[t] = make_uint2(0u, 0u);
      if (g < groups && j < 3) a[t] = *reinterpret_cast<const uint2*>(xr + (size_t)(g * 16 + n) * 12 + 4 * j);
    }
#pragma unroll
    for (int t = 0; t < kInFlight; ++t) {
      const int g = g0 + t * TEAM;
      if (g >= groups) break;                                // wave-uniform
      const f32x4 d = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(bf16x4_bits, a[t]), b,
                                                                (f32x4){0.0f, 0.0f, 0.0f, 0.0f}, 0, 0, 0);
      if (n < 12) {
        float* out = slab + (size_t)(g * 16 + 4 * j) * 12 + n;
        out[0] = d[0];
        out[12] = d[1];
        out[24] = d[2];
        out[36] = d[3];
      }
    }
  }
  team_sync<TEAM>();
}

// `lane` is the thread's index inside its team (0 .. 64 TEAM - 1); paley_done: the Paley pass has been applied
template <int TEAM>
__device__ __forceinline__ void hadamard_row(float* slab, int K, int pow2, int m, int lane, bool paley_done = false) {
  if (m == 12 && !paley_done) paley_pass<12, TEAM>(slab, pow2, lane);
  if (m == 20) paley_pass<20, TEAM>(slab, pow2, lane);
  int inner = m;                       // weight of the current Sylvester digit, in elements
  int rem = pow2;
  while (rem >= 16) {
    sylvester_pass<16, TEAM>(slab, inner, K / 16, lane);
    inner *= 16;
    rem /= 16;
  }
  if (rem == 8) sylvester_pass<8, TEAM>(slab, inner, K / 8, lane);
  if (rem == 4) sylvester_pass<4, TEAM>(slab, inner, K / 4, lane);
  if (rem == 2) sylvester_pass<2, TEAM>(slab, inner, K / 2, lane);
}

template <int FMT, int G, int NORM, int TEAM>
__global__ __launch_bounds__(64 * kNormMaxWaves) void norm_rows_kernel(
    const uint16_t* __restrict__ x, int64_t rows, int64_t K, int64_t ld, const float* __restrict__ tensor_scale,
    int64_t steps, int64_t units, uint8_t* __restrict__ p_codes, uint16_t* __restrict__ p_scales,
    float* __restrict__ p_mul, NormArgs na) {
  constexpr bool QUANT = FMT != kFmtNone;
  constexpr bool IS_INT = FMT == kInt4 || FMT == kInt3;
  constexpr int LPG = G / 8;                                 // lanes that share a group
  // chunks a lane works on at a time (AdaLN holds more per chunk: two keep it at five waves per SIMD)
  constexpr int kBatch = NORM == kNormAdaLn ? 2 : 3;
  static_assert(LPG >= 1 && LPG <= 64, "a group lies inside one wave-wide run of chunks");
  // dynamic LDS: [vectors: K bf16 (RMSNorm) or K words (AdaLN)] [per row: K bf16 (Hadamard: fp32) slab]
  //              [per row, INT: `units` fp32 group maxima] [per wave: 4 floats for team reductions]
  // TEAM == 1: every wave owns a row.  TEAM > 1: the workgroup is one team of TEAM waves and owns one row.
  constexpr int TL = 64 * TEAM;                              // threads of a team
  extern __shared__ __align__(16) unsigned char lds_raw[];
  const int tid = threadIdx.x, lane = tid & 63, n_waves = blockDim.x >> 6;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int tl = TEAM == 1 ? lane : tid;                     // index inside the team
  const int slot = TEAM == 1 ? wave : 0;                     // row slot inside the workgroup
  const int rows_per_wg = TEAM == 1 ? n_waves : 1;
  const int Ki = (int)K;
  const int k_chunks = Ki / 8;                               // chunks that exist
  const int n_chunks = (int)steps * 8;                       // chunks the panel holds (a half step past K included)
  const int n_units = (int)units;
  // TEAM > 1: the workgroup takes na.rows_seq consecutive rows one after the other, so that the vectors
  // are staged once for all of them
  const int rows_seq = TEAM == 1 ? 1 : na.rows_seq;
  const int64_t row0 = (int64_t)blockIdx.x * (TEAM == 1 ? rows_per_wg : rows_seq);

  uint16_t* vec_g = reinterpret_cast<uint16_t*>(lds_raw);
  uint32_t* vec_sb = reinterpret_cast<uint32_t*>(lds_raw);
  constexpr int kSlabElem = NORM == kHadamard ? 4 : 2;       // Hadamard rows are held as fp32
  const size_t vec_bytes = NORM == kHadamard ? 0 : (size_t)Ki * (NORM == kNormRms ? 2 : 4);
  uint16_t* slab = reinterpret_cast<uint16_t*>(lds_raw + vec_bytes) + (size_t)slot * Ki;
  float* slab_f = reinterpret_cast<float*>(lds_raw + vec_bytes) + (size_t)slot * Ki;
  const size_t slab_bytes = (size_t)rows_per_wg * Ki * kSlabElem;
  float* h_lds = reinterpret_cast<float*>(lds_raw + vec_bytes + slab_bytes) + (size_t)slot * n_units;
  float* team_red = reinterpret_cast<float*>(lds_raw + vec_bytes + slab_bytes) + (size_t)(IS_INT ? rows_per_wg * n_units : 0);
  // sum / maximum over the team, the same value in every thread (fixed order of the waves)
  auto team_sum = [&](float v) -> float {
    v = wave_sum_f32(v);
    if constexpr (TEAM > 1) {
      if (lane == 0) team_red[wave] = v;
      __syncthreads();
      float t = 0.0f;
#pragma unroll
      for (int w = 0; w < TEAM; ++w) t += team_red[w];
      __syncthreads();
      v = t;
    }
    return v;
  };
  auto team_max = [&](float v) -> float {
    v = wave_max(v);
    if constexpr (TEAM > 1) {
      if (lane == 0) team_red[wave] = v;
      __syncthreads();
      float t = 0.0f;
#pragma unroll
      for (int w = 0; w < TEAM; ++w) t = fmaxf(t, team_red[w]);
      __syncthreads();
      v = t;
    }
    return v;
  };

  // ---- the vectors of the first row's sample, reordered, into LDS (all threads).  Scattered
  // 2-byte loads from memory cost the texture addresser a cycle per lane, so the vectors are first
  // copied as they lie (whole lines) into the space of the row slabs, which is still free, and
  // reordered from there with LDS reads, one vector at a time.
  int64_t mod0 = 0;
  if constexpr (NORM == kNormAdaLn) mod0 = row0 / na.rows_per_mod;
  if constexpr (NORM != kHadamard) {
    const uint16_t* v0 = NORM == kNormRms ? na.gamma : (na.mod_scale ? na.mod_scale + mod0 * K : nullptr);
    const uint16_t* v1 = NORM == kNormRms ? nullptr : (na.mod_shift ? na.mod_shift + mod0 * K : nullptr);
    constexpr uint32_t kDefault0 = NORM == kNormRms ? 0x3F80u : 0u;      // gamma = 1, s = 0
    uint16_t* tmp = reinterpret_cast<uint16_t*>(lds_raw + vec_bytes);    // the slab space: at least 2 K bytes
    // one vector at a time: copy as it lies, barrier, permuted read
    auto permuted = [&](const uint16_t* v, int c, uint32_t dflt, uint32_t (&out)[8]) {
      if (!v) {
#pragma unroll
        for (int e = 0; e < 8; ++e) out[e] = dflt;
        return;
      }
      if (na.perm) {
        const int4 i0 = *reinterpret_cast<const int4*>(na.perm + (size_t)c * 8);
        const int4 i1 = *reinterpret_cast<const int4*>(na.perm + (size_t)c * 8 + 4);
        const int idx[8] = {i0.x, i0.y, i0.z, i0.w, i1.x, i1.y, i1.z, i1.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) out[e] = tmp[idx[e]];
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) out[e] = tmp[c * 8 + e];
      }
    };
    if (v0) {
      for (int c = tid; c < k_chunks; c += blockDim.x)
        *reinterpret_cast<uint4*>(tmp + c * 8) = *reinterpret_cast<const uint4*>(v0 + (size_t)c * 8);
    }
    __syncthreads();
    for (int c = tid; c < k_chunks; c += blockDim.x) {
      uint32_t a0[8];
      permuted(v0, c, kDefault0, a0);
      if constexpr (NORM == kNormRms) {
        *reinterpret_cast<uint4*>(vec_g + c * 8) = make_uint4(a0[0] | (a0[1] << 16), a0[2] | (a0[3] << 16),
                                                               a0[4] | (a0[5] << 16), a0[6] | (a0[7] << 16));
      } else {
        *reinterpret_cast<uint4*>(vec_sb + c * 8) = make_uint4(a0[0], a0[1], a0[2], a0[3]);
        *reinterpret_cast<uint4*>(vec_sb + c * 8 + 4) = make_uint4(a0[4], a0[5], a0[6], a0[7]);
      }
    }
    if constexpr (NORM == kNormAdaLn) {
      if (v1) {                              // uniform over the workgroup
        __syncthreads();
        for (int c = tid; c < k_chunks; c += blockDim.x)
          *reinterpret_cast<uint4*>(tmp + c * 8) = *reinterpret_cast<const uint4*>(v1 + (size_t)c * 8);
        __syncthreads();
        for (int c = tid; c < k_chunks; c += blockDim.x) {      // the chunks this thread wrote above
          uint32_t a1[8];
          permuted(v1, c, 0u, a1);
          uint4 q0 = *reinterpret_cast<uint4*>(vec_sb + c * 8), q1 = *reinterpret_cast<uint4*>(vec_sb + c * 8 + 4);
          q0.x |= a1[0] << 16; q0.y |= a1[1] << 16; q0.z |= a1[2] << 16; q0.w |= a1[3] << 16;
          q1.x |= a1[4] << 16; q1.y |= a1[5] << 16; q1.z |= a1[6] << 16; q1.w |= a1[7] << 16;
          *reinterpret_cast<uint4*>(vec_sb + c * 8) = q0;
          *reinterpret_cast<uint4*>(vec_sb + c * 8 + 4) = q1;
        }
      }
    }
  }
  __syncthreads();                       // the last barrier; every wave reaches it (the slabs are free again)
  if (TEAM == 1 && row0 + slot >= rows) return;      // wave-uniform; a team stays together to the end

  // indices pi(j) of chunk c (clamped to an existing chunk: the address is always valid)
  auto load_idx = [&](int c) -> Idx8 {
    const int cc = min(c, k_chunks - 1);
    Idx8 ix;
    if (na.perm) {
      ix.lo = *reinterpret_cast<const int4*>(na.perm + (size_t)cc * 8);
      ix.hi = *reinterpret_cast<const int4*>(na.perm + (size_t)cc * 8 + 4);
    } else {
      ix.lo = make_int4(cc * 8, cc * 8 + 1, cc * 8 + 2, cc * 8 + 3);
      ix.hi = make_int4(cc * 8 + 4, cc * 8 + 5, cc * 8 + 6, cc * 8 + 7);
    }
    return ix;
  };
  const float k_f = (float)Ki;
  float T = 0.0f, encT = 0.0f;
  if constexpr (FMT == kNvfp4) {
    T = *tensor_scale;
    encT = nv4_enc_scale(T);
  }
  const int n_iter = (n_chunks + TL - 1) / TL;

  for (int ri = 0; ri < rows_seq; ++ri) {
  const int64_t row_u = TEAM == 1 ? row0 + slot : row0 + ri;
  const bool active = row_u < rows;                          // a team runs past the last row without storing
  const int64_t row = active ? row_u : rows - 1;
  // the first batch of indices does not depend on the row's values
  Idx8 ix_cur[kBatch];
#pragma unroll
  for (int q = 0; q < kBatch; ++q) ix_cur[q] = load_idx(tl + TL * q);

  const uint16_t* xr = x + row * ld;
  float rstd = 0.0f, nmr = 0.0f;                             // LN(x) = x * rstd + nmr
  if constexpr (NORM == kHadamard) {
    // ---- 1. the row as fp32 in the wave's slab, transformed in place
    constexpr int kInFlight = 8;
    const bool paley_on_mfma = na.had_m == 12 && na.had_pow2 >= 16;      // uniform
    if (paley_on_mfma) paley12_pass_from_memory<TEAM>(xr, slab_f, na.had_pow2, tl);
    for (int c0 = 0; c0 < (paley_on_mfma ? 0 : k_chunks); c0 += kInFlight * TL) {
      uint4 lines[kInFlight];
#pragma unroll
      for (int t = 0; t < kInFlight; ++t) {
        const int c = min(c0 + t * TL + tl, k_chunks - 1);
        lines[t] = *reinterpret_cast<const uint4*>(xr + (size_t)c * 8);
      }
#pragma unroll
      for (int t = 0; t < kInFlight; ++t) {
        const int c = c0 + t * TL + tl;
        if (c < k_chunks) {
          const uint4 p = lines[t];
          *reinterpret_cast<float4*>(slab_f + c * 8) = make_float4(bf16_lo(p.x), bf16_hi(p.x), bf16_lo(p.y), bf16_hi(p.y));
          *reinterpret_cast<float4*>(slab_f + c * 8 + 4) = make_float4(bf16_lo(p.z), bf16_hi(p.z), bf16_lo(p.w), bf16_hi(p.w));
        }
      }
    }
    team_sync<TEAM>();
    hadamard_row<TEAM>(slab_f, Ki, na.had_pow2, na.had_m, tl, paley_on_mfma);
    rstd = na.had_scale;
  } else {
  // ---- 1. the row: statistics, and a copy in the wave's slab
  float s1 = 0.0f, s2 = 0.0f;
  {
    const bf16x2_t ones = __builtin_bit_cast(bf16x2_t, 0x3F803F80u);
    constexpr int kInFlight = 8;                            // lines per lane requested together
    for (int c0 = 0; c0 < k_chunks; c0 += kInFlight * TL) {
      uint4 lines[kInFlight];
#pragma unroll
      for (int t = 0; t < kInFlight; ++t) {
        const int c = min(c0 + t * TL + tl, k_chunks - 1);
        lines[t] = *reinterpret_cast<const uint4*>(xr + (size_t)c * 8);
      }
#pragma unroll
      for (int t = 0; t < kInFlight; ++t) {
        const int c = c0 + t * TL + tl;
        if (c < k_chunks) {
          *reinterpret_cast<uint4*>(slab + c * 8) = lines[t];
          const uint32_t d[4] = {lines[t].x, lines[t].y, lines[t].z, lines[t].w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const bf16x2_t v = __builtin_bit_cast(bf16x2_t, d[e]);
            if constexpr (NORM == kNormAdaLn) s1 = __builtin_amdgcn_fdot2_f32_bf16(v, ones, s1, false);
            s2 = __builtin_amdgcn_fdot2_f32_bf16(v, v, s2, false);
          }
        }
      }
    }
  }
  s2 = team_sum(s2);                     // (with TEAM > 1 also the barrier after the slab writes)
  float mean = 0.0f;
  if constexpr (NORM == kNormAdaLn) {
    mean = team_sum(s1) / k_f;
    // variance = mean square - mean^2 loses accuracy when the mean dominates; then (rare, uniform
    // over the wave) it is recomputed from the deviations, on the lane's own chunks in LDS
    const float mean_sq = s2 / k_f;
    const float var = mean_sq - mean * mean;
    if (mean_sq > 16.0f * var) {
      float s3 = 0.0f;
      for (int c = tl; c < k_chunks; c += TL) {
        const uint4 p = *reinterpret_cast<const uint4*>(slab + c * 8);
        const uint32_t d[4] = {p.x, p.y, p.z, p.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float lo = bf16_lo(d[e]) - mean, hi = bf16_hi(d[e]) - mean;
          s3 = fmaf(hi, hi, fmaf(lo, lo, s3));
        }
      }
      s2 = team_sum(s3);
    } else {
      s2 = var * k_f;
    }
  }
  rstd = 1.0f / sqrtf(s2 / k_f + na.eps);
  nmr = -mean * rstd;
  }

  // AdaLN: a row of another sample than the staged one reads its vectors from memory
  bool own_mod = false;
  const uint16_t* g_scale = nullptr;
  const uint16_t* g_shift = nullptr;
  if constexpr (NORM == kNormAdaLn) {
    const int64_t mod = row / na.rows_per_mod;
    own_mod = mod != mod0;                                   // wave-uniform
    g_scale = na.mod_scale ? na.mod_scale + mod * K : nullptr;
    g_shift = na.mod_shift ? na.mod_shift + mod * K : nullptr;
  }

  float row_max = 0.0f;
  uint16_t* y_row = na.y ? na.y + row * na.ldy : nullptr;

  // ---- 2./3. chunks lane, lane + 64, ... of the reordered row, kBatch at a time
  for (int it0 = 0; it0 < n_iter; it0 += kBatch) {
    // next batch's indices while this one is worked on
    Idx8 ix_next[kBatch];
#pragma unroll
    for (int q = 0; q < kBatch; ++q) ix_next[q] = load_idx(tl + TL * (it0 + kBatch + q));
    // gathers of the whole batch in flight together
    float xv[kBatch][8];
#pragma unroll
    for (int q = 0; q < kBatch; ++q) {
      const int idx[8] = {ix_cur[q].lo.x, ix_cur[q].lo.y, ix_cur[q].lo.z, ix_cur[q].lo.w,
                          ix_cur[q].hi.x, ix_cur[q].hi.y, ix_cur[q].hi.z, ix_cur[q].hi.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) xv[q][e] = NORM == kHadamard ? slab_f[idx[e]] : bf16_to_f32(slab[idx[e]]);
    }
#pragma unroll
    for (int q = 0; q < kBatch; ++q) {
      const int c = tl + TL * (it0 + q);
      if (it0 + q >= n_iter) break;                          // wave-uniform
      const bool in_row = c < k_chunks;
      const int cc = min(c, k_chunks - 1);
      float yv[8];
      if constexpr (NORM == kHadamard) {
#pragma unroll
        for (int e = 0; e < 8; ++e) yv[e] = xv[q][e] * rstd;             // 1 / sqrt(K)
      } else if constexpr (NORM == kNormRms) {
        const uint4 gq = *reinterpret_cast<const uint4*>(vec_g + cc * 8);
        const uint32_t gw[4] = {gq.x, gq.y, gq.z, gq.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          yv[2 * e] = (xv[q][2 * e] * rstd) * bf16_lo(gw[e]);
          yv[2 * e + 1] = (xv[q][2 * e + 1] * rstd) * bf16_hi(gw[e]);
        }
      } else {
        uint32_t sb[8];
        if (own_mod) {
          const int idx[8] = {ix_cur[q].lo.x, ix_cur[q].lo.y, ix_cur[q].lo.z, ix_cur[q].lo.w,
                              ix_cur[q].hi.x, ix_cur[q].hi.y, ix_cur[q].hi.z, ix_cur[q].hi.w};
#pragma unroll
          for (int e = 0; e < 8; ++e)
            sb[e] = (g_scale ? (uint32_t)g_scale[idx[e]] : 0u) | (g_shift ? (uint32_t)g_shift[idx[e]] << 16 : 0u);
        } else {
          const uint4 q0 = *reinterpret_cast<const uint4*>(vec_sb + cc * 8);
          const uint4 q1 = *reinterpret_cast<const uint4*>(vec_sb + cc * 8 + 4);
          sb[0] = q0.x; sb[1] = q0.y; sb[2] = q0.z; sb[3] = q0.w;
          sb[4] = q1.x; sb[5] = q1.y; sb[6] = q1.z; sb[7] = q1.w;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float ln = fmaf(xv[q][e], rstd, nmr);
          yv[e] = fmaf(bf16_lo(sb[e]), ln, bf16_hi(sb[e])) + ln;       // (1 + s) ln + b
        }
      }
      uint4 yb = make_uint4(pack_bf16_rne(yv[0], yv[1]), pack_bf16_rne(yv[2], yv[3]),
                            pack_bf16_rne(yv[4], yv[5]), pack_bf16_rne(yv[6], yv[7]));
      if (!in_row) yb = make_uint4(0u, 0u, 0u, 0u);          // the half step past K holds zeros
      if (y_row && in_row && active) *reinterpret_cast<uint4*>(y_row + (size_t)c * 8) = yb;

      if constexpr (QUANT) {
        // the quantizer of pq_quantize.hip on the rounded values
        float v[8] = {bf16_lo(yb.x), bf16_hi(yb.x), bf16_lo(yb.y), bf16_hi(yb.y),
                      bf16_lo(yb.z), bf16_hi(yb.z), bf16_lo(yb.w), bf16_hi(yb.w)};
        float a = 0.0f;
#pragma unroll
        for (int j = 0; j < 8; ++j) a = fmaxf(a, fabsf(v[j]));
        a = group_max<LPG>(a);
        uint32_t codes;
        if constexpr (FMT == kNvfp4) {
          const Nv4Scale sc = nv4_scale(a, T, encT);
          codes = 0;
          codes = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(codes, v[0] * sc.inv, v[1] * sc.inv, 1.0f, 0);
          codes = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(codes, v[2] * sc.inv, v[3] * sc.inv, 1.0f, 1);
          codes = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(codes, v[4] * sc.inv, v[5] * sc.inv, 1.0f, 2);
          codes = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(codes, v[6] * sc.inv, v[7] * sc.inv, 1.0f, 3);
          // a scale unit is the two bytes of 32 positions = four lanes; the first lane of the quad
          // collects the byte of the second pair
          const uint32_t other = dpp_u32<0x4E>(sc.byte);         // lane ^ 2
          const int u = c >> 2;
          if ((lane & 3) == 0 && u < n_units && active) p_scales[(int64_t)u * rows + row] = (uint16_t)(sc.byte | (other << 8));
        } else {
          constexpr int FI = IS_INT ? FMT : kInt4;
          const IntScale sc = int_scale<FI>(a);
          codes = int_codes8(v, sc.inv);
          row_max = fmaxf(row_max, a);
          const int g = c / LPG;
          if (lane % LPG == 0 && g < n_units) h_lds[g] = a;
        }
        if (c < n_chunks && active) *reinterpret_cast<uint32_t*>(p_codes + ((int64_t)(c >> 3) * rows + row) * 32 + (c & 7) * 4) = codes;
      }
    }
#pragma unroll
    for (int q = 0; q < kBatch; ++q) ix_cur[q] = ix_next[q];
  }

  if constexpr (IS_INT) {
    // the per-row power of two of the operand layout: E = exponent(row maximum) - 10 puts the
    // largest group maximum in [2^10, 2^11) (see pack_operand_kernel); scale units are the fp16
    // group maxima times 2^-E, the row factor 2^E / Q
    constexpr float Q = qmax_of(FMT);
    const float mx = team_max(row_max);    // (with TEAM > 1 also the barrier after the h_lds writes)
    int e = (int)((as_u32(mx) >> 23) & 0xFF) - 127;
    if (mx == 0.0f) e = 0;
    const int E = max(-120, min(120, e - 10));
    const float down = as_f32((uint32_t)(127 - E) << 23);
    if (tl == 0 && active) p_mul[row] = as_f32((uint32_t)(127 + E) << 23) / Q;
    for (int u = tl; u < n_units; u += TL) {         // the team's own LDS writes, ordered above
      const _Float16 hn = (_Float16)(h_lds[u] * down);
      if (active) p_scales[(int64_t)u * rows + row] = __builtin_bit_cast(uint16_t, hn);
    }
  }
  if constexpr (TEAM > 1) __syncthreads();     // the slab and the group maxima are free for the next row
  }  // rows of the workgroup
}

constexpr size_t kNormLdsLimit = 160 * 1024 - 1024;      // dynamic LDS a workgroup may ask for

// rows: row slabs of the workgroup (= waves when every wave owns a row, 1 for a team of waves)
size_t norm_lds_bytes(int norm, bool is_int, int rows_per_wg, int n_waves, int64_t K, int64_t units) {
  const size_t tail = (is_int ? (size_t)rows_per_wg * units * 4 : 0) + (size_t)n_waves * 16;
  if (norm == kHadamard) return (size_t)rows_per_wg * K * 4 + tail;
  return (size_t)K * (norm == kNormRms ? 2 : 4) + (size_t)rows_per_wg * K * 2 + tail;
}

// Waves (= rows) per workgroup: as many as still let the launch run in one round of resident
// workgroups, so that the reordered vectors are built as rarely as possible without leaving a
// tail of workgroups that start when the others are done.  How many workgroups of a given size a
// compute unit holds (registers, LDS, wave slots) is asked of the runtime.
template <typename Kern>
int norm_waves_per_group(Kern kern, int norm, bool is_int, int64_t rows, int64_t K, int64_t units) {
  int best = 1;
  double best_cost = 1e30;
  for (int w = 1; w <= kNormMaxWaves; ++w) {
    const size_t lds = norm_lds_bytes(norm, is_int, w, w, K, units);
    if (lds > kNormLdsLimit) break;
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, 64 * w, lds) != hipSuccess || per_cu < 1)
      per_cu = 1;
    const int64_t groups = (rows + w - 1) / w;
    const int64_t rounds = (groups + 256 * (int64_t)per_cu - 1) / (256 * (int64_t)per_cu);
    // time ~ rounds x (row work + vector staging shared by w rows), in units of one row's work;
    // among equal costs prefer more waves in flight per compute unit
    const double cost = (double)rounds * (1.0 + 0.35 / w) - 1e-3 * (double)std::min(per_cu * w, 32);
    if (cost < best_cost) best_cost = cost, best = w;
  }
  return best;
}

constexpr int kWideTeam = 4;             // waves that share a row wider than kWideRow channels
constexpr int64_t kWideRow = 4096;

template <int FMT, int G, int NORM, int TEAM>
int launch_norm_team(const void* x, int64_t rows, int64_t K, int64_t ld, const float* ts, const OperandLayout& L,
                     uint8_t* operand, const NormArgs& na, hipStream_t st) {
  constexpr bool is_int = FMT == kInt4 || FMT == kInt3;
  const size_t least = norm_lds_bytes(NORM, is_int, 1, TEAM, K, L.units);
  if (least > kNormLdsLimit)
    return fail(PQ_ERR_SHAPE, "K=%lld needs %zu bytes of LDS for one row and the vectors, more than the %zu available",
                (long long)K, least, kNormLdsLimit);
  auto kern = norm_rows_kernel<FMT, G, NORM, TEAM>;
  // the choice depends on the shape only: remembered from the previous launch of this kernel
  static thread_local struct { int64_t rows, K; int n_waves; } memo = {0, 0, 0};
  if (memo.rows != rows || memo.K != K) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)kNormLdsLimit);
    if (e != hipSuccess) return check_hip(e, "hipFuncSetAttribute(norm_rows_kernel)");
    memo.n_waves = TEAM == 1 ? norm_waves_per_group(kern, NORM, is_int, rows, K, L.units) : TEAM;
    memo.rows = rows;
    memo.K = K;
  }
  const int n_waves = memo.n_waves;
  const int rows_per_wg = TEAM == 1 ? n_waves : 1;
  const size_t shmem = norm_lds_bytes(NORM, is_int, rows_per_wg, n_waves, K, L.units);
  NormArgs args = na;
  // a team takes several rows in sequence where that still leaves about three workgroups per compute
  // unit: the staging of the vectors is then shared by those rows
  args.rows_seq = 1;
  if (TEAM > 1 && NORM != kHadamard) args.rows_seq = (int)std::max<int64_t>(1, std::min<int64_t>(8, rows / 768));
  const int64_t per_group = TEAM == 1 ? rows_per_wg : args.rows_seq;
  const int64_t groups = (rows + per_group - 1) / per_group;
  hipLaunchKernelGGL(kern, dim3((unsigned)groups), dim3(64 * n_waves), shmem, st, (const uint16_t*)x, rows, K, ld, ts,
                     L.steps, L.units, operand ? operand + L.codes : nullptr,
                     (uint16_t*)(operand ? operand + L.scales : nullptr),
                     (float*)(operand ? operand + L.mul : nullptr), args);
  return check_hip(hipGetLastError(), "norm_rows_kernel");
}

// One wave per row up to kWideRow channels; wider rows are shared by the kWideTeam waves of a workgroup
// (a wave alone would leave a compute unit with two or three rows in flight).
template <int FMT, int G, int NORM>
int launch_norm_rows(const void* x, int64_t rows, int64_t K, int64_t ld, const float* ts, const OperandLayout& L,
                     uint8_t* operand, const NormArgs& na, hipStream_t st) {
  if (K > kWideRow) return launch_norm_team<FMT, G, NORM, kWideTeam>(x, rows, K, ld, ts, L, operand, na, st);
  return launch_norm_team<FMT, G, NORM, 1>(x, rows, K, ld, ts, L, operand, na, st);
}

template <int FMT, int G>
int launch_norm(int norm, const void* x, int64_t rows, int64_t K, int64_t ld, const float* ts,
                const OperandLayout& L, uint8_t* operand, const NormArgs& na, hipStream_t st) {
  if (norm == kNormRms) return launch_norm_rows<FMT, G, kNormRms>(x, rows, K, ld, ts, L, operand, na, st);
  if (norm == kHadamard) return launch_norm_rows<FMT, G, kHadamard>(x, rows, K, ld, ts, L, operand, na, st);
  return launch_norm_rows<FMT, G, kNormAdaLn>(x, rows, K, ld, ts, L, operand, na, st);
}

NormArgs norm_args(const pq_norm_params& p, void* y, int64_t ldy) {
  NormArgs na;
  na.perm = p.perm;
  na.gamma = (const uint16_t*)p.gamma;
  na.mod_scale = (const uint16_t*)p.mod_scale;
  na.mod_shift = (const uint16_t*)p.mod_shift;
  na.rows_per_mod = p.rows_per_mod > 0 ? p.rows_per_mod : INT64_MAX;
  na.eps = p.eps;
  na.y = (uint16_t*)y;
  na.ldy = ldy;
  na.rows_seq = 1;
  na.had_pow2 = na.had_m = 0;
  na.had_scale = 0.0f;
  return na;
}

// K = 2^k * m with m in {1, 12, 20} (the smallest such m): false if there is none
bool hadamard_factor(int64_t K, int* pow2, int* m) {
  const int ms[3] = {1, 12, 20};
  for (int i = 0; i < 3; ++i) {
    if (K % ms[i]) continue;
    const int64_t p = K / ms[i];
    if (p >= 1 && (p & (p - 1)) == 0) {
      *pow2 = (int)p;
      *m = ms[i];
      return true;
    }
  }
  return false;
}

NormArgs hadamard_args(const int32_t* perm, int64_t K, void* y, int64_t ldy, int pow2, int m) {
  NormArgs na = {};
  na.perm = perm;
  na.rows_per_mod = INT64_MAX;
  na.y = (uint16_t*)y;
  na.ldy = ldy;
  na.had_pow2 = pow2;
  na.had_m = m;
  na.had_scale = (float)(1.0 / sqrt((double)K));
  return na;
}

}  // namespace

int run_norm_reorder(const pq_norm_params& p, const void* x, int64_t rows, int64_t K, int64_t ld, void* y,
                     int64_t ldy, hipStream_t st) {
  OperandLayout L = {};
  L.steps = (K + 63) / 64;
  const int norm = p.kind == PQ_NORM_RMS ? kNormRms : kNormAdaLn;
  return launch_norm<kFmtNone, 64>(norm, x, rows, K, ld, nullptr, L, nullptr, norm_args(p, y, ldy), st);
}

int run_norm_quantize_packed(const pq_norm_params& p, pq_format fmt, int group, const void* x, int64_t rows,
                             int64_t K, int64_t ld, const float* ts, void* operand, void* y, int64_t ldy,
                             hipStream_t st) {
  const OperandLayout L = operand_layout(fmt, group, rows, K);
  const int norm = p.kind == PQ_NORM_RMS ? kNormRms : kNormAdaLn;
  const NormArgs na = norm_args(p, y, ldy);
  uint8_t* o = (uint8_t*)operand;
  if (fmt == PQ_FMT_NVFP4) return launch_norm<kNvfp4, 16>(norm, x, rows, K, ld, ts, L, o, na, st);
#define PQ_INT_CASE(F, FE)                                                      \
  if (fmt == F) {                                                               \
    switch (group) {                                                            \
      case 32: return launch_norm<FE, 32>(norm, x, rows, K, ld, ts, L, o, na, st);   \
      case 64: return launch_norm<FE, 64>(norm, x, rows, K, ld, ts, L, o, na, st);   \
      case 128: return launch_norm<FE, 128>(norm, x, rows, K, ld, ts, L, o, na, st); \
      case 256: return launch_norm<FE, 256>(norm, x, rows, K, ld, ts, L, o, na, st); \
    }                                                                           \
  }
  PQ_INT_CASE(PQ_FMT_INT4, kInt4)
  PQ_INT_CASE(PQ_FMT_INT3, kInt3)
#undef PQ_INT_CASE
  return fail(PQ_ERR_FORMAT, "unsupported (format, group) = (%d, %d)", (int)fmt, group);
}

bool hadamard_width_ok(int64_t K) {
  int p, m;
  return hadamard_factor(K, &p, &m);
}

int run_hadamard_reorder(const int32_t* perm, const void* x, int64_t rows, int64_t K, int64_t ld, void* y,
                         int64_t ldy, hipStream_t st) {
  int p, m;
  if (!hadamard_factor(K, &p, &m)) return fail(PQ_ERR_SHAPE, "no Hadamard construction for K=%lld", (long long)K);
  OperandLayout L = {};
  L.steps = (K + 63) / 64;
  return launch_norm<kFmtNone, 64>(kHadamard, x, rows, K, ld, nullptr, L, nullptr, hadamard_args(perm, K, y, ldy, p, m), st);
}

int run_hadamard_quantize_packed(const int32_t* perm, pq_format fmt, int group, const void* x, int64_t rows,
                                 int64_t K, int64_t ld, const float* ts, void* operand, void* y, int64_t ldy,
                                 hipStream_t st) {
  int p, m;
  if (!hadamard_factor(K, &p, &m)) return fail(PQ_ERR_SHAPE, "no Hadamard construction for K=%lld", (long long)K);
  const OperandLayout L = operand_layout(fmt, group, rows, K);
  const NormArgs na = hadamard_args(perm, K, y, ldy, p, m);
  uint8_t* o = (uint8_t*)operand;
  if (fmt == PQ_FMT_NVFP4) return launch_norm<kNvfp4, 16>(kHadamard, x, rows, K, ld, ts, L, o, na, st);
#define PQ_INT_CASE(F, FE)                                                           \
  if (fmt == F) {                                                                    \
    switch (group) {                                                                 \
      case 32: return launch_norm<FE, 32>(kHadamard, x, rows, K, ld, ts, L, o, na, st);   \
      case 64: return launch_norm<FE, 64>(kHadamard, x, rows, K, ld, ts, L, o, na, st);   \
      case 128: return launch_norm<FE, 128>(kHadamard, x, rows, K, ld, ts, L, o, na, st); \
      case 256: return launch_norm<FE, 256>(kHadamard, x, rows, K, ld, ts, L, o, na, st); \
    }                                                                                \
  }
  PQ_INT_CASE(PQ_FMT_INT4, kInt4)
  PQ_INT_CASE(PQ_FMT_INT3, kInt3)
#undef PQ_INT_CASE
  return fail(PQ_ERR_FORMAT, "unsupported (format, group) = (%d, %d)", (int)fmt, group);
}

}  // namespace pq
