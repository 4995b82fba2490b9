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
// LDS rows are 64 fp16 plus one 16-byte piece of padding (144 bytes): measured on gfx950, the
// 16-byte fragment reads of the 32-row MFMA operand pattern run at full LDS rate with this
// stride (an XOR swizzle of unpadded rows reaches two thirds of it).
#include <string.h>

#include "pq_qgemm_common.h"

namespace pq {

// Software pipeline of one K step s (P = s & 1 is the LDS stage being multiplied):
//   - global loads for step s + 3 are issued first (two steps ahead of their use),
//   - the MFMAs of step s run on stage P, fragment reads for the next 16-wide k slice are
//     issued one slice ahead,
//   - between MFMAs the wave unpacks its slice of step s + 1 (already in registers) pair by
//     pair and writes it to stage P ^ 1,
//   - one barrier ends the step.
// Every MFMA is followed by its share of vector-ALU and LDS work in program order, pinned
// with scheduling barriers, so that the matrix pipe and the vector ALU overlap inside a wave
// instead of alternating in phases.
template <int FMT, int G, int BM, int BN, int WGM, int WGN, bool OUT_F32>
__global__ __launch_bounds__(WGM* WGN * 64) void qgemm_kernel(OperandView A, OperandView W, int M, int N,
                                                              int K, void* __restrict__ y, int64_t ldy,
                                                              int tiles_m, int tiles_n) {
  const float* __restrict__ a_mul = A.mul;
  const float* __restrict__ w_mul = W.mul;
  const int a_mul_stride = A.mul_stride, w_mul_stride = W.mul_stride;
  constexpr int T = WGM * WGN * 64;
  // wave tile: WTM x WTN outputs.  BM need not divide evenly over the WGM wave rows: the last wave row
  // then owns TM_LAST < TM MFMA tiles along M (a 224-row tile is 128 + 96), and the waves are numbered so
  // that every SIMD hosts one wave of each kind (see below)
  constexpr int WTM = (BM + WGM * 32 - 1) / (WGM * 32) * 32, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;        // MFMA tiles per wave
  constexpr int TM_LAST = (BM - (WGM - 1) * WTM) / 32;
  constexpr bool RAGGED_M = TM_LAST != TM;
  constexpr int SL = BN * 2 / T;                     // slices per operand per thread
  static_assert(BN * 2 % T == 0 && (BM * 2 + T - 1) / T == SL, "whole slices per thread, as many for A as for W");
  static_assert(BM % 32 == 0 && WTN % 32 == 0 && TM_LAST >= 1 && TM_LAST <= TM, "wave tile");
  static_assert(!RAGGED_M || (WGM == 2 && WGN == 4), "the uneven split is laid out for 2 x 4 waves");
  // the loader covers SL * T / 2 rows of each operand; an A tile of fewer rows (BM = 224) still gets all
  // of them in LDS, so that no thread needs a predicate around its unpack writes (the spare rows hold zeros
  // and are never read)
  constexpr int A_TILE_BYTES = SL * (T / 2) * kRowBytes, W_TILE_BYTES = BN * kRowBytes;
  constexpr int STAGE_BYTES = A_TILE_BYTES + W_TILE_BYTES;
  constexpr int NT = 8 * SL;                         // unpack pair tasks per k slice

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  // ---- tile assignment: consecutive workgroup ids land on different XCDs (8 of them, each
  // with its own L2); give every XCD a contiguous range of tiles, and walk tiles in bands of
  // 8 along M so that concurrently running workgroups share A and W strips.
  const int n_tiles = tiles_m * tiles_n;
  int pid = blockIdx.x;
  {
    // XCD x runs the workgroups with id % 8 == x: (n_tiles - x + 7) / 8 of them, which get the tiles
    // from x * (n_tiles / 8) + min(x, n_tiles % 8) on
    const int x = pid & 7, q8 = n_tiles >> 3, r8 = n_tiles & 7;
    pid = x * q8 + min(x, r8) + (pid >> 3);
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
  // Waves of a workgroup go to the four SIMDs in turn (wave w on SIMD w % 4).  With the uneven split
  // waves w and w + 4 take different wave rows, so that every SIMD's matrix pipe gets TM + TM_LAST tile
  // rows of work per step.
  const int wave_m = RAGGED_M ? ((wave >> 2) ^ wave) & 1 : wave % WGM;
  const int wave_n = RAGGED_M ? wave >> 1 : wave / WGM;
  // MFMA tile rows this wave owns (wave-uniform, kept in a scalar register)
  const int tm_cnt = RAGGED_M ? __builtin_amdgcn_readfirstlane(wave_m == WGM - 1 ? TM_LAST : TM) : TM;

  // loader: this thread owns tile rows tid / 2 + q * (T / 2), k offset 32 * (tid & 1), of both
  // operands
  const int ld_row = tid >> 1, ld_half = tid & 1;
  bool a_ok[SL], w_ok[SL];
  const uint8_t *a_crow[SL], *w_crow[SL];
  const uint8_t *a_srow[SL], *w_srow[SL];
#pragma unroll
  for (int q = 0; q < SL; ++q) {
    const int r = ld_row + q * (T / 2);
    a_ok[q] = m0 + r < M && r < BM;
    w_ok[q] = n0 + r < N;
    const int a_row = min(m0 + r, M - 1), w_row = min(n0 + r, N - 1);
    a_crow[q] = A.codes + (int64_t)a_row * A.code_row;
    w_crow[q] = W.codes + (int64_t)w_row * W.code_row;
    a_srow[q] = A.scales + (int64_t)a_row * A.sc_row;
    w_srow[q] = W.scales + (int64_t)w_row * W.sc_row;
  }
  auto load_a = [&](int step, Slice (&ra)[SL]) {
#pragma unroll
    for (int q = 0; q < SL; ++q)
      ra[q] = load_slice<FMT, G>(a_crow[q], A.code_step, a_srow[q], A.sc_step, K, step, ld_half);
  };
  auto load_w = [&](int step, Slice (&rw)[SL]) {
#pragma unroll
    for (int q = 0; q < SL; ++q)
      rw[q] = load_slice<FMT, G>(w_crow[q], W.code_step, w_srow[q], W.sc_step, K, step, ld_half);
  };
  // byte offsets of this thread's 16-byte pieces inside an operand tile: [slot][piece]
  int st_off[SL][4];
#pragma unroll
  for (int q = 0; q < SL; ++q)
#pragma unroll
    for (int c = 0; c < 4; ++c) st_off[q][c] = lds_off(ld_row + q * (T / 2), ld_half * 4 + c);

  const int frag_row = lane & 31, frag_half = lane >> 5;
  // fragment read offsets: row part + swizzled piece for each of the four k slices
  int w_frag_base[TN], x_frag_base[TM];
#pragma unroll
  for (int i = 0; i < TN; ++i) w_frag_base[i] = (wave_n * WTN + i * 32 + frag_row) * kRowBytes;
#pragma unroll
  for (int j = 0; j < TM; ++j) x_frag_base[j] = (wave_m * WTM + j * 32 + frag_row) * kRowBytes;
  int piece_off[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) piece_off[kk] = (kk * 2 + frag_half) << 4;

  float16_t acc[TN][TM];
#pragma unroll
  for (int i = 0; i < TN; ++i)
#pragma unroll
    for (int j = 0; j < TM; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  Slice raw_a[2][SL], raw_w[2][SL];
  const int ksteps = (K + kBK - 1) / kBK;

  // one operand slice -> its four 16-byte pieces in LDS (used by the prologue only)
  auto unpack_all = [&](const Slice& sl, bool ok, unsigned char* tile, int q) {
    PairScale s0, s1;
    slice_scales<FMT>(sl, ok, s0, s1);
    const uint32_t d[4] = {sl.codes.x, sl.codes.y, sl.codes.z, sl.codes.w};
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const PairScale& sc = c < 2 ? s0 : s1;
      uint4 v = make_uint4(unpack_pair<FMT, 0>(d[c], sc), unpack_pair<FMT, 1>(d[c], sc),
                           unpack_pair<FMT, 2>(d[c], sc), unpack_pair<FMT, 3>(d[c], sc));
      *reinterpret_cast<uint4*>(tile + st_off[q][c]) = v;
    }
  };

  // ---- prologue: stage 0 <- step 0, raw[1] <- step 1, raw[0] <- step 2
  load_a(0, raw_a[0]);
  load_w(0, raw_w[0]);
  load_a(1, raw_a[1]);
  load_w(1, raw_w[1]);
#pragma unroll
  for (int q = 0; q < SL; ++q) {
    unpack_all(raw_a[0][q], a_ok[q] && ld_half * 32 < K, smem, q);
    unpack_all(raw_w[0][q], w_ok[q] && ld_half * 32 < K, smem + A_TILE_BYTES, q);
  }
  load_a(2, raw_a[0]);
  load_w(2, raw_w[0]);
  __syncthreads();

  // TMc: the MFMA tile rows of the calling wave as a compile-time constant (TM, or TM_LAST for the
  // short wave row of an uneven split) -- each kind of wave runs its own straight-line loop
  auto body = [&](auto Pc, auto TMc, int s) {
    constexpr int P = decltype(Pc)::value;
    constexpr int TMW = decltype(TMc)::value;
    constexpr int NM = TN * TMW;                     // MFMAs per 16-wide k slice
    const unsigned char* a_t = smem + P * STAGE_BYTES;
    const unsigned char* w_t = a_t + A_TILE_BYTES;
    unsigned char* a_nx = smem + (P ^ 1) * STAGE_BYTES;
    unsigned char* w_nx = a_nx + A_TILE_BYTES;

    // step s + 1 sits in raw[P ^ 1]; it is unpacked during this step and the registers are
    // refilled with step s + 3 as soon as they are free (A after half the step, W at the end)
    Slice(&ca)[SL] = raw_a[P ^ 1];
    Slice(&cw)[SL] = raw_w[P ^ 1];
    PairScale sc_a[SL][2], sc_w[SL][2];
#pragma unroll
    for (int q = 0; q < SL; ++q) {
      const bool k_ok = (s + 1) * kBK + ld_half * 32 < K;
      slice_scales<FMT>(ca[q], a_ok[q] && k_ok, sc_a[q][0], sc_a[q][1]);
      slice_scales<FMT>(cw[q], w_ok[q] && k_ok, sc_w[q][0], sc_w[q][1]);
    }

    // weight fragments: one set, each reloaded for the next k slice right after its last MFMA;
    // activation fragments: two sets (they are used by every MFMA of a slice)
    half8_t wf[TN], xf[2][TM];
    auto read_w = [&](int kk, int i) {
      wf[i] = *reinterpret_cast<const half8_t*>(w_t + w_frag_base[i] + piece_off[kk]);
    };
    auto read_x = [&](int set, int kk, int j) {
      xf[set][j] = *reinterpret_cast<const half8_t*>(a_t + x_frag_base[j] + piece_off[kk]);
    };
#pragma unroll
    for (int j = 0; j < TMW; ++j) read_x(0, 0, j);
#pragma unroll
    for (int i = 0; i < TN; ++i) read_w(0, i);

    uint32_t pk[4];        // the unit (one dword of codes -> one 16-byte piece) being assembled
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const int cur = kk & 1;
#pragma unroll
      for (int mi = 0; mi < NM; ++mi) {
        const int i = mi / TMW, j = mi % TMW;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wf[i], xf[cur][j], acc[i][j], 0, 0, 0);
        if (kk < 3) {
          if (j == TMW - 1) read_w(kk + 1, i);                // wf[i] is free now
          if (mi < TMW) read_x(cur ^ 1, kk + 1, mi);          // next slice's activations, early
        }
        // unpack tasks: NT pairs per k slice, spread evenly over the MFMAs.  Task order over
        // the whole step: A slot 0 (4 pieces x 4 pairs), A slot 1, ..., then the W slots.
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          if (t * NM / NT != mi) continue;
          const int g = kk * NT + t;          // global pair task 0 .. 32 * SL - 1
          const int u = g / 4;                // unit: one dword of codes -> one LDS piece
          const int jp = g % 4;
          const bool is_w = u >= 4 * SL;
          const int q = (u / 4) % SL, c = u % 4;
          const Slice& src = is_w ? cw[q] : ca[q];
          const uint32_t d = c == 0 ? src.codes.x : c == 1 ? src.codes.y : c == 2 ? src.codes.z : src.codes.w;
          const PairScale& sc = is_w ? sc_w[q][c / 2] : sc_a[q][c / 2];
          if (jp == 0) pk[0] = unpack_pair<FMT, 0>(d, sc);
          if (jp == 1) pk[1] = unpack_pair<FMT, 1>(d, sc);
          if (jp == 2) pk[2] = unpack_pair<FMT, 2>(d, sc);
          if (jp == 3) {
            pk[3] = unpack_pair<FMT, 3>(d, sc);
            unsigned char* dst = (is_w ? w_nx : a_nx) + st_off[q][c];
            *reinterpret_cast<uint4*>(dst) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
          }
        }
        if (kk == 1 && mi == NM - 1) load_a(s + 3, ca);
        if (kk == 3 && mi == NM - 1) load_w(s + 3, cw);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    __syncthreads();
  };

  // two steps per trip so that the LDS stage and the register set are compile-time constants;
  // an odd step count runs one extra step on all-zero operands (loads beyond K are zeroed),
  // which keeps a single loop exit (two exits would double the live accumulators)
  if (!RAGGED_M || tm_cnt == TM) {
    for (int s = 0; s < ksteps; s += 2) {
      body(IntC<0>{}, IntC<TM>{}, s);
      body(IntC<1>{}, IntC<TM>{}, s + 1);
    }
  } else {
    // same number of barriers as the other kind of wave: one per step
    for (int s = 0; s < ksteps; s += 2) {
      body(IntC<0>{}, IntC<TM_LAST>{}, s);
      body(IntC<1>{}, IntC<TM_LAST>{}, s + 1);
    }
  }

  // ---- epilogue: lane holds, per MFMA tile, column m = lane % 32 and rows
  // n = 8 * (r / 4) + 4 * (lane / 32) + r % 4.  The bf16 tile is staged through LDS (the
  // operand stages are free after the last barrier) so that global stores are 16 bytes per
  // lane and contiguous along n; the fp32 variant (a checking aid) stores directly.
  constexpr int C_ROW_BYTES = BN * 2 + 16;
  static_assert(BM * C_ROW_BYTES <= 2 * STAGE_BYTES, "output tile fits in the operand stages");
  // The column factors (and the optional bias of the linear layer, y = x W^T + b) do not depend on
  // the row block: loaded once (16 per MFMA tile column).
  const uint16_t* __restrict__ bias = W.bias;               // uniform
  float wm[TN][16], wb[TN][16];
#pragma unroll
  for (int i = 0; i < TN; ++i)
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int n = n0 + wave_n * WTN + i * 32 + q * 8 + frag_half * 4 + e;
        wm[i][q * 4 + e] = w_mul[(int64_t)(min(n, N - 1) * w_mul_stride)];
        wb[i][q * 4 + e] = bias ? bf16_to_f32(bias[min(n, N - 1)]) : 0.0f;
      }
#pragma unroll
  for (int j = 0; j < TM; ++j) {
    if (RAGGED_M && j >= tm_cnt) break;         // wave-uniform
    const int ml = wave_m * WTM + j * 32 + frag_row;
    const int m = m0 + ml;
    const float am = a_mul[(int64_t)(min(m, M - 1) * a_mul_stride)];
#pragma unroll
    for (int i = 0; i < TN; ++i) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int nl = wave_n * WTN + i * 32 + q * 8 + frag_half * 4;
        const int n = n0 + nl;
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = acc[i][j][q * 4 + e] * (am * wm[i][q * 4 + e]);
        if (bias) {                     // without a bias the product is stored as it is (a -0 stays -0)
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] += wb[i][q * 4 + e];
        }
        if constexpr (OUT_F32) {
          if (m < M && n < N) {
            float* yo = reinterpret_cast<float*>(y) + (int64_t)m * ldy + n;
            if (n + 3 < N) {
              *reinterpret_cast<float4*>(yo) = make_float4(v[0], v[1], v[2], v[3]);
            } else {
              for (int e = 0; e < 4 && n + e < N; ++e) yo[e] = v[e];
            }
          }
        } else {
          // round to nearest even, two values per instruction (v_cvt_pk_bf16_f32)
          typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
          typedef float f32x2_t __attribute__((ext_vector_type(2)));
          const bf16x2_t lo = __builtin_convertvector((f32x2_t){v[0], v[1]}, bf16x2_t);
          const bf16x2_t hi = __builtin_convertvector((f32x2_t){v[2], v[3]}, bf16x2_t);
          *reinterpret_cast<uint2*>(smem + ml * C_ROW_BYTES + nl * 2) =
              make_uint2(__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi));
        }
      }
    }
  }
  if constexpr (!OUT_F32) {
    __syncthreads();
    constexpr int CHUNKS_PER_ROW = BN / 8;               // 16-byte chunks of 8 bf16
    uint16_t* yb = reinterpret_cast<uint16_t*>(y);
#pragma unroll 4
    for (int c = tid; c < BM * CHUNKS_PER_ROW; c += T) {
      const int row = c / CHUNKS_PER_ROW, cc = c % CHUNKS_PER_ROW;
      const int m = m0 + row, n = n0 + cc * 8;
      if (m >= M || n >= N) continue;
      const uint4 v = *reinterpret_cast<const uint4*>(smem + row * C_ROW_BYTES + cc * 16);
      uint16_t* yo = yb + (int64_t)m * ldy + n;
      if (n + 7 < N) {
        // the output is not read again by this kernel: a streaming store keeps it from displacing
        // the operand strips in L2
        typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
        __builtin_nontemporal_store((u32x4){v.x, v.y, v.z, v.w}, reinterpret_cast<u32x4*>(yo));
      } else {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
        for (int e = 0; e < 8 && n + e < N; ++e) yo[e] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
      }
    }
  }
}

// ------------------------------------------------------------------------ INT scale prepass
// One wave per row of scales: recover each group's bf16 maximum h = bf16_rne(s * Q), find the
// row's largest exponent, and emit fp16 h * 2^-E plus the fp32 epilogue factor 2^E / Q, with E
// chosen so that the largest h * 2^-E stays below 2^11.
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
  // E = exponent(mx) - 10: the row maximum lands in [2^10, 2^11), so that the addend 24 * h of
  // the unpack fma (and with it Q * h) stays below the fp16 maximum
  int e = (int)((as_u32(mx) >> 23) & 0xFF) - 127;
  if (mx == 0.0f) e = 0;
  int E = e - 10;
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

// ------------------------------------------------------------------------ INT scale form check
// The product folds the group maximum h = bf16_rne(s * Q) into its fp16 operands instead of the stored
// scale s, which is the same number only if s = fl32(h / Q) -- true for what the quantizers of this
// library write from bf16 inputs, not for arbitrary fp32 scales.  This kernel counts the scales that
// are not of that form (and the negative or non-finite ones).
__global__ __launch_bounds__(256) void check_int_scales_kernel(const float* __restrict__ s, int64_t n, float Q,
                                                               unsigned long long* __restrict__ bad) {
  unsigned int mine = 0;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const float v = s[i];
    const float h = as_f32(f32_to_bf16_rne(v * Q) << 16);
    const bool ok = v >= 0.0f && v <= 3.0e38f && div_const(h, Q, 1.0f / Q) == v;
    mine += ok ? 0u : 1u;
  }
  // wave total, one atomic per wave
  for (int off = 32; off >= 1; off >>= 1) mine += (unsigned int)__shfl_xor((int)mine, off, kWave);
  if ((threadIdx.x & 63) == 0 && mine) atomicAdd(bad, (unsigned long long)mine);
}

__global__ void zero_u64_kernel(unsigned long long* p) { *p = 0ull; }

int run_check_int_scales(pq_format fmt, int group, const void* scales, int64_t rows, int64_t K, int64_t* bad_count,
                         void* ws, hipStream_t st) {
  const int64_t n = rows * (K / group);
  unsigned long long* bad = (unsigned long long*)ws;
  hipLaunchKernelGGL(zero_u64_kernel, dim3(1), dim3(1), 0, st, bad);
  int64_t blocks = (n + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(check_int_scales_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const float*)scales, n,
                     qmax_of((int)fmt), bad);
  int rc = check_hip(hipGetLastError(), "check_int_scales_kernel");
  if (rc) return rc;
  double* h = pinned_doubles(1);
  if (!h) return fail(PQ_ERR_HIP, "pq_qgemm_check_int_scales: no pinned host memory");
  if ((rc = check_hip(hipMemcpyAsync(h, bad, 8, hipMemcpyDeviceToHost, st), "copy count"))) return rc;
  if ((rc = check_hip(hipStreamSynchronize(st), "hipStreamSynchronize"))) return rc;
  unsigned long long c;
  memcpy(&c, h, 8);
  *bad_count = (int64_t)c;
  return PQ_OK;
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
static int launch_gemm(const OperandView& A, const OperandView& W, int M, int N, int K, void* y, int64_t ldy,
                       hipStream_t st) {
  constexpr int T = WGM * WGN * 64;
  constexpr size_t shmem = 2 * (size_t)((BM * 2 + T - 1) / T * (T / 2) + BN) * kRowBytes;
  auto kern = qgemm_kernel<FMT, G, BM, BN, WGM, WGN, OUT_F32>;
  if (shmem > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
    if (e != hipSuccess) return check_hip(e, "hipFuncSetAttribute(qgemm_kernel)");
  }
  int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  int64_t n_tiles = (int64_t)tiles_m * tiles_n;
  if (n_tiles > 0x7FFFFFFF) return fail(PQ_ERR_SHAPE, "too many output tiles");
  hipLaunchKernelGGL(kern, dim3((unsigned)n_tiles), dim3(T), shmem, st, A, W, M, N, K, y, ldy, tiles_m, tiles_n);
  return check_hip(hipGetLastError(), "qgemm_kernel");
}

// Tile choice.  The cost of a variant is the number of rounds its tiles need on the 256 compute units
// (one workgroup per unit: the LDS stages take 135 KB or more) times the tile area:
//   256 x 256, eight waves                          the default;
//   224 x 256, eight waves (wave rows of 128 + 96)  when that saves a round or shortens the only one: at
//                                                   M = 4608 (18 x 256 = 20.6 x 224) a grid of 18 x 12 tiles
//                                                   leaves 40 units idle, one of 21 x 12 keeps 252 busy with
//                                                   7/8 of the work each;
//   128 x 128, four waves                           small outputs (about 35 % more operand traffic per
//                                                   output, but more of the units get a tile).
static int choose_tile(int M, int N) {
  auto rounds = [&](int bm, int bn) {
    int64_t tiles = (int64_t)((M + bm - 1) / bm) * ((N + bn - 1) / bn);
    return (double)((tiles + 255) / 256);
  };
  const double c256 = rounds(256, 256) * 256 * 256;
  const double c224 = rounds(224, 256) * 224 * 256;
  const double c128 = rounds(128, 128) * 128 * 128 * 1.35;
  if (c128 < c256 && c128 < c224) return 2;
  return c224 < c256 ? 3 : 1;
}

template <int FMT, int G, bool OUT_F32>
static int pick_tile(const OperandView& A, const OperandView& W, int M, int N, int K, void* y, int64_t ldy,
                     hipStream_t st) {
  const int choice = choose_tile(M, N);
  if (choice == 1) return launch_gemm<FMT, G, 256, 256, 2, 4, OUT_F32>(A, W, M, N, K, y, ldy, st);
  if (choice == 3) return launch_gemm<FMT, G, 224, 256, 2, 4, OUT_F32>(A, W, M, N, K, y, ldy, st);
  return launch_gemm<FMT, G, 128, 128, 2, 2, OUT_F32>(A, W, M, N, K, y, ldy, st);
}

template <int FMT, int G>
static int launch_views_fg(const OperandView& A, const OperandView& W, int M, int N, int K, void* y,
                           int64_t ldy, bool out_f32, hipStream_t st) {
  if (out_f32) return pick_tile<FMT, G, true>(A, W, M, N, K, y, ldy, st);
  return pick_tile<FMT, G, false>(A, W, M, N, K, y, ldy, st);
}

// the product kernel on two operand views (any mix of layouts)
int launch_qgemm_views(pq_format fmt, int group, const OperandView& A, const OperandView& W, int64_t M,
                       int64_t N, int64_t K, void* y, int64_t ldy, bool out_f32, hipStream_t st) {
#define PQ_ARGS A, W, (int)M, (int)N, (int)K, y, ldy, out_f32, st
  if (fmt == PQ_FMT_NVFP4) return launch_views_fg<kNvfp4, 16>(PQ_ARGS);
  if (fmt == PQ_FMT_INT4) {
    switch (group) {
      case 32: return launch_views_fg<kInt4, 32>(PQ_ARGS);
      case 64: return launch_views_fg<kInt4, 64>(PQ_ARGS);
      case 128: return launch_views_fg<kInt4, 128>(PQ_ARGS);
      case 256: return launch_views_fg<kInt4, 256>(PQ_ARGS);
    }
  }
  if (fmt == PQ_FMT_INT3) {
    switch (group) {
      case 32: return launch_views_fg<kInt3, 32>(PQ_ARGS);
      case 64: return launch_views_fg<kInt3, 64>(PQ_ARGS);
      case 128: return launch_views_fg<kInt3, 128>(PQ_ARGS);
      case 256: return launch_views_fg<kInt3, 256>(PQ_ARGS);
    }
  }
#undef PQ_ARGS
  return fail(PQ_ERR_FORMAT, "unsupported (format, group) = (%d, %d)", (int)fmt, group);
}

// Operands in the row-major layout of the quantizers.  NVFP4 scales are read in place; INT
// scales go through the per-row normalisation pass into `ws` first (phases & 1), the product
// (phases & 2) then reads that working copy.
int run_qgemm(pq_format fmt, int group, const uint8_t* a_codes, const void* a_scales,
              const float* a_ts, const uint8_t* w_codes, const void* w_scales, const float* w_ts,
              int64_t M, int64_t N, int64_t K, void* y, int64_t ldy, bool out_f32, int phases,
              void* ws, hipStream_t st) {
  OperandView A{a_codes, K / 2, 32, nullptr, 0, 2, nullptr, 0};
  OperandView W{w_codes, K / 2, 32, nullptr, 0, 2, nullptr, 0};
  if (fmt == PQ_FMT_NVFP4) {
    A.scales = (const uint8_t*)a_scales;
    W.scales = (const uint8_t*)w_scales;
    A.sc_row = W.sc_row = K / 16;
    A.mul = a_ts;
    W.mul = w_ts;
  } else {
    if (fmt != PQ_FMT_INT4 && fmt != PQ_FMT_INT3)
      return fail(PQ_ERR_FORMAT, "unsupported (format, group) = (%d, %d)", (int)fmt, group);
    GemmWs G;
    carve_gemm(ws, fmt, group, M, N, K, &G);
    const float Q = qmax_of((int)fmt);
    if (phases & 1) {
      hipLaunchKernelGGL(int_scale_prep_kernel, dim3((unsigned)((M + 3) / 4)), dim3(256), 0, st,
                         (const float*)a_scales, (int)M, (int)(K / group), Q, G.a_h, G.a_mul);
      hipLaunchKernelGGL(int_scale_prep_kernel, dim3((unsigned)((N + 3) / 4)), dim3(256), 0, st,
                         (const float*)w_scales, (int)N, (int)(K / group), Q, G.w_h, G.w_mul);
      int rc = check_hip(hipGetLastError(), "int_scale_prep_kernel");
      if (rc) return rc;
    }
    A.scales = (const uint8_t*)G.a_h;
    W.scales = (const uint8_t*)G.w_h;
    A.sc_row = W.sc_row = (K / group) * 2;
    A.mul = G.a_mul;
    W.mul = G.w_mul;
    A.mul_stride = W.mul_stride = 1;
  }
  if (!(phases & 2)) return PQ_OK;
  return launch_qgemm_views(fmt, group, A, W, M, N, K, y, ldy, out_f32, st);
}

}  // namespace pq
