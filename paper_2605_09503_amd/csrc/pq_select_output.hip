// Permutation selection with the layer-output error as the calibration metric -- the other reading
// of "the candidate with the smallest quantization error on the calibration data" (paper Sec. 3.3):
//     E_out(pi) = sum_b ||X_b W^T - Q(X_b P) Q(P^T W)^T||^2 / sum_b ||X_b W^T||^2        (Eq. 8)
// The candidate orders are those of pq_select_perm (joint score, Eq. 9, alpha grid).  The quantized
// product runs through the forward path itself (gathering quantizer -> operand layout -> product
// kernel with an fp32 result); the unquantized product comes from a plain bf16 MFMA kernel below.
// Offline work: per candidate and batch four launches; nothing here is tuned beyond being correct
// and deterministic (fixed summation order).
#include <string.h>

#include "pq_qgemm_common.h"

namespace pq {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

constexpr int kRefTile = 128;                 // output tile edge
constexpr int kRefStep = 32;                  // K elements per step
constexpr int kRefRowBytes = kRefStep * 2 + 16;   // padded LDS row: 80 bytes

// Y[m, n] = sum_k X[m, k] W[n, k], bf16 inputs, fp32 accumulation (v_mfma_f32_32x32x16_bf16),
// fp32 output.  128 x 128 tile, four waves of 64 x 64; K % 32 == 0.
__global__ __launch_bounds__(256) void ref_gemm_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ w,
                                                       int M, int N, int K, float* __restrict__ y, int64_t ldy) {
  __shared__ __align__(16) unsigned char lds[2 * kRefTile * kRefRowBytes];
  unsigned char* a_t = lds;
  unsigned char* w_t = lds + kRefTile * kRefRowBytes;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave & 1, wave_n = wave >> 1;
  const int m0 = blockIdx.x * kRefTile, n0 = blockIdx.y * kRefTile;
  // loader: 128 rows x 64 bytes per operand = 512 pieces of 16 bytes; thread t takes pieces t, t + 256
  const int ld_row = tid >> 2, ld_piece = tid & 3;
  const uint16_t* xa = x + (int64_t)min(m0 + ld_row, M - 1) * K + ld_piece * 8;
  const uint16_t* xb = x + (int64_t)min(m0 + ld_row + 64, M - 1) * K + ld_piece * 8;
  const uint16_t* wa = w + (int64_t)min(n0 + ld_row, N - 1) * K + ld_piece * 8;
  const uint16_t* wb2 = w + (int64_t)min(n0 + ld_row + 64, N - 1) * K + ld_piece * 8;
  const int st_a = ld_row * kRefRowBytes + ld_piece * 16;
  const int st_b = (ld_row + 64) * kRefRowBytes + ld_piece * 16;
  const int frag_row = lane & 31, frag_half = lane >> 5;

  float16_t acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  uint4 ra = *reinterpret_cast<const uint4*>(xa), rb = *reinterpret_cast<const uint4*>(xb);
  uint4 rc = *reinterpret_cast<const uint4*>(wa), rd = *reinterpret_cast<const uint4*>(wb2);
  for (int k0 = 0; k0 < K; k0 += kRefStep) {
    *reinterpret_cast<uint4*>(a_t + st_a) = ra;
    *reinterpret_cast<uint4*>(a_t + st_b) = rb;
    *reinterpret_cast<uint4*>(w_t + st_a) = rc;
    *reinterpret_cast<uint4*>(w_t + st_b) = rd;
    __syncthreads();
    if (k0 + kRefStep < K) {                       // next step's pieces while this one is multiplied
      ra = *reinterpret_cast<const uint4*>(xa + k0 + kRefStep);
      rb = *reinterpret_cast<const uint4*>(xb + k0 + kRefStep);
      rc = *reinterpret_cast<const uint4*>(wa + k0 + kRefStep);
      rd = *reinterpret_cast<const uint4*>(wb2 + k0 + kRefStep);
    }
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
      bf16x8_t xf[2], wf[2];
#pragma unroll
      for (int j = 0; j < 2; ++j)
        xf[j] = *reinterpret_cast<const bf16x8_t*>(a_t + (wave_m * 64 + j * 32 + frag_row) * kRefRowBytes +
                                                   (kk * 2 + frag_half) * 16);
#pragma unroll
      for (int i = 0; i < 2; ++i)
        wf[i] = *reinterpret_cast<const bf16x8_t*>(w_t + (wave_n * 64 + i * 32 + frag_row) * kRefRowBytes +
                                                   (kk * 2 + frag_half) * 16);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[i], xf[j], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
  }
  // lane holds, per 32 x 32 block, column m = lane % 32 and rows n = 8 (r / 4) + 4 (lane / 32) + r % 4
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int m = m0 + wave_m * 64 + j * 32 + frag_row;
    if (m >= M) continue;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = n0 + wave_n * 64 + i * 32 + q * 8 + frag_half * 4;
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (n + e < N) y[(int64_t)m * ldy + n + e] = acc[i][j][q * 4 + e];
      }
  }
}

constexpr int kDiffBlocks = 1024;

// partial[b] = sum over the block's share of (ref - hat)^2, partial[kDiffBlocks + b] of ref^2 (fp64)
__global__ __launch_bounds__(256) void sqdiff_partial_kernel(const float* __restrict__ ref, const float* __restrict__ hat,
                                                             int64_t rows, int N, int64_t ld, double* __restrict__ partial) {
  __shared__ double red[2][4];
  double d2 = 0.0, r2 = 0.0;
  const int64_t total = rows * N;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t r = i / N;
    const int64_t at = r * ld + (i - r * N);
    const double a = (double)ref[at], b = (double)hat[at];
    d2 += (a - b) * (a - b);
    r2 += a * a;
  }
  d2 = wave_sum(d2);
  r2 = wave_sum(r2);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) {
    red[0][wave] = d2;
    red[1][wave] = r2;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    partial[blockIdx.x] = (red[0][0] + red[0][1]) + (red[0][2] + red[0][3]);
    partial[kDiffBlocks + blockIdx.x] = (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]);
  }
}

// sums[0] += sum of the first kDiffBlocks partials, sums[1] += sum of the second (one wave, fixed order)
__global__ __launch_bounds__(64) void sqdiff_finish_kernel(const double* __restrict__ partial, double* __restrict__ num,
                                                           double* __restrict__ den) {
  double a = 0.0, b = 0.0;
  for (int i = threadIdx.x; i < kDiffBlocks; i += 64) {
    a += partial[i];
    b += partial[kDiffBlocks + i];
  }
  a = wave_sum(a);
  b = wave_sum(b);
  if (threadIdx.x == 0) {
    *num += a;
    if (den) *den += b;
  }
}

// moved[j] = number of positions where candidate j differs from the identity; block 0 also clears the
// n_sums running sums (which do not overlap moved[])
__global__ __launch_bounds__(256) void moved_kernel(const int32_t* __restrict__ cands, int K, double* __restrict__ sums,
                                                    int n_sums, double* __restrict__ moved) {
  const int j = blockIdx.x;
  int c = 0;
  for (int i = threadIdx.x; i < K; i += 256) c += cands[(int64_t)j * K + i] != i;
  __shared__ int red[256];
  red[threadIdx.x] = c;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) moved[j] = (double)red[0];
  if (j == 0)
    for (int i = threadIdx.x; i < n_sums; i += 256) sums[i] = 0.0;
}

struct OutWs {
  double* keys;
  int32_t* cands;
  int32_t* rank;
  float* y_ref;        // [n_batches][M][ldn]
  float* y_hat;        // [M][ldn]
  uint8_t* x_codes;
  void* x_scales;
  uint8_t* w_codes;
  void* w_scales;
  uint8_t* x_op;
  uint8_t* w_op;
  float* ts;           // [2] activation and weight tensor scale
  double* partial;     // [2 * kDiffBlocks]
  double* sums;        // [kMaxCandOut] numerators, [1] denominator, [PQ_MAX_ALPHAS] moved counts
};
constexpr int kMaxCandOut = PQ_MAX_ALPHAS + 1;
constexpr int kNumSums = kMaxCandOut + 1 + PQ_MAX_ALPHAS;

size_t scale_bytes(pq_format fmt, int group, int64_t rows, int64_t K) {
  return fmt == PQ_FMT_NVFP4 ? (size_t)rows * (K / 16) : (size_t)rows * (K / group) * 4;
}

size_t carve_out(void* base, pq_format fmt, int group, int64_t M, int64_t N, int64_t K, int n_batches, OutWs* w) {
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off = align_up(off + bytes, 256);
    return o;
  };
  const int64_t ldn = (N + 7) / 8 * 8;
  const size_t o_keys = take((size_t)PQ_MAX_ALPHAS * K * 8);
  const size_t o_cands = take((size_t)PQ_MAX_ALPHAS * K * 4);
  const size_t o_rank = take((size_t)PQ_MAX_ALPHAS * K * 4);
  const size_t o_ref = take((size_t)n_batches * M * ldn * 4);
  const size_t o_hat = take((size_t)M * ldn * 4);
  const size_t o_xc = take((size_t)M * K / 2);
  const size_t o_xs = take(scale_bytes(fmt, group, M, K));
  const size_t o_wc = take((size_t)N * K / 2);
  const size_t o_wsc = take(scale_bytes(fmt, group, N, K));
  const size_t o_xop = take(operand_bytes(fmt, group, M, K));
  const size_t o_wop = take(operand_bytes(fmt, group, N, K));
  const size_t o_ts = take(2 * sizeof(float));
  const size_t o_part = take((size_t)2 * kDiffBlocks * 8);
  const size_t o_sums = take((size_t)kNumSums * 8);
  if (w) {
    char* b = (char*)base;
    w->keys = (double*)(b + o_keys);
    w->cands = (int32_t*)(b + o_cands);
    w->rank = (int32_t*)(b + o_rank);
    w->y_ref = (float*)(b + o_ref);
    w->y_hat = (float*)(b + o_hat);
    w->x_codes = (uint8_t*)(b + o_xc);
    w->x_scales = b + o_xs;
    w->w_codes = (uint8_t*)(b + o_wc);
    w->w_scales = b + o_wsc;
    w->x_op = (uint8_t*)(b + o_xop);
    w->w_op = (uint8_t*)(b + o_wop);
    w->ts = (float*)(b + o_ts);
    w->partial = (double*)(b + o_part);
    w->sums = (double*)(b + o_sums);
  }
  return off;
}

}  // namespace

size_t select_output_workspace_bytes(pq_format fmt, int group, int64_t M, int64_t N, int64_t K, int n_batches) {
  return carve_out(nullptr, fmt, group, M, N, K, n_batches, nullptr);
}

int run_select_output(pq_format fmt, int group, const double* act_sumsq, const double* w_sumsq, int64_t K,
                      const void* const* x_calib, int n_batches, int64_t M, const void* w, int64_t N,
                      float act_ts, float w_ts, const double* alphas, int n_alpha, double tau,
                      int32_t* perm_out, pq_select_report* report, void* ws, hipStream_t st) {
  OutWs W;
  carve_out(ws, fmt, group, M, N, K, n_batches, &W);
  const int64_t ldn = (N + 7) / 8 * 8;
  const int n_cand = n_alpha + 1;              // candidate 0 is the original order
  int rc;
  if ((rc = launch_candidate_orders(act_sumsq, w_sumsq, K, alphas, n_alpha, W.keys, W.rank, W.cands, st))) return rc;
  hipLaunchKernelGGL(moved_kernel, dim3(n_alpha), dim3(256), 0, st, W.cands, (int)K, W.sums, kMaxCandOut + 1,
                     W.sums + kMaxCandOut + 1);
  if ((rc = check_hip(hipGetLastError(), "moved_kernel"))) return rc;
  if ((rc = launch_fill_float(W.ts, act_ts, st))) return rc;
  if ((rc = launch_fill_float(W.ts + 1, w_ts, st))) return rc;

  // the unquantized products, once
  const dim3 ref_grid((unsigned)((M + kRefTile - 1) / kRefTile), (unsigned)((N + kRefTile - 1) / kRefTile));
  for (int b = 0; b < n_batches; ++b) {
    hipLaunchKernelGGL(ref_gemm_kernel, ref_grid, dim3(256), 0, st, (const uint16_t*)x_calib[b], (const uint16_t*)w,
                       (int)M, (int)N, (int)K, W.y_ref + (size_t)b * M * ldn, ldn);
  }
  if ((rc = check_hip(hipGetLastError(), "ref_gemm_kernel"))) return rc;

  for (int c = 0; c < n_cand; ++c) {
    const int32_t* perm = c == 0 ? nullptr : W.cands + (int64_t)(c - 1) * K;
    // the tensor scale of the weights does not depend on the order: the caller's value is used
    if ((rc = launch_quantize_rows(fmt, group, w, N, K, K, perm, W.ts + 1, W.w_codes, W.w_scales, st))) return rc;
    if ((rc = run_pack_operand(fmt, group, W.w_codes, W.w_scales, N, K, W.w_op, false, st))) return rc;
    for (int b = 0; b < n_batches; ++b) {
      if ((rc = launch_quantize_rows(fmt, group, x_calib[b], M, K, K, perm, W.ts, W.x_codes, W.x_scales, st))) return rc;
      if ((rc = run_pack_operand(fmt, group, W.x_codes, W.x_scales, M, K, W.x_op, false, st))) return rc;
      if ((rc = run_qgemm_packed(fmt, group, W.x_op, W.ts, W.w_op, W.ts + 1, M, N, K, nullptr, W.y_hat, ldn, true, st)))
        return rc;
      hipLaunchKernelGGL(sqdiff_partial_kernel, dim3(kDiffBlocks), dim3(256), 0, st,
                         W.y_ref + (size_t)b * M * ldn, W.y_hat, M, (int)N, ldn, W.partial);
      hipLaunchKernelGGL(sqdiff_finish_kernel, dim3(1), dim3(64), 0, st, W.partial, W.sums + c,
                         c == 0 ? W.sums + kMaxCandOut : nullptr);
    }
    if ((rc = check_hip(hipGetLastError(), "sqdiff kernels"))) return rc;
  }

  double* h = pinned_doubles(kNumSums);
  if (!h) return fail(PQ_ERR_HIP, "pq_select_perm_output_error: no pinned host memory for the sums");
  if ((rc = check_hip(hipMemcpyAsync(h, W.sums, (size_t)kNumSums * 8, hipMemcpyDeviceToHost, st), "copy sums")))
    return rc;
  if ((rc = check_hip(hipStreamSynchronize(st), "hipStreamSynchronize"))) return rc;

  const double den = h[kMaxCandOut];
  double E[kMaxCandOut];
  for (int c = 0; c < n_cand; ++c) E[c] = h[c] / den;
  int best = 0;
  for (int j = 1; j < n_alpha; ++j)
    if (E[1 + j] < E[1 + best]) best = j;         // first minimum: smallest alpha on ties
  const double e_orig = E[0], e_best = E[1 + best];
  const bool accepted = h[kMaxCandOut + 1 + best] != 0.0 && e_orig > 0.0 && ((e_orig - e_best) / e_orig > tau);
  memset(report, 0, sizeof(*report));
  report->accepted = accepted ? 1 : 0;
  report->alpha_index = best;
  report->e_orig = e_orig;
  report->e_best = e_best;
  for (int j = 0; j < n_alpha; ++j) report->e_cand[j] = E[1 + j];
  report->sum_x2 = den;            // here: ||X W^T||^2 over the calibration batches
  report->sum_w2 = 0.0;
  if (accepted)
    return check_hip(hipMemcpyAsync(perm_out, W.cands + (int64_t)best * K, (size_t)K * 4, hipMemcpyDeviceToDevice, st),
                     "copy permutation");
  return launch_identity_order(perm_out, K, st);
}

}  // namespace pq
