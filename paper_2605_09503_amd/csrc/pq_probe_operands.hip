// Measurement aid: a matrix-pipe-only loop on the values the product kernel multiplies.
//
// The rate the matrix pipes sustain depends on the operand values: the chip runs into its power limit and
// lowers its clock, and how soon depends on the switching activity of the operands.  A loop that reuses
// one pair of constant fragments (pq_probe_mfma) therefore overstates what a GEMM on real data can reach.
// Here every lane unpacks eight fragments of the activation operand and four of the weight operand --
// with the product kernel's own loader and unpack code, from rows and K positions spread over the
// operands -- and the loop cycles through them, so that both MFMA inputs change from one instruction to
// the next.  No LDS, no vector work, no memory traffic inside the loop.
#include "pq_qgemm_common.h"

namespace pq {

template <int FMT, int G>
__global__ __launch_bounds__(512) void probe_mfma_operands_kernel(OperandView A, OperandView W, int M, int N,
                                                                 int K, int iters, float* __restrict__ sink) {
  const int t = threadIdx.x;
  const int ksteps = K / kBK;
  auto fragment = [&](const OperandView& V, int rows, int idx) {
    const int row = (int)(((int64_t)blockIdx.x * 64 + (t >> 3) + (int64_t)idx * 8191) % rows);
    const int step = (idx * 5 + (int)blockIdx.x) % ksteps;
    const Slice sl = load_slice<FMT, G>(V.codes + (int64_t)row * V.code_row, V.code_step,
                                        V.scales + (int64_t)row * V.sc_row, V.sc_step, K, step, t & 1);
    PairScale s0, s1;
    slice_scales<FMT>(sl, true, s0, s1);
    const int c = (t >> 1) & 3;
    const uint32_t d = c == 0 ? sl.codes.x : c == 1 ? sl.codes.y : c == 2 ? sl.codes.z : sl.codes.w;
    const PairScale& sc = c < 2 ? s0 : s1;
    return make_uint4(unpack_pair<FMT, 0>(d, sc), unpack_pair<FMT, 1>(d, sc), unpack_pair<FMT, 2>(d, sc),
                      unpack_pair<FMT, 3>(d, sc));
  };
  uint4 ra[8], rb[4];
#pragma unroll
  for (int i = 0; i < 8; ++i) ra[i] = fragment(A, M, i);
#pragma unroll
  for (int i = 0; i < 4; ++i) rb[i] = fragment(W, N, i);
  float16_t acc[8];
#pragma unroll
  for (int q = 0; q < 8; ++q)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[q][r] = 0.0f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int q = 0; q < 8; ++q)
      acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, rb[q & 3]),
                                                      __builtin_bit_cast(half8_t, ra[q]), acc[q], 0, 0, 0);
  }
  float s = 0.0f;
#pragma unroll
  for (int q = 0; q < 8; ++q)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[q][r];
  sink[(size_t)blockIdx.x * blockDim.x + t] = s;
}

template <int FMT, int G>
static int launch_fg(const OperandView& A, const OperandView& W, int M, int N, int K, int iters, float* sink,
                     hipStream_t st) {
  hipLaunchKernelGGL((probe_mfma_operands_kernel<FMT, G>), dim3(256), dim3(512), 0, st, A, W, M, N, K, iters, sink);
  return check_hip(hipGetLastError(), "probe_mfma_operands_kernel");
}

int launch_probe_mfma_operands(pq_format fmt, int group, const void* a_operand, const void* w_operand, int64_t M,
                               int64_t N, int64_t K, int iters, float* sink, double* flops_out, hipStream_t st) {
  const OperandView A = panel_view(fmt, group, a_operand, M, K, nullptr);
  const OperandView W = panel_view(fmt, group, w_operand, N, K, nullptr);
  if (flops_out) *flops_out = (double)iters * 8.0 * (2.0 * 32 * 32 * 16) * 8 * 256;
#define PQ_ARGS A, W, (int)M, (int)N, (int)K, iters, sink, st
  if (fmt == PQ_FMT_NVFP4) return launch_fg<kNvfp4, 16>(PQ_ARGS);
  if (fmt == PQ_FMT_INT4 || fmt == PQ_FMT_INT3) {
    const bool i4 = fmt == PQ_FMT_INT4;
    switch (group) {
      case 32: return i4 ? launch_fg<kInt4, 32>(PQ_ARGS) : launch_fg<kInt3, 32>(PQ_ARGS);
      case 64: return i4 ? launch_fg<kInt4, 64>(PQ_ARGS) : launch_fg<kInt3, 64>(PQ_ARGS);
      case 128: return i4 ? launch_fg<kInt4, 128>(PQ_ARGS) : launch_fg<kInt3, 128>(PQ_ARGS);
      case 256: return i4 ? launch_fg<kInt4, 256>(PQ_ARGS) : launch_fg<kInt3, 256>(PQ_ARGS);
    }
  }
#undef PQ_ARGS
  return fail(PQ_ERR_FORMAT, "unsupported (format, group) = (%d, %d)", (int)fmt, group);
}

}  // namespace pq
