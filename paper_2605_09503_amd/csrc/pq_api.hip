// C ABI entry points: host-side validation, then dispatch to the kernel launchers.
// Every check happens before anything is queued on the stream.
#include <stdio.h>
#include <string.h>

#include "pq_host.h"

namespace pq {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

int check_hip(hipError_t e, const char* what) {
  if (e == hipSuccess) return PQ_OK;
  return fail(PQ_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

int check_format(pq_format fmt, int group, int64_t K) {
  if (fmt != PQ_FMT_NVFP4 && fmt != PQ_FMT_INT4 && fmt != PQ_FMT_INT3)
    return fail(PQ_ERR_FORMAT, "unknown format %d", (int)fmt);
  if (fmt == PQ_FMT_NVFP4) {
    if (group != 16) return fail(PQ_ERR_FORMAT, "NVFP4 uses groups of 16, got %d", group);
  } else if (group != 32 && group != 64 && group != 128 && group != 256) {
    return fail(PQ_ERR_FORMAT, "INT formats offer group 32, 64, 128 or 256, got %d", group);
  }
  if (K <= 0) return fail(PQ_ERR_SHAPE, "K must be positive, got %lld", (long long)K);
  if (K % group) return fail(PQ_ERR_SHAPE, "K=%lld is not a multiple of group=%d", (long long)K, group);
  return PQ_OK;
}

}  // namespace pq

using namespace pq;

extern "C" {

const char* pq_last_error(void) { return g_err; }

int pq_version(void) { return 100; }

size_t pq_workspace_bytes(pq_op op, pq_format fmt, int group, int64_t M, int64_t N, int64_t K,
                          int n_batches) {
  switch (op) {
    case PQ_OP_CALIB_MOMENTS:
      if (M <= 0 || K <= 0) return 0;
      return moments_workspace_bytes(M, K, n_batches);
    case PQ_OP_SELECT_PERM:
      if (M <= 0 || N <= 0 || K <= 0 || K > kSelectMaxK || n_batches <= 0) return 0;
      return select_workspace_bytes(M, N, K, n_batches);
    case PQ_OP_QUANT_ERROR:
      if (M <= 0 || K > kSelectMaxK) return 0;
      return quant_error_workspace_bytes(M, K);
    case PQ_OP_CHANNEL_STATS:
      if (M <= 0 || K <= 0) return 0;
      return channel_stats_workspace_bytes(M, K);
    case PQ_OP_ORDER:
      if (K <= 0) return 0;
      return random_order_workspace_bytes(K);
    case PQ_OP_SELECT_PERM_OUTPUT:
      if (M <= 0 || N <= 0 || K <= 0 || n_batches <= 0 || check_format(fmt, group, K) || K % 32) return 0;
      return select_output_workspace_bytes(fmt, group, M, N, K, n_batches);
    case PQ_OP_QGEMM:
      if (M <= 0 || N <= 0 || K <= 0 || group <= 0) return 0;
      return qgemm_workspace_bytes(fmt, group, M, N, K);
    default:
      return 0;
  }
}

static int calib_moments_check(const char* who, const void* const* xs, int n_batches, int64_t rows,
                               int64_t K, int64_t ld, double* sumsq) {
  if (!xs || !sumsq) return fail(PQ_ERR_NULL, "%s: x and sumsq must not be NULL", who);
  if (n_batches <= 0) return fail(PQ_ERR_SHAPE, "%s: n_batches=%d must be positive", who, n_batches);
  if (rows <= 0 || K <= 0) return fail(PQ_ERR_SHAPE, "%s: rows=%lld K=%lld must be positive", who,
                                        (long long)rows, (long long)K);
  if (K % 8 || ld % 8) return fail(PQ_ERR_SHAPE, "%s: K=%lld and ld=%lld must be multiples of 8", who,
                                   (long long)K, (long long)ld);
  if (ld < K) return fail(PQ_ERR_SHAPE, "%s: ld=%lld < K=%lld", who, (long long)ld, (long long)K);
  for (int b = 0; b < n_batches; ++b) {
    if (!xs[b]) return fail(PQ_ERR_NULL, "%s: batch %d is NULL", who, b);
    if (!aligned16(xs[b])) return fail(PQ_ERR_SHAPE, "%s: batch %d must be 16-byte aligned", who, b);
  }
  return PQ_OK;
}

static int calib_moments_common(const char* who, const void* const* xs, int n_batches, int64_t rows,
                                int64_t K, int64_t ld, double* sumsq, float* absmax, void* workspace,
                                size_t workspace_bytes, void* stream) {
  int rc = calib_moments_check(who, xs, n_batches, rows, K, ld, sumsq);
  if (rc) return rc;
  size_t need = moments_workspace_bytes(rows, K, n_batches);
  if (!workspace || workspace_bytes < need)
    return fail(PQ_ERR_WORKSPACE, "%s: workspace of %zu bytes needed, %zu given", who, need,
                workspace ? workspace_bytes : (size_t)0);
  return launch_moments(xs, n_batches, rows, K, ld, sumsq, absmax, workspace, as_stream(stream));
}

int pq_calib_moments(const void* x, int64_t rows, int64_t K, int64_t ld, double* sumsq,
                     float* absmax, void* workspace, size_t workspace_bytes, void* stream) {
  const void* xs[1] = {x};
  return calib_moments_common("pq_calib_moments", x ? xs : nullptr, 1, rows, K, ld, sumsq, absmax,
                              workspace, workspace_bytes, stream);
}

int pq_calib_moments_static(const void* x, int64_t rows, int64_t K, int64_t ld, double* sumsq, float* absmax,
                            void* stream) {
  const void* xs[1] = {x};
  int rc = calib_moments_check("pq_calib_moments_static", x ? xs : nullptr, 1, rows, K, ld, sumsq);
  if (rc) return rc;
  return launch_moments_static(x, rows, K, ld, sumsq, absmax, as_stream(stream));
}

int pq_calib_moments_batched(const void* const* x_batches, int n_batches, int64_t rows, int64_t K,
                             int64_t ld, double* sumsq, float* absmax, void* workspace,
                             size_t workspace_bytes, void* stream) {
  return calib_moments_common("pq_calib_moments_batched", x_batches, n_batches, rows, K, ld, sumsq,
                              absmax, workspace, workspace_bytes, stream);
}

int pq_tensor_scale(const float* absmax, float* tensor_scale_out, void* stream) {
  if (!absmax || !tensor_scale_out) return fail(PQ_ERR_NULL, "pq_tensor_scale: NULL pointer");
  return launch_tensor_scale(absmax, tensor_scale_out, as_stream(stream));
}

static int select_common(bool output_metric, pq_format fmt, int group, const double* act_sumsq,
                         const double* w_sumsq, int64_t K, const void* const* x_calib, int n_batches, int64_t M,
                         const void* w_bf16, int64_t N, float act_tensor_scale, float w_tensor_scale,
                         const double* alphas, int n_alpha, double tau, int32_t* perm_out,
                         pq_select_report* report, void* workspace, size_t workspace_bytes, void* stream,
                         const float* act_ts_dev = nullptr, const float* w_ts_dev = nullptr) {
  const char* who = output_metric ? "pq_select_perm_output_error" : "pq_select_perm";
  if (!act_sumsq || !w_sumsq || !x_calib || !w_bf16 || !alphas || !perm_out || !report)
    return fail(PQ_ERR_NULL, "%s: a required pointer is NULL", who);
  int rc = check_format(fmt, group, K);
  if (rc) return rc;
  if (M <= 0 || N <= 0) return fail(PQ_ERR_SHAPE, "%s: M=%lld N=%lld must be positive", who, (long long)M, (long long)N);
  if (n_batches <= 0) return fail(PQ_ERR_SHAPE, "%s: n_batches=%d must be positive", who, n_batches);
  if (n_alpha <= 0 || n_alpha > PQ_MAX_ALPHAS)
    return fail(PQ_ERR_SHAPE, "%s: n_alpha=%d outside 1..%d", who, n_alpha, PQ_MAX_ALPHAS);
  if (K > (output_metric ? 65536 : kSelectMaxK))
    return fail(PQ_ERR_SHAPE, "%s: K=%lld above the supported %lld%s", who, (long long)K,
                (long long)(output_metric ? 65536 : kSelectMaxK),
                output_metric ? "" : " (a row must fit the error evaluation's LDS)");
  if (output_metric && K % 32) return fail(PQ_ERR_SHAPE, "%s: K=%lld must be a multiple of 32", who, (long long)K);
  if (output_metric && (M > (1 << 24) || N > (1 << 24))) return fail(PQ_ERR_SHAPE, "%s: a dimension exceeds 2^24", who);
  for (int j = 0; j < n_alpha; ++j)
    if (!(alphas[j] >= 0.0 && alphas[j] <= 1.0))
      return fail(PQ_ERR_SHAPE, "%s: alphas[%d]=%g outside [0, 1]", who, j, alphas[j]);
  if (!(tau == tau)) return fail(PQ_ERR_SHAPE, "%s: tau is NaN", who);
  for (int b = 0; b < n_batches; ++b) {
    if (!x_calib[b]) return fail(PQ_ERR_NULL, "%s: x_calib[%d] is NULL", who, b);
    if (!aligned16(x_calib[b])) return fail(PQ_ERR_SHAPE, "%s: x_calib[%d] must be 16-byte aligned", who, b);
  }
  if (!aligned16(w_bf16)) return fail(PQ_ERR_SHAPE, "%s: w must be 16-byte aligned", who);
  const size_t need = output_metric ? select_output_workspace_bytes(fmt, group, M, N, K, n_batches)
                                    : select_workspace_bytes(M, N, K, n_batches);
  if (!workspace || workspace_bytes < need)
    return fail(PQ_ERR_WORKSPACE, "%s: workspace of %zu bytes needed, %zu given", who, need,
                workspace ? workspace_bytes : (size_t)0);
  if (output_metric)
    return run_select_output(fmt, group, act_sumsq, w_sumsq, K, x_calib, n_batches, M, w_bf16, N, act_tensor_scale,
                             w_tensor_scale, alphas, n_alpha, tau, perm_out, report, workspace, as_stream(stream));
  return run_select(fmt, group, act_sumsq, w_sumsq, K, x_calib, n_batches, M, w_bf16, N,
                    act_tensor_scale, w_tensor_scale, act_ts_dev, w_ts_dev, alphas, n_alpha, tau, perm_out, report,
                    workspace, as_stream(stream));
}

int pq_select_perm_device_scales(pq_format fmt, int group, const double* act_sumsq, const double* w_sumsq,
                                 int64_t K, const void* const* x_calib, int n_batches, int64_t M,
                                 const void* w_bf16, int64_t N, const float* act_tensor_scale,
                                 const float* w_tensor_scale, const double* alphas, int n_alpha, double tau,
                                 int32_t* perm_out, pq_select_report* report, void* workspace,
                                 size_t workspace_bytes, void* stream) {
  if (fmt == PQ_FMT_NVFP4 && (!act_tensor_scale || !w_tensor_scale))
    return fail(PQ_ERR_NULL, "pq_select_perm_device_scales: NVFP4 needs both tensor scales");
  const bool nv = fmt == PQ_FMT_NVFP4;
  return select_common(false, fmt, group, act_sumsq, w_sumsq, K, x_calib, n_batches, M, w_bf16, N, 1.0f, 1.0f,
                       alphas, n_alpha, tau, perm_out, report, workspace, workspace_bytes, stream,
                       nv ? act_tensor_scale : nullptr, nv ? w_tensor_scale : nullptr);
}

int pq_select_perm(pq_format fmt, int group, const double* act_sumsq, const double* w_sumsq,
                   int64_t K, const void* const* x_calib, int n_batches, int64_t M,
                   const void* w_bf16, int64_t N, float act_tensor_scale, float w_tensor_scale,
                   const double* alphas, int n_alpha, double tau, int32_t* perm_out,
                   pq_select_report* report, void* workspace, size_t workspace_bytes,
                   void* stream) {
  return select_common(false, fmt, group, act_sumsq, w_sumsq, K, x_calib, n_batches, M, w_bf16, N,
                       act_tensor_scale, w_tensor_scale, alphas, n_alpha, tau, perm_out, report, workspace,
                       workspace_bytes, stream);
}

int pq_select_perm_output_error(pq_format fmt, int group, const double* act_sumsq, const double* w_sumsq,
                                int64_t K, const void* const* x_calib, int n_batches, int64_t M,
                                const void* w_bf16, int64_t N, float act_tensor_scale, float w_tensor_scale,
                                const double* alphas, int n_alpha, double tau, int32_t* perm_out,
                                pq_select_report* report, void* workspace, size_t workspace_bytes,
                                void* stream) {
  return select_common(true, fmt, group, act_sumsq, w_sumsq, K, x_calib, n_batches, M, w_bf16, N,
                       act_tensor_scale, w_tensor_scale, alphas, n_alpha, tau, perm_out, report, workspace,
                       workspace_bytes, stream);
}

int pq_quant_error(pq_format fmt, int group, const void* x, int64_t rows, int64_t K,
                   const int32_t* perm, float tensor_scale, double* err_out, void* workspace,
                   size_t workspace_bytes, void* stream) {
  if (!x || !err_out) return fail(PQ_ERR_NULL, "pq_quant_error: x and err_out must not be NULL");
  int rc = check_format(fmt, group, K);
  if (rc) return rc;
  if (rows <= 0) return fail(PQ_ERR_SHAPE, "pq_quant_error: rows=%lld must be positive", (long long)rows);
  if (K > kSelectMaxK)
    return fail(PQ_ERR_SHAPE, "pq_quant_error: K=%lld above the supported %lld (a row must fit the kernel's LDS)",
                (long long)K, (long long)kSelectMaxK);
  if (!aligned16(x)) return fail(PQ_ERR_SHAPE, "pq_quant_error: x must be 16-byte aligned");
  size_t need = quant_error_workspace_bytes(rows, K);
  if (!workspace || workspace_bytes < need)
    return fail(PQ_ERR_WORKSPACE, "pq_quant_error: workspace of %zu bytes needed, %zu given", need,
                workspace ? workspace_bytes : (size_t)0);
  return run_quant_error(fmt, group, x, rows, K, perm, tensor_scale, err_out, workspace,
                         as_stream(stream));
}

int pq_quantize_weights(pq_format fmt, int group, const void* w, int64_t N, int64_t K,
                        const int32_t* perm, uint8_t* codes, void* scales, float* tensor_scale_out,
                        void* stream) {
  if (!w || !codes || !scales || !tensor_scale_out)
    return fail(PQ_ERR_NULL, "pq_quantize_weights: a required pointer is NULL");
  int rc = check_format(fmt, group, K);
  if (rc) return rc;
  if (N <= 0) return fail(PQ_ERR_SHAPE, "pq_quantize_weights: N=%lld must be positive", (long long)N);
  if (!aligned16(w) || !aligned16(codes) || !aligned16(scales))
    return fail(PQ_ERR_SHAPE, "pq_quantize_weights: tensors must be 16-byte aligned");
  hipStream_t st = as_stream(stream);
  if (fmt == PQ_FMT_NVFP4) {
    rc = launch_absmax_to_tensor_scale(w, N * K, tensor_scale_out, st);
  } else {
    rc = launch_fill_float(tensor_scale_out, 1.0f, st);
  }
  if (rc) return rc;
  return launch_quantize_rows(fmt, group, w, N, K, K, perm, tensor_scale_out, codes, scales, st);
}

int pq_quantize_act(pq_format fmt, int group, const void* x, int64_t M, int64_t K, int64_t ld,
                    const int32_t* perm, const float* tensor_scale, uint8_t* codes, void* scales,
                    void* stream) {
  if (!x || !codes || !scales) return fail(PQ_ERR_NULL, "pq_quantize_act: a required pointer is NULL");
  int rc = check_format(fmt, group, K);
  if (rc) return rc;
  if (fmt == PQ_FMT_NVFP4 && !tensor_scale)
    return fail(PQ_ERR_NULL, "pq_quantize_act: NVFP4 needs the per-tensor scale");
  if (M <= 0) return fail(PQ_ERR_SHAPE, "pq_quantize_act: M=%lld must be positive", (long long)M);
  if (ld < K || ld % 8)
    return fail(PQ_ERR_SHAPE, "pq_quantize_act: ld=%lld must be >= K=%lld and a multiple of 8",
                (long long)ld, (long long)K);
  if (!aligned16(x) || !aligned16(codes) || !aligned16(scales))
    return fail(PQ_ERR_SHAPE, "pq_quantize_act: tensors must be 16-byte aligned");
  return launch_quantize_rows(fmt, group, x, M, K, ld, perm, tensor_scale, codes, scales,
                              as_stream(stream));
}

static int qgemm_common(pq_format fmt, int group, const uint8_t* a_codes, const void* a_scales,
                        const float* a_ts, const uint8_t* w_codes, const void* w_scales,
                        const float* w_ts, int64_t M, int64_t N, int64_t K, void* y, int64_t ldy,
                        bool out_f32, int phases, void* workspace, size_t workspace_bytes,
                        void* stream) {
  const bool need_codes = (phases & 2) != 0;
  if (!a_scales || !w_scales || (need_codes && (!a_codes || !w_codes || !y)))
    return fail(PQ_ERR_NULL, "pq_qgemm: a required pointer is NULL");
  int rc = check_format(fmt, group, K);
  if (rc) return rc;
  if (fmt == PQ_FMT_NVFP4 && need_codes && (!a_ts || !w_ts))
    return fail(PQ_ERR_NULL, "pq_qgemm: NVFP4 needs both per-tensor scales");
  if (M <= 0 || N <= 0) return fail(PQ_ERR_SHAPE, "pq_qgemm: M=%lld N=%lld must be positive",
                                    (long long)M, (long long)N);
  if (K % 32) return fail(PQ_ERR_SHAPE, "pq_qgemm: K=%lld must be a multiple of 32", (long long)K);
  if (M > (1 << 24) || N > (1 << 24) || K > (1 << 24))
    return fail(PQ_ERR_SHAPE, "pq_qgemm: a dimension exceeds 2^24");
  if (need_codes && (ldy < N || ldy % 8))
    return fail(PQ_ERR_SHAPE, "pq_qgemm: ldy=%lld must be >= N=%lld and a multiple of 8",
                (long long)ldy, (long long)N);
  if (!aligned16(a_codes) || !aligned16(w_codes) || !aligned16(a_scales) || !aligned16(w_scales) ||
      !aligned16(y))
    return fail(PQ_ERR_SHAPE, "pq_qgemm: tensors must be 16-byte aligned");
  size_t need = qgemm_workspace_bytes(fmt, group, M, N, K);
  if (need && (!workspace || workspace_bytes < need))
    return fail(PQ_ERR_WORKSPACE, "pq_qgemm: workspace of %zu bytes needed, %zu given", need,
                workspace ? workspace_bytes : (size_t)0);
  if (need && !aligned16(workspace)) return fail(PQ_ERR_SHAPE, "pq_qgemm: workspace must be 16-byte aligned");
  return run_qgemm(fmt, group, a_codes, a_scales, a_ts, w_codes, w_scales, w_ts, M, N, K, y, ldy,
                   out_f32, phases, workspace, as_stream(stream));
}

int pq_qgemm(pq_format fmt, int group, const uint8_t* a_codes, const void* a_scales,
             const float* a_tensor_scale, const uint8_t* w_codes, const void* w_scales,
             const float* w_tensor_scale, int64_t M, int64_t N, int64_t K, void* y_bf16, int64_t ldy,
             void* workspace, size_t workspace_bytes, void* stream) {
  return qgemm_common(fmt, group, a_codes, a_scales, a_tensor_scale, w_codes, w_scales,
                      w_tensor_scale, M, N, K, y_bf16, ldy, false, 3, workspace, workspace_bytes, stream);
}

int pq_qgemm_prep(pq_format fmt, int group, const void* a_scales, const void* w_scales, int64_t M,
                  int64_t N, int64_t K, void* workspace, size_t workspace_bytes, void* stream) {
  return qgemm_common(fmt, group, nullptr, a_scales, nullptr, nullptr, w_scales, nullptr, M, N, K, nullptr,
                      0, false, 1, workspace, workspace_bytes, stream);
}

int pq_qgemm_run(pq_format fmt, int group, const uint8_t* a_codes, const void* a_scales,
                 const float* a_tensor_scale, const uint8_t* w_codes, const void* w_scales,
                 const float* w_tensor_scale, int64_t M, int64_t N, int64_t K, void* y_bf16, int64_t ldy,
                 void* workspace, size_t workspace_bytes, void* stream) {
  return qgemm_common(fmt, group, a_codes, a_scales, a_tensor_scale, w_codes, w_scales,
                      w_tensor_scale, M, N, K, y_bf16, ldy, false, 2, workspace, workspace_bytes, stream);
}

int pq_qgemm_f32(pq_format fmt, int group, const uint8_t* a_codes, const void* a_scales,
                 const float* a_tensor_scale, const uint8_t* w_codes, const void* w_scales,
                 const float* w_tensor_scale, int64_t M, int64_t N, int64_t K, float* y_f32,
                 int64_t ldy, void* workspace, size_t workspace_bytes, void* stream) {
  return qgemm_common(fmt, group, a_codes, a_scales, a_tensor_scale, w_codes, w_scales,
                      w_tensor_scale, M, N, K, y_f32, ldy, true, 3, workspace, workspace_bytes, stream);
}

size_t pq_operand_bytes(pq_format fmt, int group, int64_t rows, int64_t K) {
  if (check_format(fmt, group, K) || rows <= 0 || K % 32) return 0;
  return operand_bytes(fmt, group, rows, K);
}

static int pack_operand_common(const char* name, pq_format fmt, int group, const uint8_t* codes, const void* scales,
                               int64_t rows, int64_t K, void* operand, size_t operand_size, bool dense3,
                               void* stream) {
  if (!codes || !scales || !operand) return fail(PQ_ERR_NULL, "%s: a required pointer is NULL", name);
  int rc = check_format(fmt, group, K);
  if (rc) return rc;
  if (rows <= 0) return fail(PQ_ERR_SHAPE, "%s: rows=%lld must be positive", name, (long long)rows);
  if (K % 32) return fail(PQ_ERR_SHAPE, "%s: K=%lld must be a multiple of 32", name, (long long)K);
  if (rows > (1 << 24) || K > (1 << 24)) return fail(PQ_ERR_SHAPE, "%s: a dimension exceeds 2^24", name);
  if (!aligned16(codes) || !aligned16(scales) || !aligned16(operand))
    return fail(PQ_ERR_SHAPE, "%s: buffers must be 16-byte aligned", name);
  const size_t need = operand_bytes(fmt, group, rows, K);
  if (operand_size < need)
    return fail(PQ_ERR_WORKSPACE, "%s: operand buffer of %zu bytes needed, %zu given", name, need, operand_size);
  return run_pack_operand(fmt, group, codes, scales, rows, K, operand, dense3, as_stream(stream));
}

int pq_pack_operand(pq_format fmt, int group, const uint8_t* codes, const void* scales, int64_t rows,
                    int64_t K, void* operand, size_t operand_size, void* stream) {
  return pack_operand_common("pq_pack_operand", fmt, group, codes, scales, rows, K, operand, operand_size, false,
                             stream);
}

int pq_pack_operand_int3(int group, const uint8_t* dense, const void* scales, int64_t rows, int64_t K,
                         void* operand, size_t operand_size, void* stream) {
  return pack_operand_common("pq_pack_operand_int3", PQ_FMT_INT3, group, dense, scales, rows, K, operand,
                             operand_size, true, stream);
}

size_t pq_int3_dense_bytes(int64_t rows, int64_t K) {
  if (rows <= 0 || K <= 0 || K % 32 || rows > (1 << 24) || K > (1 << 24)) return 0;
  return (size_t)rows * (size_t)(K / 8 * 3);
}

static int int3_common(const char* name, const void* src, void* dst, int64_t rows, int64_t K) {
  if (!src || !dst) return fail(PQ_ERR_NULL, "%s: a required pointer is NULL", name);
  if (rows <= 0) return fail(PQ_ERR_SHAPE, "%s: rows=%lld must be positive", name, (long long)rows);
  if (K <= 0 || K % 32) return fail(PQ_ERR_SHAPE, "%s: K=%lld must be a positive multiple of 32", name, (long long)K);
  if (rows > (1 << 24) || K > (1 << 24)) return fail(PQ_ERR_SHAPE, "%s: a dimension exceeds 2^24", name);
  if (!aligned16(src) || !aligned16(dst)) return fail(PQ_ERR_SHAPE, "%s: buffers must be 16-byte aligned", name);
  return PQ_OK;
}

int pq_int3_pack(const uint8_t* codes, int64_t rows, int64_t K, uint8_t* dense, void* stream) {
  int rc = int3_common("pq_int3_pack", codes, dense, rows, K);
  if (rc) return rc;
  return launch_int3_pack(codes, rows, K, dense, as_stream(stream));
}

int pq_int3_unpack(const uint8_t* dense, int64_t rows, int64_t K, uint8_t* codes, void* stream) {
  int rc = int3_common("pq_int3_unpack", dense, codes, rows, K);
  if (rc) return rc;
  return launch_int3_unpack(dense, rows, K, codes, as_stream(stream));
}

int pq_quantize_act_packed(pq_format fmt, int group, const void* x, int64_t M, int64_t K, int64_t ld,
                           const float* tensor_scale, void* operand, size_t operand_size,
                           uint8_t* codes, void* scales, void* stream) {
  if (!x || !operand) return fail(PQ_ERR_NULL, "pq_quantize_act_packed: a required pointer is NULL");
  if ((codes == nullptr) != (scales == nullptr))
    return fail(PQ_ERR_NULL, "pq_quantize_act_packed: give both of codes and scales or neither");
  int rc = check_format(fmt, group, K);
  if (rc) return rc;
  if (fmt == PQ_FMT_NVFP4 && !tensor_scale)
    return fail(PQ_ERR_NULL, "pq_quantize_act_packed: NVFP4 needs the per-tensor scale");
  if (M <= 0) return fail(PQ_ERR_SHAPE, "pq_quantize_act_packed: M=%lld must be positive", (long long)M);
  if (K % 32) return fail(PQ_ERR_SHAPE, "pq_quantize_act_packed: K=%lld must be a multiple of 32", (long long)K);
  if (M > (1 << 24) || K > (1 << 24)) return fail(PQ_ERR_SHAPE, "pq_quantize_act_packed: a dimension exceeds 2^24");
  if (ld < K || ld % 8)
    return fail(PQ_ERR_SHAPE, "pq_quantize_act_packed: ld=%lld must be >= K=%lld and a multiple of 8",
                (long long)ld, (long long)K);
  if (!aligned16(x) || !aligned16(operand) || !aligned16(codes) || !aligned16(scales))
    return fail(PQ_ERR_SHAPE, "pq_quantize_act_packed: buffers must be 16-byte aligned");
  const size_t need = operand_bytes(fmt, group, M, K);
  if (operand_size < need)
    return fail(PQ_ERR_WORKSPACE, "pq_quantize_act_packed: operand buffer of %zu bytes needed, %zu given", need,
                operand_size);
  return run_quantize_packed(fmt, group, x, M, K, ld, tensor_scale, operand, codes, scales, as_stream(stream));
}

int pq_calib_channel_stats(const void* x, int64_t rows, int64_t K, int64_t ld, double* sum, float* absmax,
                           void* workspace, size_t workspace_bytes, void* stream) {
  if (!x || (!sum && !absmax)) return fail(PQ_ERR_NULL, "pq_calib_channel_stats: x and one of sum, absmax are required");
  if (rows <= 0 || K <= 0) return fail(PQ_ERR_SHAPE, "pq_calib_channel_stats: rows=%lld K=%lld must be positive",
                                        (long long)rows, (long long)K);
  if (rows > (1 << 24) || K > (1 << 24)) return fail(PQ_ERR_SHAPE, "pq_calib_channel_stats: a dimension exceeds 2^24");
  if (K % 8 || ld < K || ld % 8)
    return fail(PQ_ERR_SHAPE, "pq_calib_channel_stats: K=%lld must be a multiple of 8, ld=%lld >= K and a multiple of 8",
                (long long)K, (long long)ld);
  if (!aligned16(x)) return fail(PQ_ERR_SHAPE, "pq_calib_channel_stats: x must be 16-byte aligned");
  const size_t need = channel_stats_workspace_bytes(rows, K);
  if (!workspace || workspace_bytes < need)
    return fail(PQ_ERR_WORKSPACE, "pq_calib_channel_stats: workspace of %zu bytes needed, %zu given", need,
                workspace ? workspace_bytes : (size_t)0);
  return launch_channel_stats(x, rows, K, ld, sum, absmax, workspace, as_stream(stream));
}

int pq_channel_statistic(pq_criterion kind, const double* sum, const double* sumsq, const float* absmax,
                         int64_t n_rows, int64_t K, double* out, void* stream) {
  if (!out) return fail(PQ_ERR_NULL, "pq_channel_statistic: out is NULL");
  if (K <= 0) return fail(PQ_ERR_SHAPE, "pq_channel_statistic: K=%lld must be positive", (long long)K);
  if (kind == PQ_CRIT_VARIANCE) {
    if (!sum || !sumsq) return fail(PQ_ERR_NULL, "pq_channel_statistic: the variance needs sum and sumsq");
    if (n_rows <= 0) return fail(PQ_ERR_SHAPE, "pq_channel_statistic: n_rows=%lld must be positive", (long long)n_rows);
    return launch_channel_variance(sum, sumsq, n_rows, K, out, as_stream(stream));
  }
  if (kind == PQ_CRIT_ABSMAX) {
    if (!absmax) return fail(PQ_ERR_NULL, "pq_channel_statistic: the absmax criterion needs absmax");
    return launch_channel_absmax_sq(absmax, K, out, as_stream(stream));
  }
  return fail(PQ_ERR_FORMAT, "pq_channel_statistic: unknown criterion %d", (int)kind);
}

static int check_order_ws(const char* who, int64_t K, const int32_t* perm_out, const void* workspace,
                          size_t workspace_bytes) {
  if (!perm_out) return fail(PQ_ERR_NULL, "%s: perm_out is NULL", who);
  if (K <= 0 || K > 65536) return fail(PQ_ERR_SHAPE, "%s: K=%lld outside 1..65536", who, (long long)K);
  const size_t need = random_order_workspace_bytes(K);
  if (!workspace || workspace_bytes < need)
    return fail(PQ_ERR_WORKSPACE, "%s: workspace of %zu bytes needed, %zu given", who, need,
                workspace ? workspace_bytes : (size_t)0);
  return PQ_OK;
}

int pq_order_by_score(const double* act_stat, const double* w_stat, int64_t K, double alpha, int32_t* perm_out,
                      void* workspace, size_t workspace_bytes, void* stream) {
  if (!act_stat || !w_stat) return fail(PQ_ERR_NULL, "pq_order_by_score: a statistic array is NULL");
  int rc = check_order_ws("pq_order_by_score", K, perm_out, workspace, workspace_bytes);
  if (rc) return rc;
  if (!(alpha >= 0.0 && alpha <= 1.0)) return fail(PQ_ERR_SHAPE, "pq_order_by_score: alpha=%g outside [0, 1]", alpha);
  double* keys = (double*)workspace;
  int32_t* rank = (int32_t*)((char*)workspace + align_up((size_t)K * 8, 256));
  return launch_candidate_orders(act_stat, w_stat, K, &alpha, 1, keys, rank, perm_out, as_stream(stream));
}

int pq_order_round_robin(const int32_t* order, int64_t K, int group, int32_t* perm_out, void* stream) {
  if (!order || !perm_out) return fail(PQ_ERR_NULL, "pq_order_round_robin: a required pointer is NULL");
  if (order == perm_out) return fail(PQ_ERR_SHAPE, "pq_order_round_robin: order and perm_out must differ");
  if (K <= 0 || group <= 0 || K % group)
    return fail(PQ_ERR_SHAPE, "pq_order_round_robin: K=%lld must be a positive multiple of group=%d", (long long)K, group);
  if (K > (1 << 24)) return fail(PQ_ERR_SHAPE, "pq_order_round_robin: K exceeds 2^24");
  return launch_round_robin(order, K, group, perm_out, as_stream(stream));
}

int pq_order_random(uint64_t seed, int64_t K, int32_t* perm_out, void* workspace, size_t workspace_bytes,
                    void* stream) {
  int rc = check_order_ws("pq_order_random", K, perm_out, workspace, workspace_bytes);
  if (rc) return rc;
  return launch_random_order(seed, K, perm_out, workspace, as_stream(stream));
}

int pq_dynamic_tensor_scale(const void* x, int64_t M, int64_t K, int64_t ld, float* tensor_scale_out,
                            void* stream) {
  if (!x || !tensor_scale_out) return fail(PQ_ERR_NULL, "pq_dynamic_tensor_scale: a required pointer is NULL");
  if (M <= 0 || K <= 0) return fail(PQ_ERR_SHAPE, "pq_dynamic_tensor_scale: M=%lld K=%lld must be positive",
                                    (long long)M, (long long)K);
  if (M > (1 << 24) || K > (1 << 24)) return fail(PQ_ERR_SHAPE, "pq_dynamic_tensor_scale: a dimension exceeds 2^24");
  if (K % 8 || ld < K || ld % 8)
    return fail(PQ_ERR_SHAPE, "pq_dynamic_tensor_scale: K=%lld must be a multiple of 8, ld=%lld >= K and a multiple of 8",
                (long long)K, (long long)ld);
  if (!aligned16(x)) return fail(PQ_ERR_SHAPE, "pq_dynamic_tensor_scale: x must be 16-byte aligned");
  return launch_dynamic_tensor_scale(x, M, K, ld, tensor_scale_out, as_stream(stream));
}

static int check_norm(const char* who, const pq_norm_params* p, const void* x, int64_t M, int64_t K, int64_t ld,
                      const void* y, int64_t ldy, bool y_required) {
  if (!p || !x || (y_required && !y)) return fail(PQ_ERR_NULL, "%s: a required pointer is NULL", who);
  if (p->kind != PQ_NORM_RMS && p->kind != PQ_NORM_ADALN)
    return fail(PQ_ERR_FORMAT, "%s: unknown normalisation kind %d", who, (int)p->kind);
  if (M <= 0 || K <= 0) return fail(PQ_ERR_SHAPE, "%s: M=%lld K=%lld must be positive", who, (long long)M, (long long)K);
  if (M > (1 << 24) || K > (1 << 24)) return fail(PQ_ERR_SHAPE, "%s: a dimension exceeds 2^24", who);
  if (K % 8 || ld < K || ld % 8)
    return fail(PQ_ERR_SHAPE, "%s: K=%lld must be a multiple of 8, ld=%lld >= K and a multiple of 8", who,
                (long long)K, (long long)ld);
  if (y && (ldy < K || ldy % 8))
    return fail(PQ_ERR_SHAPE, "%s: ldy=%lld must be >= K=%lld and a multiple of 8", who, (long long)ldy, (long long)K);
  if (!(p->eps >= 0.0f)) return fail(PQ_ERR_SHAPE, "%s: eps must be non-negative", who);
  if (!aligned16(x) || !aligned16(y) || !aligned16(p->perm) || !aligned16(p->gamma) ||
      !aligned16(p->mod_scale) || !aligned16(p->mod_shift))
    return fail(PQ_ERR_SHAPE, "%s: buffers must be 16-byte aligned", who);
  return PQ_OK;
}

int pq_norm_reorder(const pq_norm_params* p, const void* x, int64_t M, int64_t K, int64_t ld, void* y,
                    int64_t ldy, void* stream) {
  int rc = check_norm("pq_norm_reorder", p, x, M, K, ld, y, ldy, true);
  if (rc) return rc;
  return run_norm_reorder(*p, x, M, K, ld, y, ldy, as_stream(stream));
}

int pq_norm_quantize_act_packed(const pq_norm_params* p, pq_format fmt, int group, const void* x, int64_t M,
                                int64_t K, int64_t ld, const float* tensor_scale, void* operand,
                                size_t operand_size, void* y, int64_t ldy, void* stream) {
  const char* who = "pq_norm_quantize_act_packed";
  int rc = check_norm(who, p, x, M, K, ld, y, ldy, false);
  if (rc) return rc;
  if (!operand) return fail(PQ_ERR_NULL, "%s: operand is NULL", who);
  rc = check_format(fmt, group, K);
  if (rc) return rc;
  if (fmt == PQ_FMT_NVFP4 && !tensor_scale) return fail(PQ_ERR_NULL, "%s: NVFP4 needs the per-tensor scale", who);
  if (K % 32) return fail(PQ_ERR_SHAPE, "%s: K=%lld must be a multiple of 32", who, (long long)K);
  if (!aligned16(operand)) return fail(PQ_ERR_SHAPE, "%s: buffers must be 16-byte aligned", who);
  const size_t need = operand_bytes(fmt, group, M, K);
  if (operand_size < need)
    return fail(PQ_ERR_WORKSPACE, "%s: operand buffer of %zu bytes needed, %zu given", who, need, operand_size);
  return run_norm_quantize_packed(*p, fmt, group, x, M, K, ld, tensor_scale, operand, y, ldy, as_stream(stream));
}

static int check_hadamard(const char* who, const int32_t* perm, const void* x, int64_t M, int64_t K, int64_t ld,
                          const void* y, int64_t ldy, bool y_required) {
  if (!x || (y_required && !y)) return fail(PQ_ERR_NULL, "%s: a required pointer is NULL", who);
  if (M <= 0 || K <= 0) return fail(PQ_ERR_SHAPE, "%s: M=%lld K=%lld must be positive", who, (long long)M, (long long)K);
  if (M > (1 << 24) || K > (1 << 24)) return fail(PQ_ERR_SHAPE, "%s: a dimension exceeds 2^24", who);
  if (K % 8 || ld < K || ld % 8)
    return fail(PQ_ERR_SHAPE, "%s: K=%lld must be a multiple of 8, ld=%lld >= K and a multiple of 8", who,
                (long long)K, (long long)ld);
  if (!hadamard_width_ok(K))
    return fail(PQ_ERR_SHAPE, "%s: K=%lld is not 2^k, 12 * 2^k or 20 * 2^k: no Hadamard construction offered", who,
                (long long)K);
  if (y && (ldy < K || ldy % 8))
    return fail(PQ_ERR_SHAPE, "%s: ldy=%lld must be >= K=%lld and a multiple of 8", who, (long long)ldy, (long long)K);
  if (!aligned16(x) || !aligned16(y) || !aligned16(perm))
    return fail(PQ_ERR_SHAPE, "%s: buffers must be 16-byte aligned", who);
  return PQ_OK;
}

int pq_hadamard_reorder(const int32_t* perm, const void* x, int64_t M, int64_t K, int64_t ld, void* y, int64_t ldy,
                        void* stream) {
  int rc = check_hadamard("pq_hadamard_reorder", perm, x, M, K, ld, y, ldy, true);
  if (rc) return rc;
  return run_hadamard_reorder(perm, x, M, K, ld, y, ldy, as_stream(stream));
}

int pq_hadamard_quantize_act_packed(const int32_t* perm, pq_format fmt, int group, const void* x, int64_t M,
                                    int64_t K, int64_t ld, const float* tensor_scale, void* operand,
                                    size_t operand_size, void* y, int64_t ldy, void* stream) {
  const char* who = "pq_hadamard_quantize_act_packed";
  int rc = check_hadamard(who, perm, x, M, K, ld, y, ldy, false);
  if (rc) return rc;
  if (!operand) return fail(PQ_ERR_NULL, "%s: operand is NULL", who);
  rc = check_format(fmt, group, K);
  if (rc) return rc;
  if (fmt == PQ_FMT_NVFP4 && !tensor_scale) return fail(PQ_ERR_NULL, "%s: NVFP4 needs the per-tensor scale", who);
  if (K % 32) return fail(PQ_ERR_SHAPE, "%s: K=%lld must be a multiple of 32", who, (long long)K);
  if (!aligned16(operand)) return fail(PQ_ERR_SHAPE, "%s: buffers must be 16-byte aligned", who);
  const size_t need = operand_bytes(fmt, group, M, K);
  if (operand_size < need)
    return fail(PQ_ERR_WORKSPACE, "%s: operand buffer of %zu bytes needed, %zu given", who, need, operand_size);
  return run_hadamard_quantize_packed(perm, fmt, group, x, M, K, ld, tensor_scale, operand, y, ldy, as_stream(stream));
}

static int qgemm_packed_common(pq_format fmt, int group, const void* a_operand, const float* a_ts,
                               const void* w_operand, const float* w_ts, int64_t M, int64_t N, int64_t K,
                               const void* bias, void* y, int64_t ldy, bool out_f32, void* stream) {
  if (!a_operand || !w_operand || !y) return fail(PQ_ERR_NULL, "pq_qgemm_packed: a required pointer is NULL");
  int rc = check_format(fmt, group, K);
  if (rc) return rc;
  if (fmt == PQ_FMT_NVFP4 && (!a_ts || !w_ts))
    return fail(PQ_ERR_NULL, "pq_qgemm_packed: NVFP4 needs both per-tensor scales");
  if (M <= 0 || N <= 0) return fail(PQ_ERR_SHAPE, "pq_qgemm_packed: M=%lld N=%lld must be positive",
                                    (long long)M, (long long)N);
  if (K % 32) return fail(PQ_ERR_SHAPE, "pq_qgemm_packed: K=%lld must be a multiple of 32", (long long)K);
  if (M > (1 << 24) || N > (1 << 24) || K > (1 << 24))
    return fail(PQ_ERR_SHAPE, "pq_qgemm_packed: a dimension exceeds 2^24");
  if (ldy < N || ldy % 8)
    return fail(PQ_ERR_SHAPE, "pq_qgemm_packed: ldy=%lld must be >= N=%lld and a multiple of 8",
                (long long)ldy, (long long)N);
  if (!aligned16(a_operand) || !aligned16(w_operand) || !aligned16(y) || !aligned16(bias))
    return fail(PQ_ERR_SHAPE, "pq_qgemm_packed: buffers must be 16-byte aligned");
  return run_qgemm_packed(fmt, group, a_operand, a_ts, w_operand, w_ts, M, N, K, bias, y, ldy, out_f32,
                          as_stream(stream));
}

int pq_qgemm_packed(pq_format fmt, int group, const void* a_operand, const float* a_tensor_scale,
                    const void* w_operand, const float* w_tensor_scale, int64_t M, int64_t N, int64_t K,
                    void* y_bf16, int64_t ldy, void* stream) {
  return qgemm_packed_common(fmt, group, a_operand, a_tensor_scale, w_operand, w_tensor_scale, M, N, K,
                             nullptr, y_bf16, ldy, false, stream);
}

int pq_qgemm_packed_bias(pq_format fmt, int group, const void* a_operand, const float* a_tensor_scale,
                         const void* w_operand, const float* w_tensor_scale, int64_t M, int64_t N, int64_t K,
                         const void* bias_bf16, void* y_bf16, int64_t ldy, void* stream) {
  if (!bias_bf16) return fail(PQ_ERR_NULL, "pq_qgemm_packed_bias: bias is NULL");
  return qgemm_packed_common(fmt, group, a_operand, a_tensor_scale, w_operand, w_tensor_scale, M, N, K,
                             bias_bf16, y_bf16, ldy, false, stream);
}

int pq_qgemm_packed_f32(pq_format fmt, int group, const void* a_operand, const float* a_tensor_scale,
                        const void* w_operand, const float* w_tensor_scale, int64_t M, int64_t N,
                        int64_t K, float* y_f32, int64_t ldy, void* stream) {
  return qgemm_packed_common(fmt, group, a_operand, a_tensor_scale, w_operand, w_tensor_scale, M, N, K,
                             nullptr, y_f32, ldy, true, stream);
}

int pq_qgemm_check_int_scales(pq_format fmt, int group, const void* scales, int64_t rows, int64_t K,
                              int64_t* bad_count, void* workspace, size_t workspace_bytes, void* stream) {
  if (!scales || !bad_count) return fail(PQ_ERR_NULL, "pq_qgemm_check_int_scales: scales and bad_count must not be NULL");
  if (fmt != PQ_FMT_INT4 && fmt != PQ_FMT_INT3)
    return fail(PQ_ERR_FORMAT, "pq_qgemm_check_int_scales: format %d has no fp32 group scales", (int)fmt);
  int rc = check_format(fmt, group, K);
  if (rc) return rc;
  if (rows <= 0) return fail(PQ_ERR_SHAPE, "pq_qgemm_check_int_scales: rows=%lld must be positive", (long long)rows);
  if (!workspace || workspace_bytes < 256)
    return fail(PQ_ERR_WORKSPACE, "pq_qgemm_check_int_scales: workspace of 256 bytes needed, %zu given",
                workspace ? workspace_bytes : (size_t)0);
  return run_check_int_scales(fmt, group, scales, rows, K, bad_count, workspace, as_stream(stream));
}

int pq_probe_stream(const void* src, size_t read_bytes, void* dst, size_t write_bytes, void* stream) {
  if ((read_bytes && !src) || (write_bytes && !dst))
    return fail(PQ_ERR_NULL, "pq_probe_stream: NULL buffer with a non-zero size");
  if (read_bytes % 16 || write_bytes % 16)
    return fail(PQ_ERR_SHAPE, "pq_probe_stream: sizes must be multiples of 16 bytes");
  if (!aligned16(src) || !aligned16(dst))
    return fail(PQ_ERR_SHAPE, "pq_probe_stream: buffers must be 16-byte aligned");
  if (write_bytes == 0 && read_bytes && !dst)
    return fail(PQ_ERR_NULL, "pq_probe_stream: dst must be a valid 16-byte buffer even when nothing is written");
  return launch_probe_stream(src, read_bytes, dst, write_bytes, as_stream(stream));
}

int pq_probe_mfma(int iters, float* sink, double* flops_out, void* stream) {
  if (!sink) return fail(PQ_ERR_NULL, "pq_probe_mfma: sink must not be NULL");
  if (iters <= 0 || iters > (1 << 24)) return fail(PQ_ERR_SHAPE, "pq_probe_mfma: iters=%d out of range", iters);
  return launch_probe_mfma(iters, sink, flops_out, as_stream(stream));
}

int pq_probe_mfma_operands(pq_format fmt, int group, const void* a_operand, const void* w_operand, int64_t M,
                           int64_t N, int64_t K, int iters, float* sink, double* flops_out, void* stream) {
  if (!a_operand || !w_operand || !sink) return fail(PQ_ERR_NULL, "pq_probe_mfma_operands: NULL pointer");
  int rc = check_format(fmt, group, K);
  if (rc) return rc;
  if (M <= 0 || N <= 0 || K % 64) return fail(PQ_ERR_SHAPE, "pq_probe_mfma_operands: M=%lld N=%lld must be positive, K=%lld a multiple of 64",
                                             (long long)M, (long long)N, (long long)K);
  if (M * 32 > 0x7FFFFFFF || N * 32 > 0x7FFFFFFF) return fail(PQ_ERR_SHAPE, "pq_probe_mfma_operands: too many rows");
  if (!aligned16(a_operand) || !aligned16(w_operand)) return fail(PQ_ERR_SHAPE, "pq_probe_mfma_operands: operands must be 16-byte aligned");
  if (iters <= 0 || iters > (1 << 24)) return fail(PQ_ERR_SHAPE, "pq_probe_mfma_operands: iters=%d out of range", iters);
  return launch_probe_mfma_operands(fmt, group, a_operand, w_operand, M, N, K, iters, sink, flops_out, as_stream(stream));
}

}  // extern "C"
