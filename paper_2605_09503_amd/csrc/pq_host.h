// Host-side plumbing shared by the entry points: error reporting, argument checks,
// workspace carving.  Nothing here is exported; the C ABI lives in include/permuquant.h.
#pragma once
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/permuquant.h"

namespace pq {

// Records a message for pq_last_error() and returns `code`.
int fail(int code, const char* fmt, ...);

// hipGetLastError / API status -> PQ_ERR_HIP with the runtime's text.
int check_hip(hipError_t e, const char* what);

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// PQ_OK, or the error for an unknown format / unsupported (format, group) pair / K % group.
int check_format(pq_format fmt, int group, int64_t K);

inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

// ---- kernel launchers (one per source file) --------------------------------------------
constexpr int kMaxMomentBatches = 16;   // batches handled by one launch of the moments kernel
size_t moments_workspace_bytes(int64_t rows, int64_t K, int n_batches);
int launch_moments(const void* const* xs, int n_batches, int64_t rows, int64_t K, int64_t ld,
                   double* sumsq, float* absmax, void* ws, hipStream_t st);

constexpr size_t kStaticScratchBytes = 3u << 20;   // scratch the library itself holds on every device
int launch_moments_static(const void* x, int64_t rows, int64_t K, int64_t ld, double* sumsq, float* absmax,
                          hipStream_t st);

int launch_absmax_to_tensor_scale(const void* x, int64_t n_elems, float* tensor_scale_out,
                                  hipStream_t st);
int launch_dynamic_tensor_scale(const void* x, int64_t rows, int64_t K, int64_t ld, float* out, hipStream_t st);
int launch_fill_float(float* p, float v, hipStream_t st);
int launch_tensor_scale(const float* absmax, float* out, hipStream_t st);
int launch_quantize_rows(pq_format fmt, int group, const void* x, int64_t rows, int64_t K, int64_t ld,
                         const int32_t* perm, const float* tensor_scale, uint8_t* codes, void* scales,
                         hipStream_t st);

// The error evaluation keeps one row as fp32 in LDS, one spare slot per eight channels: 4.5 K bytes of the
// 150 KB a workgroup may take.
constexpr int64_t kSelectMaxK = 34128;      // largest multiple of 16 with 4.5 K <= 150 * 1024
size_t select_workspace_bytes(int64_t M, int64_t N, int64_t K, int n_batches);
size_t quant_error_workspace_bytes(int64_t rows, int64_t K);
int run_select(pq_format fmt, int group, const double* act_sumsq, const double* w_sumsq, int64_t K,
               const void* const* x_calib, int n_batches, int64_t M, const void* w, int64_t N,
               float act_ts, float w_ts, const float* act_ts_dev, const float* w_ts_dev, const double* alphas,
               int n_alpha, double tau, int32_t* perm_out, pq_select_report* report, void* ws, hipStream_t st);
int launch_candidate_orders(const double* act_sumsq, const double* w_sumsq, int64_t K, const double* alphas,
                            int n_alpha, double* keys, int32_t* rank, int32_t* cands, hipStream_t st,
                            int32_t* offs = nullptr, int slot_bytes = 0, uint32_t* differs = nullptr);
int launch_identity_order(int32_t* perm, int64_t K, hipStream_t st);
double* pinned_doubles(size_t n);     // the calling thread's pinned host buffer, kept for the process lifetime
int launch_round_robin(const int32_t* order, int64_t K, int group, int32_t* perm, hipStream_t st);
size_t random_order_workspace_bytes(int64_t K);      // also enough for one candidate order (keys + ranks)
int launch_random_order(uint64_t seed, int64_t K, int32_t* perm, void* ws, hipStream_t st);
size_t channel_stats_workspace_bytes(int64_t rows, int64_t K);
int launch_channel_stats(const void* x, int64_t rows, int64_t K, int64_t ld, double* sum, float* absmax, void* ws,
                         hipStream_t st);
int launch_channel_variance(const double* sum, const double* sumsq, int64_t n_rows, int64_t K, double* out,
                            hipStream_t st);
int launch_channel_absmax_sq(const float* absmax, int64_t K, double* out, hipStream_t st);
size_t select_output_workspace_bytes(pq_format fmt, int group, int64_t M, int64_t N, int64_t K, int n_batches);
int run_select_output(pq_format fmt, int group, const double* act_sumsq, const double* w_sumsq, int64_t K,
                      const void* const* x_calib, int n_batches, int64_t M, const void* w, int64_t N,
                      float act_ts, float w_ts, const double* alphas, int n_alpha, double tau,
                      int32_t* perm_out, pq_select_report* report, void* ws, hipStream_t st);
int run_quant_error(pq_format fmt, int group, const void* x, int64_t rows, int64_t K,
                    const int32_t* perm, float ts, double* err_out, void* ws, hipStream_t st);

size_t qgemm_workspace_bytes(pq_format fmt, int group, int64_t M, int64_t N, int64_t K);
int run_qgemm(pq_format fmt, int group, const uint8_t* a_codes, const void* a_scales,
              const float* a_ts, const uint8_t* w_codes, const void* w_scales, const float* w_ts,
              int64_t M, int64_t N, int64_t K, void* y, int64_t ldy, bool out_f32, int phases,
              void* ws, hipStream_t st);   // phases: 1 = scale preparation, 2 = product


// Panel layout of a quantized operand (see pq_pack.hip): byte offsets of its parts.
struct OperandLayout {
  size_t codes, scales, mul, total;     // byte offsets and total size
  int64_t steps, units;
};
inline OperandLayout operand_layout(pq_format fmt, int group, int64_t rows, int64_t K) {
  OperandLayout L;
  L.steps = (K + 63) / 64;
  L.units = fmt == PQ_FMT_NVFP4 ? (K + 31) / 32 : K / group;
  L.codes = 0;
  L.scales = align_up((size_t)L.steps * rows * 32, 256);
  L.mul = L.scales + align_up((size_t)L.units * rows * 2, 256);
  L.total = L.mul + (fmt == PQ_FMT_NVFP4 ? 0 : align_up((size_t)rows * 4, 256));
  return L;
}
size_t operand_bytes(pq_format fmt, int group, int64_t rows, int64_t K);
int run_pack_operand(pq_format fmt, int group, const uint8_t* codes, const void* scales, int64_t rows,
                     int64_t K, void* operand, bool dense3, hipStream_t st);   // dense3: codes as pq_int3_pack stores them
int launch_int3_pack(const uint8_t* codes, int64_t rows, int64_t K, uint8_t* dense, hipStream_t st);
int launch_int3_unpack(const uint8_t* dense, int64_t rows, int64_t K, uint8_t* codes, hipStream_t st);
int run_quantize_packed(pq_format fmt, int group, const void* x, int64_t rows, int64_t K, int64_t ld,
                        const float* ts, void* operand, uint8_t* codes, void* scales, hipStream_t st);
int run_norm_reorder(const pq_norm_params& p, const void* x, int64_t rows, int64_t K, int64_t ld, void* y,
                     int64_t ldy, hipStream_t st);
int run_norm_quantize_packed(const pq_norm_params& p, pq_format fmt, int group, const void* x, int64_t rows,
                             int64_t K, int64_t ld, const float* ts, void* operand, void* y, int64_t ldy,
                             hipStream_t st);
bool hadamard_width_ok(int64_t K);
int run_hadamard_reorder(const int32_t* perm, const void* x, int64_t rows, int64_t K, int64_t ld, void* y,
                         int64_t ldy, hipStream_t st);
int run_hadamard_quantize_packed(const int32_t* perm, pq_format fmt, int group, const void* x, int64_t rows,
                                 int64_t K, int64_t ld, const float* ts, void* operand, void* y, int64_t ldy,
                                 hipStream_t st);
int run_qgemm_packed(pq_format fmt, int group, const void* a_operand, const float* a_ts,
                     const void* w_operand, const float* w_ts, int64_t M, int64_t N, int64_t K,
                     const void* bias, void* y, int64_t ldy, bool out_f32, hipStream_t st);

int run_check_int_scales(pq_format fmt, int group, const void* scales, int64_t rows, int64_t K, int64_t* bad_count,
                         void* ws, hipStream_t st);
int launch_probe_stream(const void* src, size_t read_bytes, void* dst, size_t write_bytes, hipStream_t st);
int launch_probe_mfma(int iters, float* sink, double* flops_out, hipStream_t st);
int launch_probe_mfma_operands(pq_format fmt, int group, const void* a_operand, const void* w_operand, int64_t M,
                               int64_t N, int64_t K, int iters, float* sink, double* flops_out, hipStream_t st);

}  // namespace pq
