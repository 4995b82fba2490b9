/*
 * permuquant.h -- C ABI of the MI355X (gfx950) per-group-quantized linear layer.
 *
 * The library implements the data-parallel hot path of PermuQuant: calibration statistics
 * and permutation selection (paper Sec. 3.2-3.3), offline weight quantization in the
 * selected channel order, dynamic per-group activation quantization, and the low-bit GEMM
 * of the reordered quantized linear layer (paper Eq. 8).  Around that path it offers the steps
 * the paper describes next to it: the normalisation layer that absorbs the activation reorder
 * (App. C), the Hadamard variant PermuQuant-H (App. D), the layer-output reading of the
 * calibration metric, a dynamic NVFP4 tensor scale, the layer's bias in the GEMM epilogue and
 * the alternative reorder criteria of the ablation (Tab. 2a).
 *
 * Conventions
 *   - X is [M, K] row-major (tokens x input channels), W is [N, K] row-major (output x input
 *     channels), Y[M, N] = X * W^T.  The paper writes Y = X W with W as in x out; its
 *     P^T W is a column permutation of W here.
 *   - K is the reduction (channel) dimension, `group` the group size g along K (the paper's
 *     d and g; the paper's K = d/g is the number of groups).
 *   - bf16 tensors are passed as const void* to 16-bit elements.
 *   - Unless a parameter says "host", every pointer is DEVICE memory owned by the caller and
 *     must stay valid until the work queued on `stream` has finished.  Tensor pointers must be
 *     16-byte aligned.  The library allocates no device memory; scratch memory comes in
 *     through `workspace` (size from pq_workspace_bytes()).  The one host allocation: the calls
 *     that synchronise anyway (the two selection calls, pq_qgemm_check_int_scales) read their
 *     results back through a small pinned host buffer (4 KB for up to 30 batches) that the calling
 *     thread allocates at its first such call and frees when the thread ends.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls are
 *     asynchronous on it unless stated otherwise.
 *   - All arguments are validated on the host before anything is launched.  Every function
 *     returns PQ_OK or a negative error code; pq_last_error() gives the message of the last
 *     failure on the calling thread.  No C++ exception crosses this boundary.
 *   - Inputs must be finite (no NaN/Inf); behaviour on non-finite inputs is unspecified.
 *
 * Stored formats (what parity is checked on)
 *   codes   two 4-bit containers per byte, element k = 2j in the low nibble, 2j+1 in the high.
 *           NVFP4: nibble = sign << 3 | E2M1 index (values 0, .5, 1, 1.5, 2, 3, 4, 6).
 *           INT4 / INT3: 4-bit two's complement of z, z in [-Q, Q], Q = 7 / 3.
 *   scales  row-major [rows, K / group]: NVFP4 one E4M3 byte (bias 7, max 448) per 16
 *           channels; INT one float per group (Eq. 1: s = max|x| / Q).
 *   tensor scale  NVFP4 only: one float per tensor, T = max|.| / (448 * 6).
 *
 * Quantizer arithmetic (every step one IEEE binary32 operation, round-to-nearest-even):
 *   INT     s = amax / Q;  inv = s normal ? 1 / s : 0;  z = clip(rint(x * inv), -Q, Q)
 *   NVFP4   encT = T normal ? 1 / T : 0;  t = (amax * encT) / 6;  s_b = E4M3_rne_sat(t);
 *           d = value(s_b) * T;  inv = d normal ? 1 / d : 0;
 *           code = sign(x) << 3 | E2M1_rne_sat(|x * inv|)     (ties to the even code)
 */
#ifndef PERMUQUANT_H
#define PERMUQUANT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { PQ_FMT_NVFP4 = 0, PQ_FMT_INT4 = 1, PQ_FMT_INT3 = 2 } pq_format;

typedef enum {
  PQ_OP_CALIB_MOMENTS = 0,
  PQ_OP_SELECT_PERM = 1,
  PQ_OP_QUANTIZE_WEIGHTS = 2,
  PQ_OP_QUANTIZE_ACT = 3,
  PQ_OP_QGEMM = 4,
  PQ_OP_QUANT_ERROR = 5,
  PQ_OP_SELECT_PERM_OUTPUT = 6,
  PQ_OP_CHANNEL_STATS = 7,       /* M = rows, K                                   */
  PQ_OP_ORDER = 8                /* K: pq_order_by_score, pq_order_random         */
} pq_op;

#define PQ_OK 0
#define PQ_ERR_NULL (-1)      /* a required pointer is NULL                                   */
#define PQ_ERR_SHAPE (-2)     /* non-positive size, K % group != 0, ld < K, misaligned pointer */
#define PQ_ERR_FORMAT (-3)    /* unknown format, or a (format, group) pair that is not offered */
#define PQ_ERR_WORKSPACE (-4) /* workspace NULL or smaller than pq_workspace_bytes()          */
#define PQ_ERR_HIP (-5)       /* the HIP runtime reported an error                            */

#define PQ_MAX_ALPHAS 15

/* Offered (format, group) pairs: NVFP4 with 16; INT4 and INT3 with 32, 64, 128 or 256.
 * K must be a multiple of the group size (hence of 16).                                     */

/* Message of the last failure on this thread ("" if none). Never NULL. Host memory owned by
 * the library, valid until the next failing call on the same thread.                        */
const char* pq_last_error(void);

/* Library version, major * 100 + minor. */
int pq_version(void);

/* Bytes of workspace `op` needs for these sizes (0 if none).  Arguments an operation does not
 * depend on may be 0.  Returns 0 for invalid arguments (the operation itself reports them). */
size_t pq_workspace_bytes(pq_op op, pq_format fmt, int group, int64_t M, int64_t N, int64_t K,
                          int n_batches);

/*
 * Per-input-channel second moments (paper Sec. 3.2, Assumption 1: mu_i^2 = E[x_i^2]; Sec. 3.3,
 * Eq. 9 uses them for activations and for the matching weight channels).  A common factor
 * does not change the sort, so sums of squares are kept instead of means.
 *
 *   sumsq[i] += sum_r x[r, i]^2   (fp64; squares of bf16 values are exact, accumulation fp64)
 *   absmax[0] = max(absmax[0], max |x|)   if absmax != NULL (feeds the NVFP4 tensor scale)
 *
 * x: bf16 [rows, ld] with ld >= K.  sumsq: double [K], in/out -- the caller zero-fills it
 * before the first batch; call once per calibration batch, and once with x = W, rows = N.
 * absmax: float [1], in/out, >= 0 (zero-filled by the caller), may be NULL.
 * workspace: pq_workspace_bytes(PQ_OP_CALIB_MOMENTS, ., ., rows, 0, K, n_batches) bytes
 * (n_batches = 1 here); contents are scratch and need not be initialised.  Results are deterministic
 * (fixed summation order for fixed sizes, no atomics).  Two launches; may be captured into a HIP graph.
 */
int pq_calib_moments(const void* x_bf16, int64_t rows, int64_t K, int64_t ld, double* sumsq,
                     float* absmax, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Same statistic over several calibration batches of equal shape in one launch (the batches of a
 * calibration set are separate tensors; one launch over all of them keeps the memory system
 * busy where one 28 MB batch alone is mostly launch latency).
 * x_batches: HOST array of n_batches DEVICE pointers, each bf16 [rows, ld].
 */
int pq_calib_moments_batched(const void* const* x_batches, int n_batches, int64_t rows, int64_t K,
                             int64_t ld, double* sumsq, float* absmax, void* workspace,
                             size_t workspace_bytes, void* stream);

/*
 * pq_calib_moments for callers that cannot allocate or bring a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same summation order
 * and therefore the same bits as pq_calib_moments; the partial sums go to a device array of
 * PQ_STATIC_SCRATCH_BYTES that is part of the library's code object (every GPU the library runs on
 * holds it until the process ends).  The call allocates nothing, on the device or on the host
 * (its first call on a device looks the array's address up once).  Shapes whose partial sums need more
 * than PQ_STATIC_SCRATCH_BYTES (= pq_workspace_bytes(PQ_OP_CALIB_MOMENTS, ., ., rows, 0, K, 1)) are
 * refused with PQ_ERR_WORKSPACE before anything is launched (the need stays near 2 MB for any row count
 * and widths up to some 390 000 channels: every tensor of a transformer layer fits).  All calls on one GPU share the one array, which keeps the last
 * call's partial sums (nothing in it has to start at zero): calls that overlap on one GPU -- on
 * different streams or from different threads -- race and must be serialised by the caller.
 * Other arguments, result and error codes as for pq_calib_moments.
 */
#define PQ_STATIC_SCRATCH_BYTES ((size_t)3 << 20)
int pq_calib_moments_static(const void* x_bf16, int64_t rows, int64_t K, int64_t ld, double* sumsq,
                            float* absmax, void* stream);

/*
 * NVFP4 per-tensor scale from a running absmax (the two-level reading of NVFP4 W4A4, paper
 * Sec. 4.4): tensor_scale_out[0] = fl32(absmax[0] / 2688), 2688 = 448 * 6, so that the largest
 * block scale lands on the E4M3 maximum.  Both pointers: float [1] device; may alias.
 */
int pq_tensor_scale(const float* absmax, float* tensor_scale_out, void* stream);

/*
 * Permutation selection (paper Sec. 3.3: joint score Eq. 9, alpha grid search, acceptance rule).
 *
 * For every alpha_j: key_i = alpha_j * ln(act_sumsq[i]) + (1 - alpha_j) * ln(w_sumsq[i]) (a
 * term with zero weight is left out; a zero sum sorts last), channels sorted by descending key
 * (Prop. 1), equal keys by ascending index.  Each candidate order pi and the original order are
 * scored by
 *     E(pi) = ||X - Xhat_pi||^2 / ||X||^2 + ||W - What_pi||^2 / ||W||^2
 * over all calibration batches (each tensor quantized with this library's quantizer in the
 * order pi, fp64 accumulation).  The candidate with the smallest E wins (ties: smallest j); it
 * is accepted iff it differs from the identity, E_orig > 0 and
 * (E_orig - E_best) / E_orig > tau.  perm_out receives the accepted order, else the identity.
 * perm[j] = original channel that moves to position j.
 *
 * act_sumsq, w_sumsq: double [K] from pq_calib_moments.
 * x_calib: HOST array of n_batches DEVICE pointers, each bf16 [M, K] contiguous.
 * w_bf16: bf16 [N, K] contiguous.
 * act_tensor_scale / w_tensor_scale: NVFP4 only (host floats, T of the header comment; the
 * activation one comes from the calibration absmax, the weight one from max|W|); ignored for INT.
 * K <= 34128: one row as fp32 must fit the LDS of the error evaluation (4.5 K bytes of 150 KB);
 * pq_workspace_bytes returns 0 beyond, the call PQ_ERR_SHAPE before anything is launched.
 * alphas: HOST array of n_alpha values in [0, 1], 1 <= n_alpha <= PQ_MAX_ALPHAS.
 * perm_out: int32 [K] device.  report: HOST struct, filled on return.
 * This call synchronises `stream` once before returning (the decision is taken on the host).
 */
typedef struct {
  int accepted;                  /* 1 if perm_out holds a reordering, 0 if the identity   */
  int alpha_index;               /* index of the best candidate in alphas                 */
  double e_orig;                 /* E of the original order                               */
  double e_best;                 /* E of the best candidate                               */
  double e_cand[PQ_MAX_ALPHAS];  /* E of every candidate                                  */
  double sum_x2;                 /* ||X||^2 over the calibration batches                  */
  double sum_w2;                 /* ||W||^2                                               */
} pq_select_report;

int pq_select_perm(pq_format fmt, int group, const double* act_sumsq, const double* w_sumsq,
                   int64_t K, const void* const* x_calib, int n_batches, int64_t M,
                   const void* w_bf16, int64_t N, float act_tensor_scale, float w_tensor_scale,
                   const double* alphas, int n_alpha, double tau, int32_t* perm_out,
                   pq_select_report* report, void* workspace, size_t workspace_bytes,
                   void* stream);

/*
 * pq_select_perm with the two NVFP4 tensor scales read from device memory (float [1] each, as
 * pq_tensor_scale leaves them) instead of passed as host values: a calibration that computes the scales
 * on the stream need not synchronise to fetch them before this call.  Ignored for INT (may be NULL).
 * Everything else, the report included, as for pq_select_perm with the same two values.
 */
int pq_select_perm_device_scales(pq_format fmt, int group, const double* act_sumsq, const double* w_sumsq,
                                 int64_t K, const void* const* x_calib, int n_batches, int64_t M,
                                 const void* w_bf16, int64_t N, const float* act_tensor_scale,
                                 const float* w_tensor_scale, const double* alphas, int n_alpha, double tau,
                                 int32_t* perm_out, pq_select_report* report, void* workspace,
                                 size_t workspace_bytes, void* stream);

/*
 * The same selection with the layer-output error as the metric -- the other reading of "smallest
 * quantization error on the calibration data" (paper Sec. 3.3), in terms of Eq. 8:
 *     E_out(pi) = sum_b ||X_b W^T - Q(X_b P) Q(P^T W)^T||^2 / sum_b ||X_b W^T||^2.
 * Candidates, argmin, tie rule, acceptance rule and arguments as for pq_select_perm; K must also be a
 * multiple of 32 (the quantized product runs through the packed forward path, the unquantized one
 * through a plain bf16 MFMA kernel, both with fp32 accumulation: E_out carries a relative error of
 * about 1e-5 against exact arithmetic).  report->sum_x2 holds sum_b ||X_b W^T||^2, sum_w2 is 0.
 * workspace: pq_workspace_bytes(PQ_OP_SELECT_PERM_OUTPUT, fmt, group, M, N, K, n_batches) bytes -- it
 * holds the fp32 reference products of all batches (4 n_batches M N bytes).
 */
int pq_select_perm_output_error(pq_format fmt, int group, const double* act_sumsq, const double* w_sumsq,
                                int64_t K, const void* const* x_calib, int n_batches, int64_t M,
                                const void* w_bf16, int64_t N, float act_tensor_scale, float w_tensor_scale,
                                const double* alphas, int n_alpha, double tau, int32_t* perm_out,
                                pq_select_report* report, void* workspace, size_t workspace_bytes,
                                void* stream);

/*
 * Squared quantization error of one tensor in a given channel order (paper Eq. 3 on a finite
 * sample; the building block of E above, also what "quantization error with / without the
 * permutation" reports):   err_out[0] = sum_{r,k} (x[r, perm[k]] - xhat)^2   (fp64).
 * x: bf16 [rows, K] contiguous.  perm: int32 [K] or NULL (identity).  tensor_scale: host float,
 * NVFP4 only.  err_out: double [1] device, overwritten.  K <= 34128 as for pq_select_perm.
 * Accuracy: the integer formats sum exact element errors in fp64.  The NVFP4 error is formed as
 * sum x^2 minus exact cross terms and is known to about 1e-15 of sum x^2 absolutely (a relative 1e-13
 * for data that fill the format): a sum that comes out negative is returned as 0, and pq_select_perm
 * reports a tensor's error as exactly 0 when it is below 1e-13 of the tensor's sum of squares.
 */
int pq_quant_error(pq_format fmt, int group, const void* x_bf16, int64_t rows, int64_t K,
                   const int32_t* perm, float tensor_scale, double* err_out, void* workspace,
                   size_t workspace_bytes, void* stream);

/*
 * Offline weight quantization in the selected channel order (paper Sec. 3.3 "Runtime-free
 * deployment": the permutation of W's input channels is applied offline; Eq. 1-2 per row and
 * group).  Element k of output row n is W[n, perm[k]].
 *
 * w_bf16: bf16 [N, K] contiguous.  perm: int32 [K] or NULL (identity).
 * codes: uint8 [N, K/2].  scales: uint8 [N, K/16] (NVFP4) or float [N, K/group] (INT).
 * tensor_scale_out: float [1] device; NVFP4: receives fl32(max|W| / 2688); INT: receives 1.0f.
 */
int pq_quantize_weights(pq_format fmt, int group, const void* w_bf16, int64_t N, int64_t K,
                        const int32_t* perm, uint8_t* codes, void* scales,
                        float* tensor_scale_out, void* stream);

/*
 * Dynamic per-group activation quantization of one batch of token rows (paper Sec. 3.1 Eq. 1-2,
 * applied online per token as in App. A.3; Eq. 8's Q(XP)).
 *
 * x_bf16: bf16 [M, ld], ld >= K, ld % 8 == 0.
 * perm: NULL when the producer already emits the permuted order (the deployment case, paper
 * Sec. 3.3); non-NULL gathers x[m, perm[k]] on load (slower; calibration / test convenience).
 * tensor_scale: float [1] device, NVFP4 only (static, from calibration); ignored for INT.
 * codes: uint8 [M, K/2].  scales: uint8 [M, K/16] (NVFP4) or float [M, K/group] (INT).
 */
int pq_quantize_act(pq_format fmt, int group, const void* x_bf16, int64_t M, int64_t K,
                    int64_t ld, const int32_t* perm, const float* tensor_scale, uint8_t* codes,
                    void* scales, void* stream);

/*
 * Low-bit GEMM of the reordered quantized layer (paper Eq. 8):
 *   Y[m, n] = Ta * Tw * sum_g sa[m, g] * sw[n, g] * sum_{k in g} a[m, k] * w[n, k]
 * with fp32 accumulation over the whole of K and one rounding (nearest-even) to bf16 at the
 * store.  Both operands must be in the same channel order and use the same (fmt, group).
 *
 * a_codes [M, K/2], a_scales [M, K/group], w_codes [N, K/2], w_scales [N, K/group] as stored by
 * the quantizers above; a_tensor_scale / w_tensor_scale: float [1] device (NVFP4; ignored for
 * INT, may be NULL).  y_bf16: bf16 [M, ldy], ldy >= N, ldy % 8 == 0.
 * INT scales must be of the form fl32(h / Q) with h a bf16 value, which is what the quantizers
 * above produce from bf16 inputs (the kernel folds h exactly into its fp16 MFMA operands; the
 * product then differs from the stored-scale one by the 2^-24 rounding of h / Q per factor).  Scales
 * of another origin give a different product without an error: check them once with
 * pq_qgemm_check_int_scales.  Inside a row the operand holds h * 2^-E with E from the row's largest
 * group: a group more than 2^24 below it loses low bits of h (below 2^-35: all of them) -- its terms
 * are then below 2^-24 of the row's largest terms, the resolution of the fp32 accumulation anyway.
 * workspace: pq_workspace_bytes(PQ_OP_QGEMM, fmt, group, M, N, K, 0) bytes.
 */
int pq_qgemm(pq_format fmt, int group, const uint8_t* a_codes, const void* a_scales,
             const float* a_tensor_scale, const uint8_t* w_codes, const void* w_scales,
             const float* w_tensor_scale, int64_t M, int64_t N, int64_t K, void* y_bf16,
             int64_t ldy, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Counts the INT group scales that pq_qgemm / pq_pack_operand would not reproduce exactly: those not of
 * the form fl32(h / Q), h a non-negative bf16 value (also negative and non-finite ones).  scales: float
 * [rows, K / group] device.  bad_count: HOST int64, written on return; 0 means the product computed from
 * these scales is the one Eq. 8 defines with them.  workspace: at least 256 bytes of device memory.
 * Synchronises `stream`.  PQ_ERR_FORMAT for NVFP4 (its E4M3 scales are always exact in the operand).
 */
int pq_qgemm_check_int_scales(pq_format fmt, int group, const void* scales, int64_t rows, int64_t K,
                              int64_t* bad_count, void* workspace, size_t workspace_bytes, void* stream);

/*
 * pq_qgemm in two steps, for callers that want the scale preparation out of the per-token path
 * (and for timing the product kernel alone).  pq_qgemm_prep turns the stored INT scales of both
 * operands into the kernel's working form inside `workspace` (per-row power-of-two
 * normalisation; nothing to do for NVFP4); pq_qgemm_run then computes the product from codes
 * and that workspace.  pq_qgemm(...) == pq_qgemm_prep(...) followed by pq_qgemm_run(...) with
 * the same workspace.  Arguments as for pq_qgemm.
 */
int pq_qgemm_prep(pq_format fmt, int group, const void* a_scales, const void* w_scales, int64_t M,
                  int64_t N, int64_t K, void* workspace, size_t workspace_bytes, void* stream);
int pq_qgemm_run(pq_format fmt, int group, const uint8_t* a_codes, const void* a_scales,
                 const float* a_tensor_scale, const uint8_t* w_codes, const void* w_scales,
                 const float* w_tensor_scale, int64_t M, int64_t N, int64_t K, void* y_bf16,
                 int64_t ldy, void* workspace, size_t workspace_bytes, void* stream);

/* Same product with the fp32 accumulator stored unrounded: y_f32 is float [M, ldy].  For
 * checking the accumulation against an fp64 reference before the bf16 rounding.           */
int pq_qgemm_f32(pq_format fmt, int group, const uint8_t* a_codes, const void* a_scales,
                 const float* a_tensor_scale, const uint8_t* w_codes, const void* w_scales,
                 const float* w_tensor_scale, int64_t M, int64_t N, int64_t K, float* y_f32,
                 int64_t ldy, void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same product from operands in the GEMM's own layout (paper Eq. 8; Sec. 3.3: the weights
 * are prepared offline).  pq_pack_operand rearranges the stored output of a quantizer -- codes
 * [rows, K/2] and scales [rows, K/group] -- into a K-step-major panel in which the 64-k pieces
 * of consecutive rows are adjacent, and for INT also applies the scale preparation of
 * pq_qgemm_prep.  Pack the weights once; pack the activations once per forward; then
 *     pq_qgemm_packed(pack(A), pack(W)) == pq_qgemm(A, W)      bit for bit,
 * with the product kernel reading whole cache lines instead of 32-byte pieces.
 *
 * operand: device buffer of pq_operand_bytes(fmt, group, rows, K) bytes (0 for an invalid
 * shape), 16-byte aligned, written by pq_pack_operand; its layout is private to the library.
 * K must be a multiple of 32.  Tensor scales as for pq_qgemm (NVFP4 only).
 *
 * pq_quantize_act_packed is pq_quantize_act (no gather: the producer emits the selected channel
 * order) writing the panel directly, so that the forward path has no packing pass: the operand
 * it leaves is byte for byte pq_pack_operand of pq_quantize_act's output.  codes / scales:
 * optional row-major copies as pq_quantize_act stores them (both or neither; NULL to skip).
 */
size_t pq_operand_bytes(pq_format fmt, int group, int64_t rows, int64_t K);
int pq_quantize_act_packed(pq_format fmt, int group, const void* x_bf16, int64_t M, int64_t K,
                           int64_t ld, const float* tensor_scale, void* operand, size_t operand_size,
                           uint8_t* codes, void* scales, void* stream);
int pq_pack_operand(pq_format fmt, int group, const uint8_t* codes, const void* scales, int64_t rows,
                    int64_t K, void* operand, size_t operand_size, void* stream);
int pq_qgemm_packed(pq_format fmt, int group, const void* a_operand, const float* a_tensor_scale,
                    const void* w_operand, const float* w_tensor_scale, int64_t M, int64_t N, int64_t K,
                    void* y_bf16, int64_t ldy, void* stream);
int pq_qgemm_packed_f32(pq_format fmt, int group, const void* a_operand, const float* a_tensor_scale,
                        const void* w_operand, const float* w_tensor_scale, int64_t M, int64_t N,
                        int64_t K, float* y_f32, int64_t ldy, void* stream);
/* The linear layer with its bias, y = Q(XP) Q(P^T W) + b (paper Eq. 8 covers the product; the layers
 * it replaces are x W^T + b): bias_bf16 is bf16 [N] device memory, 16-byte aligned, added in fp32
 * to the scaled accumulator before the single rounding to bf16.  Otherwise as pq_qgemm_packed.     */
int pq_qgemm_packed_bias(pq_format fmt, int group, const void* a_operand, const float* a_tensor_scale,
                         const void* w_operand, const float* w_tensor_scale, int64_t M, int64_t N, int64_t K,
                         const void* bias_bf16, void* y_bf16, int64_t ldy, void* stream);

/*
 * Dense 3-bit storage of INT3 codes (paper Eq. 1-2 with b = 3: codes in -3..3).  The quantizers store
 * INT3 codes in nibbles like INT4; these calls hold them at three bits each, which is what the weights of
 * a W3 model occupy at rest.  The paper prints no layout; this one is the library's: a row of K codes is
 * a stream of 3 K bits, code k in bits 3k..3k+2 as the 3-bit two's complement of z (least significant
 * bit first), bit b of the stream in bit b mod 8 of byte b div 8; a row takes 3 K / 8 bytes and rows
 * follow each other unpadded.
 *
 * codes: [rows, K/2] bytes of nibbles as pq_quantize_weights / pq_quantize_act write them for INT3;
 * dense: [rows, 3 K / 8] bytes = pq_int3_dense_bytes(rows, K) (0 for an invalid shape).  Both device
 * memory, 16-byte aligned, caller-owned, and they must not overlap.  K: a positive multiple of 32; rows
 * and K at most 2^24.  pq_int3_pack keeps the low three bits of every nibble: for the codes the
 * quantizers emit (and for -4) pq_int3_unpack(pq_int3_pack(c)) == c, other nibbles are not checked.
 * pq_pack_operand_int3 is pq_pack_operand for PQ_FMT_INT3 reading the dense form directly, so that the
 * weights go from their stored form to the GEMM's in one pass:
 *     pq_pack_operand_int3(g, pq_int3_pack(c), s) == pq_pack_operand(PQ_FMT_INT3, g, c, s)   byte for byte.
 * Errors: PQ_ERR_NULL, PQ_ERR_SHAPE (rows, K, alignment), PQ_ERR_FORMAT (group), PQ_ERR_WORKSPACE
 * (operand_size too small), PQ_ERR_HIP.  Asynchronous on `stream`.
 */
size_t pq_int3_dense_bytes(int64_t rows, int64_t K);
int pq_int3_pack(const uint8_t* codes, int64_t rows, int64_t K, uint8_t* dense, void* stream);
int pq_int3_unpack(const uint8_t* dense, int64_t rows, int64_t K, uint8_t* codes, void* stream);
int pq_pack_operand_int3(int group, const uint8_t* dense, const void* scales, int64_t rows, int64_t K,
                         void* operand, size_t operand_size, void* stream);

/*
 * The other reorder criteria of the ablation (paper Tab. 2a: variance, absmax, round-robin, random; the
 * paper names them without formulas, the readings are the library's).  A criterion supplies one
 * non-negative statistic per channel and side that takes the place of the second moment in the joint
 * score of Eq. 9: pq_select_perm accepts any such pair of arrays as act_sumsq / w_sumsq.
 *
 * pq_calib_channel_stats: per channel the sum (fp64, accumulated into sum[K]) and the largest magnitude
 *   (fp32, folded into absmax[K] by max) of x, bf16 [rows, ld]; either output may be NULL.  Call once per
 *   batch; workspace: pq_workspace_bytes(PQ_OP_CHANNEL_STATS, ., ., rows, 0, K, 0).
 * pq_channel_statistic: the statistic of a criterion from those sums, out[K] fp64:
 *   PQ_CRIT_VARIANCE  out = max(sumsq - sum^2 / n_rows, 0)   (n_rows times the biased variance)
 *   PQ_CRIT_ABSMAX    out = absmax^2
 * pq_order_by_score: the order of one alpha (Eq. 9, descending, ties in ascending channel order) without
 *   the error evaluation.  workspace: pq_workspace_bytes(PQ_OP_ORDER, ., ., 0, 0, K, 0).
 * pq_order_round_robin: deals the channels of `order` (best first) to the K / group groups in turn: rank r
 *   goes to position (r mod (K/group)) * group + r / (K/group).  K % group == 0; order != perm_out.
 * pq_order_random: a seeded permutation: channels sorted by splitmix64(seed + channel) >> 11, ascending,
 *   equal hashes in ascending channel order.  workspace as for pq_order_by_score.
 * All arrays are device memory; everything runs on `stream`.  Evaluate any order with pq_quant_error.
 */
typedef enum { PQ_CRIT_VARIANCE = 0, PQ_CRIT_ABSMAX = 1 } pq_criterion;
int pq_calib_channel_stats(const void* x_bf16, int64_t rows, int64_t K, int64_t ld, double* sum, float* absmax,
                           void* workspace, size_t workspace_bytes, void* stream);
int pq_channel_statistic(pq_criterion kind, const double* sum, const double* sumsq, const float* absmax,
                         int64_t n_rows, int64_t K, double* out, void* stream);
int pq_order_by_score(const double* act_stat, const double* w_stat, int64_t K, double alpha, int32_t* perm_out,
                      void* workspace, size_t workspace_bytes, void* stream);
int pq_order_round_robin(const int32_t* order, int64_t K, int group, int32_t* perm_out, void* stream);
int pq_order_random(uint64_t seed, int64_t K, int32_t* perm_out, void* workspace, size_t workspace_bytes,
                    void* stream);

/*
 * Dynamic per-tensor scale of the NVFP4 activation format (paper App. A.1: E4M3 block scales under an
 * fp32 tensor scale; the paper does not say whether the activation tensor scale is static).  The
 * default in this library is a static scale from the calibration absmax (pq_tensor_scale), which
 * keeps activation quantization a single pass.  This call is the first pass of the two-pass
 * alternative: T = max|x| / (448 * 6) of the live tensor x (bf16 [M, ld], first K columns), written to
 * tensor_scale_out (device float) on `stream`; pass it to pq_quantize_act(_packed) and to the product
 * that follows on the same stream -- nothing returns to the host.  K % 8 == 0, ld >= K, ld % 8 == 0.
 */
int pq_dynamic_tensor_scale(const void* x_bf16, int64_t M, int64_t K, int64_t ld, float* tensor_scale_out,
                            void* stream);

/*
 * The normalisation layer in front of a quantized linear layer, with the channel reorder
 * absorbed into its row load (paper App. C: RMSNorm and LayerNorm commute with a channel
 * permutation if the channel-wise vectors are permuted with it, so the layer can emit
 * y_P[m, j] = y[m, pi(j)] directly and the reorder costs no pass of its own).
 *
 *   PQ_NORM_RMS:    y[m, i] = x[m, i] / sqrt(mean_i x[m, i]^2 + eps) * gamma[i]
 *   PQ_NORM_ADALN:  y[m, i] = (1 + s[b(m), i]) * LN(x[m, :])[i] + b[b(m), i],
 *                   LN(x) = (x - mu) / sqrt(sigma^2 + eps), sigma^2 the biased variance,
 *                   b(m) = m / rows_per_mod (modulation vectors per sample).  A plain affine
 *                   LayerNorm is s = gamma - 1, b = beta with one modulation row.
 * Statistics and the affine part are computed in fp32 from the bf16 inputs; the result is
 * rounded once to bf16 (nearest even).  The quantizing variant then quantizes those bf16 values:
 *     pq_norm_quantize_act_packed(p, x) == pq_quantize_act_packed(pq_norm_reorder(p, x))   bit for bit.
 *
 * pq_norm_params (all pointers device memory, 16-byte aligned; vectors in the ORIGINAL channel order,
 * the library gathers them with the same pi):
 *   perm          int32 [K], a permutation of 0..K-1 as pq_select_perm emits it, or NULL (identity)
 *   gamma         bf16 [K] (RMS), NULL = ones
 *   mod_scale     bf16 [ceil(M / rows_per_mod), K] (ADALN), NULL = zeros
 *   mod_shift     bf16 [ceil(M / rows_per_mod), K] (ADALN), NULL = zeros
 *   rows_per_mod  tokens per modulation row; <= 0 means one row for all tokens
 *   eps           added to the mean square / variance under the root
 * x: bf16 [M, ld], ld >= K, ld % 8 == 0.  y: bf16 [M, ldy], ldy >= K, ldy % 8 == 0, may not overlap x.
 * K % 8 == 0 (K % 32 == 0 for the quantizing variant) and small enough for one row and the vectors
 * to be staged in a workgroup's LDS: 6 K bytes (RMS: 4 K) plus 4 bytes per INT group of a row must
 * stay below 159 KB (K <= 26000 for AdaLN), else PQ_ERR_SHAPE.
 * pq_norm_quantize_act_packed: operand as for pq_quantize_act_packed; y optional (NULL to skip;
 * ldy ignored then).  Both run on `stream` and return PQ_OK or a PQ_ERR_* code.
 */
typedef enum { PQ_NORM_RMS = 0, PQ_NORM_ADALN = 1 } pq_norm_kind;
typedef struct {
  pq_norm_kind kind;
  const int32_t* perm;
  const void* gamma;
  const void* mod_scale;
  const void* mod_shift;
  int64_t rows_per_mod;
  float eps;
} pq_norm_params;
int pq_norm_reorder(const pq_norm_params* p, const void* x_bf16, int64_t M, int64_t K, int64_t ld,
                    void* y_bf16, int64_t ldy, void* stream);
int pq_norm_quantize_act_packed(const pq_norm_params* p, pq_format fmt, int group, const void* x_bf16,
                                int64_t M, int64_t K, int64_t ld, const float* tensor_scale, void* operand,
                                size_t operand_size, void* y_bf16, int64_t ldy, void* stream);

/*
 * PermuQuant-H (paper App. D): the Hadamard rotation with the reorder applied after it, x H P -- the
 * permutation is the order in which the fast transform's output is consumed, no pass of its own.
 *     y_P[m, j] = (x[m, :] H)[pi(j)],   H H^T = I, entries +-1 / sqrt(K),
 * H = S_{2^k} (x) P_m / sqrt(K): the Sylvester matrix in natural order times, for K = 12 * 2^k or
 * 20 * 2^k, the Paley (type I) Hadamard matrix of order 12 or 20 (channel i = a * m + b); other widths
 * return PQ_ERR_SHAPE.  Computed in fp32 from the bf16 input, rounded once to bf16.  The same call on the
 * weight matrix (rows = output channels) gives the rotated weights to quantize offline, and on the
 * calibration batches the tensors whose moments drive the selection; (xH)(WH)^T = x W^T.
 * pq_hadamard_quantize_act_packed feeds the rounded values to the activation quantizer:
 *     == pq_quantize_act_packed(pq_hadamard_reorder(x))   bit for bit.
 * perm: int32 [K] device or NULL (identity).  x, y, ld, ldy, operand, tensor_scale as for pq_norm_reorder /
 * pq_norm_quantize_act_packed.  One fp32 row per wave is held in LDS: K <= 39000.
 */
int pq_hadamard_reorder(const int32_t* perm, const void* x_bf16, int64_t M, int64_t K, int64_t ld,
                        void* y_bf16, int64_t ldy, void* stream);
int pq_hadamard_quantize_act_packed(const int32_t* perm, pq_format fmt, int group, const void* x_bf16,
                                    int64_t M, int64_t K, int64_t ld, const float* tensor_scale,
                                    void* operand, size_t operand_size, void* y_bf16, int64_t ldy,
                                    void* stream);

/*
 * Measurement aids (no part of the method and not covered by the version contract of the calls above:
 * they may change with the kernels they are references for; they give the timings of the kernels above
 * a reference measured on the same device in the same run).
 *
 * pq_probe_stream: a plain streaming kernel that reads read_bytes from src and writes
 * write_bytes to dst (16 bytes per lane and access, no arithmetic worth naming) -- the time a
 * bandwidth-bound kernel with that footprint cannot beat.  Both sizes multiples of 16; src, dst
 * device buffers of at least those sizes, 16-byte aligned, may not overlap.
 *
 * pq_probe_mfma: every compute unit runs `iters` rounds of 8 independent
 * v_mfma_f32_32x32x16_f16 per wave (8 waves per unit, operands in registers, no memory
 * traffic); flops_out[0] (host double, may be NULL) receives the number of floating-point
 * operations issued, so that flops / time is the matrix rate the device sustains at the clock
 * it holds under that load.  sink: float [256 * 512] device buffer.
 */
int pq_probe_stream(const void* src, size_t read_bytes, void* dst, size_t write_bytes, void* stream);
int pq_probe_mfma(int iters, float* sink, double* flops_out, void* stream);
/*
 * pq_probe_mfma_operands: the same matrix-pipe-only loop on the values pq_qgemm_packed multiplies.  The
 * rate the matrix pipes sustain depends on the operand values (under its power limit the chip lowers its
 * clock, the sooner the more the operands switch from one instruction to the next), so the reference for
 * the product on given data is this loop on that data: every lane unpacks eight fragments of a_operand
 * and four of w_operand (operands as written by pq_quantize_act_packed / pq_pack_operand for these
 * fmt, group, M, N, K; K a multiple of 64) with the product kernel's own code and the loop cycles
 * through them.  sink, flops_out as for pq_probe_mfma.
 */
int pq_probe_mfma_operands(pq_format fmt, int group, const void* a_operand, const void* w_operand, int64_t M,
                           int64_t N, int64_t K, int iters, float* sink, double* flops_out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PERMUQUANT_H */
