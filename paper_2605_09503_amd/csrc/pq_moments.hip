// Column second moments and running absmax (paper Sec. 3.2, mu_i^2 = E[x_i^2]; Sec. 3.3 uses
// them for activations and weights).  HBM-bound: every bf16 element is read once.
//
// A workgroup is 8 waves; a wave reads four rows at a time, sixteen lanes per row, a lane owning 8
// consecutive columns (one 16-byte load): a workgroup covers a strip of 128 columns (256 contiguous
// bytes per row) and a slab of rows.  grid.x tiles the columns, grid.y the row slabs, grid.z runs over
// the batches of one call.  Each workgroup reduces its slab to one fp64 partial per column (squares of
// bf16 are exact, the accumulation is fp64) and one absmax, written to partial[batch][slab][col] /
// blockmax[...]; a second small kernel adds the partials in (batch, slab) order to sumsq and folds the
// maxima, which keeps the result independent of scheduling and free of atomics.
//
// (One launch instead of two -- the workgroup that arrives last at a strip's counter adds the strip's
// partials up -- was built and measured on c1's 28 MB batch, 9 us with two launches: 160 us with
// device-scope fences around the hand-over (each one writes back and invalidates a whole L2), 77 us
// with device-scope atomic accesses for the few values that cross and a compare-and-swap ticket, 23 us
// with a fetch-add ticket -- the 32 arrivals at one address are served one after the other, about
// 0.6 us each.  Two launches stay.)
#include <mutex>

#include "pq_device.h"
#include "pq_host.h"

namespace pq {

constexpr int kTy = 8;               // waves per workgroup
constexpr int kColsPerLane = 8;
constexpr int kLanesPerRow = 16;     // lanes of a wave that share a row
constexpr int kRowsPerWave = 64 / kLanesPerRow;
constexpr int kRowsPerPass = kTy * kRowsPerWave;            // rows a workgroup reads per pass
constexpr int kStripCols = kLanesPerRow * kColsPerLane;     // 128 columns per workgroup
constexpr int kMaxSlabs = 64;

struct BatchPtrs {
  const uint16_t* p[kMaxMomentBatches];
};

static int64_t strip_count(int64_t K) { return (K + kStripCols - 1) / kStripCols; }

// Row slabs per (strip, batch): about three workgroups per compute unit in total, every slab at least
// two passes long.
static int moments_slabs(int64_t rows, int64_t K, int n_batches) {
  const int64_t per_slab = strip_count(K) * n_batches;
  int64_t want = (768 + per_slab - 1) / per_slab;
  const int64_t max_slabs = (rows + 2 * kRowsPerPass - 1) / (2 * kRowsPerPass);
  if (want > max_slabs) want = max_slabs;
  if (want > kMaxSlabs) want = kMaxSlabs;
  if (want < 1) want = 1;
  return (int)want;
}

struct MomentsWs {
  double* partial;                // [n_batches * slabs][K]
  float* blockmax;                // [n_batches * slabs][strips]
};

static size_t carve_moments(void* base, int64_t K, int slabs, int n_batches, MomentsWs* w) {
  const size_t strips = (size_t)strip_count(K);
  const size_t o_max = align_up((size_t)n_batches * slabs * (size_t)K * sizeof(double), 256);
  const size_t total = o_max + align_up((size_t)n_batches * slabs * strips * sizeof(float), 256);
  if (w) {
    w->partial = (double*)base;
    w->blockmax = (float*)((char*)base + o_max);
  }
  return total;
}

size_t moments_workspace_bytes(int64_t rows, int64_t K, int n_batches) {
  if (n_batches < 1) n_batches = 1;
  const int per_launch = n_batches < kMaxMomentBatches ? n_batches : kMaxMomentBatches;
  // a call is cut into launches of at most kMaxMomentBatches batches; cover the largest need
  size_t need = 0;
  for (int nb = 1; nb <= per_launch; ++nb) {
    const size_t b = carve_moments(nullptr, K, moments_slabs(rows, K, nb), nb, nullptr);
    if (b > need) need = b;
  }
  return need;
}

__global__ __launch_bounds__(64 * kTy) void moments_partial_kernel(BatchPtrs xs, int64_t rows, int64_t K,
                                                                  int64_t ld, int rows_per_slab,
                                                                  double* __restrict__ partial,
                                                                  float* __restrict__ blockmax) {
  __shared__ double red[kTy * kRowsPerWave][kLanesPerRow][kColsPerLane + 1];
  __shared__ double share[4][kStripCols];
  __shared__ float red_max[kTy];
  const int lane = threadIdx.x;
  const int ty = threadIdx.y;
  const int tid = ty * 64 + lane;
  const int sub = lane / kLanesPerRow, cl = lane % kLanesPerRow;
  const uint16_t* __restrict__ x = xs.p[blockIdx.z];
  const int64_t col0 = (int64_t)blockIdx.x * kStripCols;
  const int64_t col = col0 + cl * kColsPerLane;
  const int64_t r0 = (int64_t)blockIdx.y * rows_per_slab;
  int64_t r1 = r0 + rows_per_slab;
  if (r1 > rows) r1 = rows;
  double acc[kColsPerLane];
#pragma unroll
  for (int c = 0; c < kColsPerLane; ++c) acc[c] = 0.0;
  // |bf16| bit patterns of finite values order like the magnitudes: the running maximum is kept
  // as two 16-bit lanes of one register (even and odd columns), one packed max per two elements
  typedef uint16_t u16x2 __attribute__((ext_vector_type(2)));
  u16x2 amax2 = {0, 0};
  auto accumulate = [&](const uint4& v) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const double d0 = (double)bf16_lo(w[j]), d1 = (double)bf16_hi(w[j]);
      acc[2 * j] = fma(d0, d0, acc[2 * j]);          // the square is exact, one rounding per element
      acc[2 * j + 1] = fma(d1, d1, acc[2 * j + 1]);
      amax2 = __builtin_elementwise_max(amax2, __builtin_bit_cast(u16x2, w[j] & 0x7FFF7FFFu));
    }
  };
  if (col < K) {
    const uint16_t* p = x + col;
    int64_t r = r0 + ty * kRowsPerWave + sub;
    // four independent 16-byte loads in flight per lane
    for (; r + 3 * kRowsPerPass < r1; r += 4 * kRowsPerPass) {
      uint4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = *reinterpret_cast<const uint4*>(p + (r + u * kRowsPerPass) * ld);
#pragma unroll
      for (int u = 0; u < 4; ++u) accumulate(v[u]);
    }
    for (; r < r1; r += kRowsPerPass) accumulate(*reinterpret_cast<const uint4*>(p + r * ld));
  }
#pragma unroll
  for (int c = 0; c < kColsPerLane; ++c) red[ty * kRowsPerWave + sub][cl][c] = acc[c];
  // widen the larger of the two 16-bit maxima to fp32 bits
  const uint32_t amax = max((uint32_t)amax2.x, (uint32_t)amax2.y);
  const float fm = wave_max(as_f32(amax << 16));
  if (lane == 0) red_max[ty] = fm;
  __syncthreads();
  // thread (part, j): column j of the strip, a quarter of the 32 row groups, added in index order; the
  // four quarters are then added in order by the threads of part 0
  const int j = tid % kStripCols, part = tid / kStripCols;
  {
    double s = 0.0;
#pragma unroll
    for (int q = 0; q < kTy * kRowsPerWave / 4; ++q)
      s += red[part * (kTy * kRowsPerWave / 4) + q][j / kColsPerLane][j % kColsPerLane];
    share[part][j] = s;
  }
  __syncthreads();
  const int64_t part_index = (int64_t)blockIdx.z * gridDim.y + blockIdx.y;
  if (part == 0 && col0 + j < K)
    partial[part_index * K + col0 + j] = ((share[0][j] + share[1][j]) + share[2][j]) + share[3][j];
  if (tid == 0) {
    float m = 0.0f;
#pragma unroll
    for (int w = 0; w < kTy; ++w) m = fmaxf(m, red_max[w]);
    blockmax[part_index * gridDim.x + blockIdx.x] = m;
  }
}

// sumsq[i] += sum of the partials of column i.  A workgroup covers kFinCols columns; its threads form
// kFinParts groups that each add a contiguous share of the partials in order, and the shares are
// combined in group order: the result does not depend on scheduling.
constexpr int kFinCols = 16, kFinParts = 16;
__global__ __launch_bounds__(kFinCols * kFinParts) void moments_finish_kernel(const double* __restrict__ partial,
                                                                             int n_partials, int64_t K,
                                                                             double* __restrict__ sumsq,
                                                                             const float* __restrict__ blockmax,
                                                                             int n_blockmax, float* __restrict__ absmax) {
  __shared__ double share[kFinParts][kFinCols];
  const int col = threadIdx.x % kFinCols, part = threadIdx.x / kFinCols;
  const int64_t i = (int64_t)blockIdx.x * kFinCols + col;
  const int per = (n_partials + kFinParts - 1) / kFinParts;
  const int r0 = part * per, r1 = min(n_partials, r0 + per);
  double s = 0.0;
  if (i < K) {
    int r = r0;
    for (; r + 8 <= r1; r += 8) {                  // independent loads, fixed order of additions
      double v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = partial[(int64_t)(r + u) * K + i];
#pragma unroll
      for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; r < r1; ++r) s += partial[(int64_t)r * K + i];
  }
  share[part][col] = s;
  __syncthreads();
  if (part == 0 && i < K) {
    double t = 0.0;
#pragma unroll
    for (int p = 0; p < kFinParts; ++p) t += share[p][col];
    sumsq[i] += t;
  }
  if (absmax && blockIdx.x == 0) {
    float m = 0.0f;
    for (int b = threadIdx.x; b < n_blockmax; b += kFinCols * kFinParts) m = fmaxf(m, blockmax[b]);
    m = wave_max(m);
    __shared__ float wm[4];
    if ((threadIdx.x & 63) == 0) wm[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
      m = fmaxf(fmaxf(wm[0], wm[1]), fmaxf(wm[2], wm[3]));
      absmax[0] = fmaxf(absmax[0], m);
    }
  }
}

int launch_moments(const void* const* xs, int n_batches, int64_t rows, int64_t K, int64_t ld,
                   double* sumsq, float* absmax, void* ws, hipStream_t st) {
  for (int b0 = 0; b0 < n_batches; b0 += kMaxMomentBatches) {
    const int nb = n_batches - b0 < kMaxMomentBatches ? n_batches - b0 : kMaxMomentBatches;
    const int slabs = moments_slabs(rows, K, nb);
    const int rows_per_slab = (int)((rows + slabs - 1) / slabs);
    BatchPtrs bp;
    for (int b = 0; b < kMaxMomentBatches; ++b) bp.p[b] = (const uint16_t*)xs[b0 + (b < nb ? b : 0)];
    MomentsWs W;
    carve_moments(ws, K, slabs, nb, &W);
    const unsigned strips = (unsigned)strip_count(K);
    hipLaunchKernelGGL(moments_partial_kernel, dim3(strips, (unsigned)slabs, (unsigned)nb), dim3(64, kTy), 0, st, bp,
                       rows, K, ld, rows_per_slab, W.partial, W.blockmax);
    int rc = check_hip(hipGetLastError(), "moments_partial_kernel");
    if (rc) return rc;
    hipLaunchKernelGGL(moments_finish_kernel, dim3((unsigned)((K + kFinCols - 1) / kFinCols)),
                       dim3(kFinCols * kFinParts), 0, st, (const double*)W.partial, nb * slabs, K, sumsq,
                       (const float*)W.blockmax, (int)(strips * slabs * nb), absmax);
    rc = check_hip(hipGetLastError(), "moments_finish_kernel");
    if (rc) return rc;
  }
  return PQ_OK;
}

// ---------------------------------------------------------------- scratch held by the library
// pq_calib_moments_static: the same two kernels with their partial sums in a device array that is
// part of the loaded code object, for callers that cannot bring a workspace (none may be allocated
// where they run).  Every GPU the library runs on holds its own copy of the array at its own
// address; in host code the array's name is only a handle for hipGetSymbolAddress, so the device
// address is looked up once per device (with that device current) and only that pointer is handed
// to the kernels.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices];      // device address of `scratch` per device, nullptr = not yet asked

static int static_scratch(void** out) {
  int dev = -1;
  int rc = check_hip(hipGetDevice(&dev), "hipGetDevice");
  if (rc) return rc;
  if (dev < 0 || dev >= kMaxDevices) return fail(PQ_ERR_HIP, "device index %d outside 0..%d", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    rc = check_hip(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)");
    if (rc) return rc;
    if (!p) return fail(PQ_ERR_HIP, "hipGetSymbolAddress(scratch) returned a null address");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return PQ_OK;
}

int launch_moments_static(const void* x, int64_t rows, int64_t K, int64_t ld, double* sumsq, float* absmax,
                          hipStream_t st) {
  const size_t need = moments_workspace_bytes(rows, K, 1);
  if (need > kStaticScratchBytes)
    return fail(PQ_ERR_WORKSPACE,
                "pq_calib_moments_static: rows=%lld K=%lld need %zu bytes of scratch, the library holds %zu; "
                "use pq_calib_moments with a workspace",
                (long long)rows, (long long)K, need, (size_t)kStaticScratchBytes);
  void* ws = nullptr;
  int rc = static_scratch(&ws);
  if (rc) return rc;
  const void* xs[1] = {x};
  // every partial sum and maximum the second kernel reads is written by the first one in this call:
  // nothing in the array has to start at zero
  return launch_moments(xs, 1, rows, K, ld, sumsq, absmax, ws, st);
}

// ---------------------------------------------------------------- per-channel sum and absmax
constexpr int kColsPerBlock = 64 * kColsPerLane;      // here a wave reads 1 KB of one row at a time
// Statistics of the alternative reorder criteria (paper Tab. 2a: variance, absmax): per column the
// sum (fp64) and the largest magnitude.  Same decomposition as above: partials per row slab, then a
// second kernel that folds them in slab order.
__global__ __launch_bounds__(64 * kTy) void channel_stats_partial_kernel(const uint16_t* __restrict__ x, int64_t rows,
                                                                        int64_t K, int64_t ld, int rows_per_slab,
                                                                        double* __restrict__ psum,
                                                                        float* __restrict__ pmax) {
  __shared__ double red[kTy][64][kColsPerLane + 1];
  __shared__ uint32_t redm[kTy][64][kColsPerLane + 1];
  const int lane = threadIdx.x, ty = threadIdx.y;
  const int64_t col = (int64_t)blockIdx.x * kColsPerBlock + lane * kColsPerLane;
  const int64_t r0 = (int64_t)blockIdx.y * rows_per_slab;
  const int64_t r1 = r0 + rows_per_slab < rows ? r0 + rows_per_slab : rows;
  double acc[kColsPerLane];
  uint32_t amax[kColsPerLane];           // |bf16| bit patterns order like the magnitudes
#pragma unroll
  for (int c = 0; c < kColsPerLane; ++c) acc[c] = 0.0, amax[c] = 0u;
  if (col < K) {
    const uint16_t* p = x + col;
    for (int64_t r = r0 + ty; r < r1; r += kTy) {
      const uint4 v = *reinterpret_cast<const uint4*>(p + r * ld);
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        acc[2 * j] += (double)bf16_lo(w[j]);
        acc[2 * j + 1] += (double)bf16_hi(w[j]);
        amax[2 * j] = max(amax[2 * j], w[j] & 0x7FFFu);
        amax[2 * j + 1] = max(amax[2 * j + 1], (w[j] >> 16) & 0x7FFFu);
      }
    }
  }
#pragma unroll
  for (int c = 0; c < kColsPerLane; ++c) red[ty][lane][c] = acc[c], redm[ty][lane][c] = amax[c];
  __syncthreads();
  if (ty < kColsPerLane && col < K) {
    double s = 0.0;
    uint32_t m = 0u;
#pragma unroll
    for (int w = 0; w < kTy; ++w) s += red[w][lane][ty], m = max(m, redm[w][lane][ty]);
    psum[(int64_t)blockIdx.y * K + col + ty] = s;
    pmax[(int64_t)blockIdx.y * K + col + ty] = as_f32(m << 16);
  }
}

__global__ __launch_bounds__(256) void channel_stats_finish_kernel(const double* __restrict__ psum,
                                                                  const float* __restrict__ pmax, int slabs,
                                                                  int64_t K, double* __restrict__ sum,
                                                                  float* __restrict__ absmax) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= K) return;
  double s = 0.0;
  float m = 0.0f;
  for (int r = 0; r < slabs; ++r) {
    s += psum[(int64_t)r * K + i];
    m = fmaxf(m, pmax[(int64_t)r * K + i]);
  }
  if (sum) sum[i] += s;
  if (absmax) absmax[i] = fmaxf(absmax[i], m);
}

static int channel_stats_slabs(int64_t rows, int64_t K) {
  const int64_t col_blocks = (K + kColsPerBlock - 1) / kColsPerBlock;
  int64_t want = (1024 + col_blocks - 1) / col_blocks;
  const int64_t max_slabs = (rows + 4 * kTy - 1) / (4 * kTy);
  if (want > max_slabs) want = max_slabs;
  if (want < 1) want = 1;
  if (want > 256) want = 256;
  return (int)want;
}

size_t channel_stats_workspace_bytes(int64_t rows, int64_t K) {
  const int slabs = channel_stats_slabs(rows, K);
  return align_up((size_t)slabs * K * sizeof(double), 256) + align_up((size_t)slabs * K * sizeof(float), 256);
}

int launch_channel_stats(const void* x, int64_t rows, int64_t K, int64_t ld, double* sum, float* absmax, void* ws,
                         hipStream_t st) {
  const int slabs = channel_stats_slabs(rows, K);
  const int rows_per_slab = (int)((rows + slabs - 1) / slabs);
  double* psum = (double*)ws;
  float* pmax = (float*)((char*)ws + align_up((size_t)slabs * K * sizeof(double), 256));
  hipLaunchKernelGGL(channel_stats_partial_kernel, dim3((unsigned)((K + kColsPerBlock - 1) / kColsPerBlock), (unsigned)slabs),
                     dim3(64, kTy), 0, st, (const uint16_t*)x, rows, K, ld, rows_per_slab, psum, pmax);
  hipLaunchKernelGGL(channel_stats_finish_kernel, dim3((unsigned)((K + 255) / 256)), dim3(256), 0, st,
                     (const double*)psum, (const float*)pmax, slabs, K, sum, absmax);
  return check_hip(hipGetLastError(), "channel_stats kernels");
}

// out[i] = max(sumsq[i] - sum[i]^2 / n, 0): n times the biased variance of channel i
__global__ __launch_bounds__(256) void channel_variance_kernel(const double* __restrict__ sum,
                                                              const double* __restrict__ sumsq, double n, int64_t K,
                                                              double* __restrict__ out) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < K) out[i] = fmax(sumsq[i] - sum[i] * sum[i] / n, 0.0);
}

// out[i] = absmax[i]^2 as a double (the statistic of the absmax criterion, in the units of a second moment)
__global__ __launch_bounds__(256) void channel_absmax_sq_kernel(const float* __restrict__ absmax, int64_t K,
                                                               double* __restrict__ out) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < K) out[i] = (double)absmax[i] * (double)absmax[i];
}

int launch_channel_variance(const double* sum, const double* sumsq, int64_t n_rows, int64_t K, double* out,
                            hipStream_t st) {
  hipLaunchKernelGGL(channel_variance_kernel, dim3((unsigned)((K + 255) / 256)), dim3(256), 0, st, sum, sumsq,
                     (double)n_rows, K, out);
  return check_hip(hipGetLastError(), "channel_variance_kernel");
}

int launch_channel_absmax_sq(const float* absmax, int64_t K, double* out, hipStream_t st) {
  hipLaunchKernelGGL(channel_absmax_sq_kernel, dim3((unsigned)((K + 255) / 256)), dim3(256), 0, st, absmax, K, out);
  return check_hip(hipGetLastError(), "channel_absmax_sq_kernel");
}

}  // namespace pq
