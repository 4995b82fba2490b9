// Column second moments and running absmax (paper Sec. 3.2, mu_i^2 = E[x_i^2]; Sec. 3.3 uses
// them for activations and weights).  HBM-bound: every bf16 element is read once.
//
// Layout: a workgroup is 64 lanes (x) by kTy row-interleaved waves (y).  Lane l of every wave
// owns 4 consecutive columns (one 8-byte load per row), so a wave reads 512 contiguous bytes
// of a row.  grid.x tiles the columns, grid.y splits the rows into R slabs.  Each workgroup
// reduces its slab to one fp64 partial per column (squares of bf16 are exact in fp32, the
// accumulation is fp64), written to partial[slab][col]; a second kernel adds the R partials in
// slab order to sumsq, which keeps the result independent of scheduling.
#include "pq_device.h"
#include "pq_host.h"

namespace pq {

constexpr int kTy = 16;            // waves per workgroup
constexpr int kColsPerLane = 4;
constexpr int kColsPerBlock = 64 * kColsPerLane;

static int moments_slabs(int64_t rows, int64_t K) {
  int64_t col_blocks = (K + kColsPerBlock - 1) / kColsPerBlock;
  int64_t want = (320 + col_blocks - 1) / col_blocks;     // ~320 workgroups of 16 waves
  int64_t max_slabs = (rows + 4 * kTy - 1) / (4 * kTy);   // at least 4 rows per wave
  if (want > max_slabs) want = max_slabs;
  if (want < 1) want = 1;
  if (want > 64) want = 64;
  return (int)want;
}

size_t moments_workspace_bytes(int64_t rows, int64_t K) {
  return (size_t)moments_slabs(rows, K) * (size_t)K * sizeof(double);
}

__global__ __launch_bounds__(64 * kTy) void moments_partial_kernel(
    const uint16_t* __restrict__ x, int64_t rows, int64_t K, int64_t ld, int rows_per_slab,
    double* __restrict__ partial, uint32_t* __restrict__ absmax_bits) {
  __shared__ double red[kTy][64][kColsPerLane + 1];
  const int lane = threadIdx.x;
  const int ty = threadIdx.y;
  const int64_t col = (int64_t)blockIdx.x * kColsPerBlock + lane * kColsPerLane;
  const int64_t r0 = (int64_t)blockIdx.y * rows_per_slab;
  int64_t r1 = r0 + rows_per_slab;
  if (r1 > rows) r1 = rows;
  double acc[kColsPerLane] = {0.0, 0.0, 0.0, 0.0};
  uint32_t amax = 0;
  if (col < K) {
    const uint16_t* p = x + col;
    int64_t r = r0 + ty;
    // four independent loads in flight per lane
    for (; r + 3 * kTy < r1; r += 4 * kTy) {
      uint2 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = *reinterpret_cast<const uint2*>(p + (r + u * kTy) * ld);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        float f0 = bf16_lo(v[u].x), f1 = bf16_hi(v[u].x), f2 = bf16_lo(v[u].y), f3 = bf16_hi(v[u].y);
        acc[0] += (double)(f0 * f0);
        acc[1] += (double)(f1 * f1);
        acc[2] += (double)(f2 * f2);
        acc[3] += (double)(f3 * f3);
        uint32_t m0 = v[u].x & 0x7FFFu, m1 = (v[u].x >> 16) & 0x7FFFu;
        uint32_t m2 = v[u].y & 0x7FFFu, m3 = (v[u].y >> 16) & 0x7FFFu;
        uint32_t m = max(max(m0, m1), max(m2, m3));
        amax = max(amax, m);
      }
    }
    for (; r < r1; r += kTy) {
      uint2 v = *reinterpret_cast<const uint2*>(p + r * ld);
      float f0 = bf16_lo(v.x), f1 = bf16_hi(v.x), f2 = bf16_lo(v.y), f3 = bf16_hi(v.y);
      acc[0] += (double)(f0 * f0);
      acc[1] += (double)(f1 * f1);
      acc[2] += (double)(f2 * f2);
      acc[3] += (double)(f3 * f3);
      uint32_t m0 = v.x & 0x7FFFu, m1 = (v.x >> 16) & 0x7FFFu;
      uint32_t m2 = v.y & 0x7FFFu, m3 = (v.y >> 16) & 0x7FFFu;
      amax = max(amax, max(max(m0, m1), max(m2, m3)));
    }
  }
#pragma unroll
  for (int c = 0; c < kColsPerLane; ++c) red[ty][lane][c] = acc[c];
  __syncthreads();
  // wave 0..3 each finish one of the four columns of every lane, adding in wave order
  if (ty < kColsPerLane && col < K) {
    double s = 0.0;
#pragma unroll
    for (int w = 0; w < kTy; ++w) s += red[w][lane][ty];
    partial[(int64_t)blockIdx.y * K + col + ty] = s;
  }
  if (absmax_bits) {
    // |bf16| bit patterns of finite values order like the magnitudes; widen to fp32 bits
    float fm = wave_max(as_f32(amax << 16));
    if (lane == 0 && fm > 0.0f) atomicMax(absmax_bits, as_u32(fm));
  }
}

__global__ __launch_bounds__(256) void moments_finish_kernel(const double* __restrict__ partial,
                                                            int slabs, int64_t K,
                                                            double* __restrict__ sumsq) {
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= K) return;
  double s = 0.0;
  for (int r = 0; r < slabs; ++r) s += partial[(int64_t)r * K + i];
  sumsq[i] += s;
}

int launch_moments(const void* x, int64_t rows, int64_t K, int64_t ld, double* sumsq, float* absmax,
                   void* ws, hipStream_t st) {
  const int slabs = moments_slabs(rows, K);
  int rows_per_slab = (int)((rows + slabs - 1) / slabs);
  dim3 grid((unsigned)((K + kColsPerBlock - 1) / kColsPerBlock), (unsigned)slabs);
  dim3 block(64, kTy);
  hipLaunchKernelGGL(moments_partial_kernel, grid, block, 0, st, (const uint16_t*)x, rows, K, ld,
                     rows_per_slab, (double*)ws, (uint32_t*)absmax);
  int rc = check_hip(hipGetLastError(), "moments_partial_kernel");
  if (rc) return rc;
  hipLaunchKernelGGL(moments_finish_kernel, dim3((unsigned)((K + 255) / 256)), dim3(256), 0, st,
                     (const double*)ws, slabs, K, sumsq);
  return check_hip(hipGetLastError(), "moments_finish_kernel");
}

}  // namespace pq
