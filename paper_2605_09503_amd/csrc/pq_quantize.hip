// Per-group quantizers (paper Sec. 3.1, Eq. 1-2; NVFP4 two-level scales): dynamic activation
// quantization and offline weight quantization share these kernels.
//
// Work split: one lane owns 8 consecutive channels (one 16-byte load of bf16, one 4-byte store
// of codes); the G/8 lanes of a group find the group maximum with a lane reduction; every lane
// then computes the (identical) group scale and its own eight codes.  HBM-bound: 2 bytes in,
// 0.5 byte + scale out per element.
//
//   quantize_flat_kernel   contiguous rows in their stored order: no index arithmetic at all
//                          (chunk c of the flattened tensor is bytes [16c, 16c+16)).
//   quantize_rows_kernel   one workgroup per row; handles a row stride and the optional
//                          channel gather x[row, perm[k]] (offline weights, calibration, tests).
#include "pq_device.h"
#include "pq_host.h"

namespace pq {

template <int FMT>
struct ChunkOut {
  uint32_t codes;   // 8 nibbles, element j at bits 4j
  uint32_t scale;   // INT: fp32 bits; NVFP4: E4M3 byte
};

// v[8]: this lane's eight channels.  G: group size.  All G/8 lanes of a group call together.
template <int FMT, int G>
__device__ __forceinline__ ChunkOut<FMT> quantize_chunk(const float (&v)[8], float T, float encT) {
  float a = fmaxf(fmaxf(fmaxf(fabsf(v[0]), fabsf(v[1])), fmaxf(fabsf(v[2]), fabsf(v[3]))),
                  fmaxf(fmaxf(fabsf(v[4]), fabsf(v[5])), fmaxf(fabsf(v[6]), fabsf(v[7]))));
  a = group_max<G / 8>(a);
  ChunkOut<FMT> o;
  uint32_t c = 0;
  if constexpr (FMT == kNvfp4) {
    Nv4Scale s = nv4_scale(a, T, encT);
    // the conversion unit rounds, saturates, keeps the sign and packs two codes per byte
    c = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(c, v[0] * s.inv, v[1] * s.inv, 1.0f, 0);
    c = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(c, v[2] * s.inv, v[3] * s.inv, 1.0f, 1);
    c = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(c, v[4] * s.inv, v[5] * s.inv, 1.0f, 2);
    c = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(c, v[6] * s.inv, v[7] * s.inv, 1.0f, 3);
    o.scale = s.byte;
  } else {
    IntScale s = int_scale<FMT>(a);
    c = int_codes8(v, s.inv);
    o.scale = as_u32(s.s);
  }
  o.codes = c;
  return o;
}

__device__ __forceinline__ void unpack8(const uint4& p, float (&v)[8]) {
  v[0] = bf16_lo(p.x); v[1] = bf16_hi(p.x);
  v[2] = bf16_lo(p.y); v[3] = bf16_hi(p.y);
  v[4] = bf16_lo(p.z); v[5] = bf16_hi(p.z);
  v[6] = bf16_lo(p.w); v[7] = bf16_hi(p.w);
}

template <int FMT>
__device__ __forceinline__ void store_scale(void* scales, int64_t g, uint32_t s) {
  if constexpr (FMT == kNvfp4) reinterpret_cast<uint8_t*>(scales)[g] = (uint8_t)s;
  else reinterpret_cast<uint32_t*>(scales)[g] = s;
}

constexpr int kFlatUnroll = 2;

template <int FMT, int G>
__global__ __launch_bounds__(256) void quantize_flat_kernel(const uint4* __restrict__ x,
                                                            int64_t n_chunks,
                                                            const float* __restrict__ tensor_scale,
                                                            uint32_t* __restrict__ codes,
                                                            void* __restrict__ scales) {
  float T = 0.0f, encT = 0.0f;
  if constexpr (FMT == kNvfp4) {
    T = *tensor_scale;
    encT = nv4_enc_scale(T);
  }
  const int64_t base = (int64_t)blockIdx.x * (256 * kFlatUnroll) + threadIdx.x;
  uint4 p[kFlatUnroll];
#pragma unroll
  for (int u = 0; u < kFlatUnroll; ++u) {
    int64_t c = base + u * 256;
    p[u] = (c < n_chunks) ? x[c] : make_uint4(0, 0, 0, 0);
  }
#pragma unroll
  for (int u = 0; u < kFlatUnroll; ++u) {
    int64_t c = base + u * 256;
    float v[8];
    unpack8(p[u], v);
    // whole groups are in or out together: n_chunks is a multiple of G/8 and c is lane-aligned
    ChunkOut<FMT> o = quantize_chunk<FMT, G>(v, T, encT);
    if (c < n_chunks) {
      codes[c] = o.codes;
      if ((c & (G / 8 - 1)) == 0) store_scale<FMT>(scales, c / (G / 8), o.scale);
    }
  }
}

template <int FMT, int G>
__global__ __launch_bounds__(256) void quantize_rows_kernel(const uint16_t* __restrict__ x, int64_t K,
                                                            int64_t ld,
                                                            const int32_t* __restrict__ perm,
                                                            const float* __restrict__ tensor_scale,
                                                            uint32_t* __restrict__ codes,
                                                            void* __restrict__ scales, int staged) {
  extern __shared__ __align__(16) uint16_t row_lds[];       // staged: the row, K elements
  float T = 0.0f, encT = 0.0f;
  if constexpr (FMT == kNvfp4) {
    T = *tensor_scale;
    encT = nv4_enc_scale(T);
  }
  const int64_t row = blockIdx.x;
  const uint16_t* xr = x + row * ld;
  const int chunks = (int)(K / 8);
  // gather: the row is read once in whole lines and the channels are picked out of LDS (scattered
  // two-byte reads from memory keep the texture addresser busy a cycle per lane)
  const uint16_t* src = xr;
  if (staged) {
    for (int c = threadIdx.x; c < chunks; c += 256)
      reinterpret_cast<uint4*>(row_lds)[c] = *reinterpret_cast<const uint4*>(xr + (int64_t)c * 8);
    __syncthreads();
    src = row_lds;
  }
  // all 256 lanes iterate together so the group reduction always sees whole groups
  for (int c0 = 0; c0 < chunks; c0 += 256) {
    int c = c0 + threadIdx.x;
    float v[8];
    if (c < chunks) {
      if (perm) {
        const int4* pp = reinterpret_cast<const int4*>(perm + (int64_t)c * 8);
        int4 i0 = pp[0], i1 = pp[1];
        v[0] = bf16_to_f32(src[i0.x]); v[1] = bf16_to_f32(src[i0.y]);
        v[2] = bf16_to_f32(src[i0.z]); v[3] = bf16_to_f32(src[i0.w]);
        v[4] = bf16_to_f32(src[i1.x]); v[5] = bf16_to_f32(src[i1.y]);
        v[6] = bf16_to_f32(src[i1.z]); v[7] = bf16_to_f32(src[i1.w]);
      } else {
        unpack8(*reinterpret_cast<const uint4*>(xr + (int64_t)c * 8), v);
      }
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = 0.0f;
    }
    ChunkOut<FMT> o = quantize_chunk<FMT, G>(v, T, encT);
    if (c < chunks) {
      codes[row * chunks + c] = o.codes;
      if ((c & (G / 8 - 1)) == 0) store_scale<FMT>(scales, row * (K / G) + c / (G / 8), o.scale);
    }
  }
}

template <int FMT, int G>
static int launch_q(const void* x, int64_t rows, int64_t K, int64_t ld, const int32_t* perm,
                    const float* ts, uint8_t* codes, void* scales, hipStream_t st) {
  if (!perm && ld == K) {
    int64_t n_chunks = rows * K / 8;
    int64_t blocks = (n_chunks + 256 * kFlatUnroll - 1) / (256 * kFlatUnroll);
    hipLaunchKernelGGL((quantize_flat_kernel<FMT, G>), dim3((unsigned)blocks), dim3(256), 0, st,
                       (const uint4*)x, n_chunks, ts, (uint32_t*)codes, scales);
    return check_hip(hipGetLastError(), "quantize_flat_kernel");
  }
  // with a gather the row goes through LDS when it fits 48 KB
  const int staged = perm && K * 2 <= 48 * 1024 ? 1 : 0;
  hipLaunchKernelGGL((quantize_rows_kernel<FMT, G>), dim3((unsigned)rows), dim3(256), staged ? (size_t)K * 2 : 0, st,
                     (const uint16_t*)x, K, ld, perm, ts, (uint32_t*)codes, scales, staged);
  return check_hip(hipGetLastError(), "quantize_rows_kernel");
}

int launch_quantize_rows(pq_format fmt, int group, const void* x, int64_t rows, int64_t K, int64_t ld,
                         const int32_t* perm, const float* ts, uint8_t* codes, void* scales,
                         hipStream_t st) {
  if (rows > 0x7FFFFFFF) return fail(PQ_ERR_SHAPE, "too many rows");
  if (fmt == PQ_FMT_NVFP4) return launch_q<kNvfp4, 16>(x, rows, K, ld, perm, ts, codes, scales, st);
#define PQ_INT_CASE(F, FE)                                                                   \
  if (fmt == F) {                                                                            \
    switch (group) {                                                                         \
      case 32: return launch_q<FE, 32>(x, rows, K, ld, perm, ts, codes, scales, st);         \
      case 64: return launch_q<FE, 64>(x, rows, K, ld, perm, ts, codes, scales, st);         \
      case 128: return launch_q<FE, 128>(x, rows, K, ld, perm, ts, codes, scales, st);       \
      case 256: return launch_q<FE, 256>(x, rows, K, ld, perm, ts, codes, scales, st);       \
    }                                                                                        \
  }
  PQ_INT_CASE(PQ_FMT_INT4, kInt4)
  PQ_INT_CASE(PQ_FMT_INT3, kInt3)
#undef PQ_INT_CASE
  return fail(PQ_ERR_FORMAT, "unsupported (format, group) = (%d, %d)", (int)fmt, group);
}

// ------------------------------------------------------------------ NVFP4 tensor scale
// The maximum of a workgroup goes to the one result word with a single atomic max (an integer max of
// non-negative float bit patterns: order-free, so the result is deterministic).  Atomics on one address
// are served one after the other, some 12 ns each from all over the chip: with an atomic per wave of
// 2048 workgroups the weight tensor of an MLP layer took 100 us, of which the read was 15; hence few
// workgroups (two per compute unit), one atomic each, and four loads in flight per lane.
constexpr int kAbsmaxBlocks = 512;
__device__ __forceinline__ void block_absmax_to(uint32_t m, uint32_t* out_bits) {
  __shared__ float wave_m[4];
  const float fm = wave_max(as_f32(m << 16));
  if ((threadIdx.x & 63) == 0) wave_m[threadIdx.x >> 6] = fm;
  __syncthreads();
  if (threadIdx.x == 0) {
    const float all = fmaxf(fmaxf(wave_m[0], wave_m[1]), fmaxf(wave_m[2], wave_m[3]));
    if (all > 0.0f) atomicMax(out_bits, as_u32(all));
  }
}
__device__ __forceinline__ uint32_t absmax16(uint32_t m, const uint4& p) {
  // |bf16| bit patterns of finite values order like the magnitudes; two 16-bit lanes per register
  typedef uint16_t u16x2 __attribute__((ext_vector_type(2)));
  u16x2 a = __builtin_bit_cast(u16x2, m);
  const uint32_t w[4] = {p.x, p.y, p.z, p.w};
#pragma unroll
  for (int j = 0; j < 4; ++j) a = __builtin_elementwise_max(a, __builtin_bit_cast(u16x2, w[j] & 0x7FFF7FFFu));
  return __builtin_bit_cast(uint32_t, a);
}
__global__ __launch_bounds__(256) void absmax_kernel(const uint4* __restrict__ x, int64_t n_chunks,
                                                     uint32_t* __restrict__ out_bits) {
  uint32_t m2 = 0;                                      // running maxima of the even and the odd elements
  const int64_t stride = (int64_t)gridDim.x * 256;
  int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;
  for (; c + 3 * stride < n_chunks; c += 4 * stride) {
    uint4 p[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) p[u] = x[c + u * stride];
#pragma unroll
    for (int u = 0; u < 4; ++u) m2 = absmax16(m2, p[u]);
  }
  for (; c < n_chunks; c += stride) m2 = absmax16(m2, x[c]);
  block_absmax_to(max(m2 & 0xFFFFu, m2 >> 16), out_bits);
}

__global__ void zero_word_kernel(uint32_t* p) { *p = 0u; }

// in place: absmax -> T = absmax / (448 * 6)
__global__ void tensor_scale_kernel(float* p) { *p = *p / 2688.0f; }

__global__ void tensor_scale_from_kernel(const float* a, float* t) { *t = *a / 2688.0f; }

__global__ void fill_float_kernel(float* p, float v) { *p = v; }

int launch_tensor_scale(const float* absmax, float* out, hipStream_t st) {
  hipLaunchKernelGGL(tensor_scale_from_kernel, dim3(1), dim3(1), 0, st, absmax, out);
  return check_hip(hipGetLastError(), "tensor_scale_from_kernel");
}

int launch_fill_float(float* p, float v, hipStream_t st) {
  hipLaunchKernelGGL(fill_float_kernel, dim3(1), dim3(1), 0, st, p, v);
  return check_hip(hipGetLastError(), "fill_float_kernel");
}

// absmax over the first K columns of every row of a tensor with row stride ld (the columns beyond
// K are not read)
__global__ __launch_bounds__(256) void absmax_rows_kernel(const uint16_t* __restrict__ x, int64_t rows, int k_chunks,
                                                          int64_t ld, uint32_t* __restrict__ out_bits) {
  uint32_t m2 = 0;
  const int64_t n_chunks = rows * k_chunks;
  for (int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x; c < n_chunks; c += (int64_t)gridDim.x * 256) {
    const int64_t r = c / k_chunks;
    const int col = (int)(c - r * k_chunks);
    m2 = absmax16(m2, *reinterpret_cast<const uint4*>(x + r * ld + (int64_t)col * 8));
  }
  block_absmax_to(max(m2 & 0xFFFFu, m2 >> 16), out_bits);
}

// The per-tensor scale of a live activation tensor, T = max|x| / (448 * 6), left in device memory
// for the quantizer and the GEMM that follow on the same stream (the first of the two passes of a
// dynamic NVFP4 tensor scale).
int launch_dynamic_tensor_scale(const void* x, int64_t rows, int64_t K, int64_t ld, float* out, hipStream_t st) {
  const int64_t n_chunks = rows * (K / 8);
  int64_t blocks = (n_chunks + 255) / 256;
  if (blocks > kAbsmaxBlocks) blocks = kAbsmaxBlocks;
  hipLaunchKernelGGL(zero_word_kernel, dim3(1), dim3(1), 0, st, (uint32_t*)out);
  if (ld == K) {
    hipLaunchKernelGGL(absmax_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const uint4*)x, n_chunks,
                       (uint32_t*)out);
  } else {
    hipLaunchKernelGGL(absmax_rows_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const uint16_t*)x, rows,
                       (int)(K / 8), ld, (uint32_t*)out);
  }
  hipLaunchKernelGGL(tensor_scale_kernel, dim3(1), dim3(1), 0, st, out);
  return check_hip(hipGetLastError(), "absmax/tensor_scale kernels");
}

int launch_absmax_to_tensor_scale(const void* x, int64_t n_elems, float* out, hipStream_t st) {
  int64_t n_chunks = n_elems / 8;          // K is a multiple of 16, so no tail
  int64_t blocks = (n_chunks + 255) / 256;
  if (blocks > kAbsmaxBlocks) blocks = kAbsmaxBlocks;
  hipLaunchKernelGGL(zero_word_kernel, dim3(1), dim3(1), 0, st, (uint32_t*)out);
  hipLaunchKernelGGL(absmax_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const uint4*)x, n_chunks,
                     (uint32_t*)out);
  hipLaunchKernelGGL(tensor_scale_kernel, dim3(1), dim3(1), 0, st, out);
  return check_hip(hipGetLastError(), "absmax/tensor_scale kernels");
}

}  // namespace pq
