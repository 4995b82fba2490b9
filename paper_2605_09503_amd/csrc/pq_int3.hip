// Dense 3-bit storage of INT3 codes (paper Eq. 1-2 with b = 3: codes in -3..3; the paper prints no
// layout, this one is the library's): a row of K codes is a stream of 3 K bits, code k in bits
// 3k..3k+2 as z mod 8, bit b of the stream in bit b mod 8 of byte b div 8, rows unpadded.  With
// K a multiple of 32 the whole tensor is a sequence of pieces of 32 codes: 16 bytes of two's
// complement nibbles on one side, 12 bytes on the other, and neither side needs a row index.
//
// A workgroup of 256 lanes moves 256 pieces.  The 16-byte side is one vector access per lane; the
// 12-byte side goes through LDS so that the global accesses are three contiguous runs of 1 KB per
// workgroup instead of 256 twelve-byte pieces (a lane's three words sit at an odd word stride in
// LDS, which spreads them over the banks).  HBM-bound: 28 bytes per 32 codes.
#include "pq_device.h"
#include "pq_host.h"

namespace pq {
namespace {

constexpr int kPieces = 256;     // pieces (of 32 codes) per workgroup

__global__ __launch_bounds__(kPieces) void int3_pack_kernel(const uint4* __restrict__ nibbles, int64_t pieces,
                                                            uint32_t* __restrict__ dense) {
  __shared__ uint32_t words[3 * kPieces];
  const int tid = threadIdx.x;
  const int64_t p0 = (int64_t)blockIdx.x * kPieces;
  if (p0 + tid < pieces) {
    uint32_t o[3];
    int3_squeeze32(nibbles[p0 + tid], o);
    words[3 * tid] = o[0];
    words[3 * tid + 1] = o[1];
    words[3 * tid + 2] = o[2];
  }
  __syncthreads();
  const int64_t n_words = 3 * (pieces - p0 < kPieces ? pieces - p0 : kPieces);
#pragma unroll
  for (int t = 0; t < 3; ++t)
    if (t * kPieces + tid < n_words) dense[3 * p0 + t * kPieces + tid] = words[t * kPieces + tid];
}

__global__ __launch_bounds__(kPieces) void int3_unpack_kernel(const uint32_t* __restrict__ dense, int64_t pieces,
                                                              uint4* __restrict__ nibbles) {
  __shared__ uint32_t words[3 * kPieces];
  const int tid = threadIdx.x;
  const int64_t p0 = (int64_t)blockIdx.x * kPieces;
  const int64_t n_words = 3 * (pieces - p0 < kPieces ? pieces - p0 : kPieces);
#pragma unroll
  for (int t = 0; t < 3; ++t)
    if (t * kPieces + tid < n_words) words[t * kPieces + tid] = dense[3 * p0 + t * kPieces + tid];
  __syncthreads();
  if (p0 + tid < pieces) nibbles[p0 + tid] = int3_spread32(words[3 * tid], words[3 * tid + 1], words[3 * tid + 2]);
}

}  // namespace

int launch_int3_pack(const uint8_t* codes, int64_t rows, int64_t K, uint8_t* dense, hipStream_t st) {
  const int64_t pieces = rows * (K / 32);
  const int64_t blocks = (pieces + kPieces - 1) / kPieces;
  if (blocks > 0x7FFFFFFF) return fail(PQ_ERR_SHAPE, "tensor too large for one launch");
  hipLaunchKernelGGL(int3_pack_kernel, dim3((unsigned)blocks), dim3(kPieces), 0, st,
                     reinterpret_cast<const uint4*>(codes), pieces, reinterpret_cast<uint32_t*>(dense));
  return check_hip(hipGetLastError(), "int3_pack_kernel");
}

int launch_int3_unpack(const uint8_t* dense, int64_t rows, int64_t K, uint8_t* codes, hipStream_t st) {
  const int64_t pieces = rows * (K / 32);
  const int64_t blocks = (pieces + kPieces - 1) / kPieces;
  if (blocks > 0x7FFFFFFF) return fail(PQ_ERR_SHAPE, "tensor too large for one launch");
  hipLaunchKernelGGL(int3_unpack_kernel, dim3((unsigned)blocks), dim3(kPieces), 0, st,
                     reinterpret_cast<const uint32_t*>(dense), pieces, reinterpret_cast<uint4*>(codes));
  return check_hip(hipGetLastError(), "int3_unpack_kernel");
}

}  // namespace pq
