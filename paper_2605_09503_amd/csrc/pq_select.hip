// Permutation selection (paper Sec. 3.3): joint second-moment score (Eq. 9), descending sort
// (Prop. 1), calibration error of every candidate order, alpha search and acceptance rule.
//
// Kernels
//   key_kernel        key[j][i] = alpha_j ln Sa[i] + (1 - alpha_j) ln Sw[i], fp64, all j in one
//                     launch; a term whose weight is zero is skipped.
//   rank_count_kernel / rank_scatter_kernel
//                     stable descending sort by counting: rank(i) = #{j : key_j > key_i or
//                     (key_j == key_i and j < i)}; perm[rank(i)] = i.  O(K^2) compares, K <= 65536,
//                     split over (channel block, key chunk, candidate) workgroups, integer
//                     counts added atomically, fully deterministic.
//   same_order_kernel  which candidate orders repeat an earlier one (or the original order): those are
//                     evaluated once.
//   quant_error_kernel a workgroup stages a few rows in LDS at a time; for every candidate order
//                     their channels are gathered from LDS (one read serves all resident rows),
//                     quantized with the same lane-cooperative quantizer as the runtime kernels,
//                     and the squared error of the dequantized values accumulated in fp64 (NVFP4:
//                     from exact fp32 group sums).  HBM traffic is one read of the tensor for all
//                     candidates.
//   select_tail_kernel fixed-order sums of the per-wave partial errors, of the moments and of the
//                     moved-channel counts (deterministic), one launch.
// The final argmin / acceptance decision is a handful of scalar operations and runs on the host.
#include <string.h>

#include <atomic>

#include "pq_device.h"
#include "pq_host.h"

namespace pq {

constexpr int kMaxCand = PQ_MAX_ALPHAS + 1;   // identity + candidates
constexpr int kMaxDevicesSeen = 64;

struct AlphaList {
  double a[PQ_MAX_ALPHAS];
};

// key[j][i] for every alpha_j of the grid (blockIdx.y = j)
__global__ __launch_bounds__(256) void key_kernel(const double* __restrict__ sa,
                                                  const double* __restrict__ sw, int64_t K,
                                                  AlphaList alphas, double* __restrict__ key,
                                                  int32_t* __restrict__ rank, uint32_t* __restrict__ differs) {
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (differs && i == 0) differs[blockIdx.y] = 0u;    // same_order_kernel ORs into it
  if (i >= K) return;
  rank[(int64_t)blockIdx.y * K + i] = 0;          // the counting pass adds to it
  const double alpha = alphas.a[blockIdx.y];
  double k = 0.0;
  if (alpha != 0.0) k += alpha * log(sa[i]);
  if (alpha != 1.0) k += (1.0 - alpha) * log(sw[i]);
  key[(int64_t)blockIdx.y * K + i] = k;
}

constexpr int kRankChunk = 128;    // keys compared per workgroup of the counting pass (divides 256)

// Counting pass of the stable descending sort: workgroup (x, y, z) compares its 256 channels i
// with the kRankChunk keys j of chunk y of candidate z and adds how many of them sort before i to
// rank[z][i] (integer atomics: the sum does not depend on the order of the workgroups).
// A chunk lies inside one channel block, so every key of a chunk in an earlier block has j < i (it
// sorts before i when key_j >= key_i), every key in a later block has j > i (key_j > key_i), and
// only the chunks of the workgroup's own block need the index comparison.  A wave's time is the
// chain of its scalar key loads, hence short chunks and deep unrolling.
__global__ __launch_bounds__(256) void rank_count_kernel(const double* __restrict__ keys, int K,
                                                         int32_t* __restrict__ rank) {
  const double* key = keys + (int64_t)blockIdx.z * K;
  const int i = blockIdx.x * 256 + threadIdx.x;
  const int j0 = blockIdx.y * kRankChunk;
  const int n = min(kRankChunk, K - j0);
  if (i >= K) return;
  const double ki = key[i];
  // the keys of the chunk are the same for every lane: they come through scalar loads and sit in
  // scalar registers, the compare takes them as an operand
  const double* tile = key + j0;
  int before = 0;
  const int key_block = blockIdx.y / (256 / kRankChunk);      // the channel block the chunk lies in
  if (key_block < (int)blockIdx.x) {
#pragma unroll 32
    for (int t = 0; t < n; ++t) before += tile[t] >= ki ? 1 : 0;
  } else if (key_block > (int)blockIdx.x) {
#pragma unroll 32
    for (int t = 0; t < n; ++t) before += tile[t] > ki ? 1 : 0;
  } else {
#pragma unroll 32
    for (int t = 0; t < n; ++t) {
      // without short-circuit evaluation: no branches, the loads of a whole unrolled trip go out together
      const double kj = tile[t];
      const int gt = kj > ki ? 1 : 0, eq = kj == ki ? 1 : 0, earlier = j0 + t < i ? 1 : 0;
      before += gt | (eq & earlier);
    }
  }
  atomicAdd(&rank[(int64_t)blockIdx.z * K + i], before);
}

// perm[z][rank(i)] = i; with offs, also the LDS byte offset of channel i's slot in the error evaluation
// (slot i + i / 8, slot_bytes each) at the same position
__global__ __launch_bounds__(256) void rank_scatter_kernel(const int32_t* __restrict__ rank, int K,
                                                           int32_t* __restrict__ perms,
                                                           int32_t* __restrict__ offs, int slot_bytes) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= K) return;
  const int64_t at = (int64_t)blockIdx.y * K + rank[(int64_t)blockIdx.y * K + i];
  perms[at] = i;
  if (offs) offs[at] = (i + (i >> 3)) * slot_bytes;
}

// Which candidate orders repeat an earlier one.  Candidate 0 is the original order, candidate 1 + j the order
// of alpha_j.  differs[j] collects a bit per earlier candidate c <= j that differs from order j somewhere
// (integer OR: no order dependence); workgroup (x, j) looks at 256 positions.  differs[] is zeroed by
// key_kernel, which runs before on the same stream.
__global__ __launch_bounds__(256) void same_order_kernel(const int32_t* __restrict__ perms, int K,
                                                         uint32_t* __restrict__ differs) {
  __shared__ unsigned block_bits;
  const int j = blockIdx.y;
  if (threadIdx.x == 0) block_bits = 0u;
  __syncthreads();
  const int i = blockIdx.x * 256 + threadIdx.x;
  unsigned d = 0u;
  if (i < K) {
    const int32_t v = perms[(int64_t)j * K + i];
    d |= v != i ? 1u : 0u;                           // bit 0: the original order
    for (int e = 0; e < j; ++e) d |= (perms[(int64_t)e * K + i] != v ? 1u : 0u) << (1 + e);
  }
  if (d) atomicOr(&block_bits, d);
  __syncthreads();
  if (threadIdx.x == 0 && block_bits) atomicOr(&differs[j], block_bits);
}
// the first candidate with the same order as candidate c (c itself if none before it)
__device__ __forceinline__ int first_same_order(const uint32_t* __restrict__ differs, int c) {
  if (c == 0) return 0;
  const uint32_t bits = differs[c - 1];
  int first = c;
  for (int e = c - 1; e >= 0; --e)
    if (!((bits >> e) & 1u)) first = e;
  return first;
}

__global__ __launch_bounds__(256) void iota_kernel(int32_t* p, int K) {
  int i = blockIdx.x * 256 + threadIdx.x;
  if (i < K) p[i] = i;
}

// NVFP4 tensor scale of a launch: a host value, or a device float read by the kernel (dev != nullptr)
struct ScaleArg {
  float value;
  const float* dev;
};

// up to kMaxMomentBatches tensors of equal shape handled by one launch
struct TensorList {
  const uint16_t* p[kMaxMomentBatches];
};

// fewest rows a workgroup of the error evaluation covers (bounds the number of partial sums)
constexpr int kQeMinRowsPerBlock = 8;
constexpr int kQeMaxWaves = 16;           // waves of such a workgroup
constexpr int64_t kQeParts(int64_t rows) { return (rows / kQeMinRowsPerBlock + 1) * kQeMaxWaves; }

template <int R>
struct FloatVec;
template <>
struct FloatVec<1> { typedef float type; };
template <>
struct FloatVec<2> { typedef float type __attribute__((ext_vector_type(2))); };
template <>
struct FloatVec<4> { typedef float type __attribute__((ext_vector_type(4))); };

// channels of one work item of a lane: a whole NVFP4 group (its scale then needs no lane exchange and is
// worked out once), eight for the integer formats, whose groups span lanes
template <int FMT>
struct QeChunk { static constexpr int value = FMT == kNvfp4 ? 16 : 8; };

// byte offset of channel e's slot in the LDS image of R resident rows: slot e + e / 8 (the spare slot per
// eight channels spreads the staging writes over the banks), R floats per slot
__host__ __device__ constexpr int qe_slot_bytes(int r) { return r * 4; }

// Workgroup (x, y) evaluates rows [x * rows_per_block, (x + 1) * rows_per_block) of tensor y of
// the list (equal shapes) for every candidate order.  R rows at a time are staged in LDS as
// fp32, channel-major with the R rows of a channel adjacent; the rows after them are already on
// their way from memory into registers while the resident ones are evaluated.  A candidate order
// comes as the byte offsets of its channels' slots (offs[cand][position]), so a lane reads the
// offsets of its chunk and gathers the R rows of each channel with one LDS read, no address
// arithmetic; the quantizer is the lane-cooperative one of the runtime kernels.  Integer formats: the
// error v - s t of an element is exact in fp32 and its square is accumulated in fp64.  NVFP4: the squared
// error of a group is sum v^2 - 2 d A + d^2 B (A = sum v q, B = sum q^2, d the group's scale): A and B are
// exact fp32 sums, the rest is fp64, and sum v^2 -- the same for every order -- is taken once when the rows
// are staged; the difference loses the bits by which sum v^2 exceeds the error (two decimal digits of
// fp64's sixteen for data that fill the format; an absolute 1e-15 of sum v^2 at worst).  Every wave owns a fixed run of work
// items (candidate, block of 64 chunks), candidate-major, sums a candidate's errors per lane and
// reduces them over the wave once per candidate and set of resident rows.  Lane c of every wave
// ends up with the wave's total for candidate c: part[y][c][x * waves + wave] (candidate-major, so
// that the sums over the workgroups read contiguous memory).
template <int FMT, int G, int R>
__global__ __launch_bounds__(64 * kQeMaxWaves) void quant_error_kernel(TensorList xs, int rows, int K,
                                                          const int32_t* __restrict__ offs,
                                                          int n_cand, int identity_first, ScaleArg t_arg,
                                                          int rows_per_block, const uint32_t* __restrict__ differs,
                                                          double* __restrict__ part) {
  typedef typename FloatVec<R>::type vec_t;
  constexpr int C = QeChunk<FMT>::value;
  constexpr int PF = 4 / R;                // staging chunks (8 channels x R rows) a thread fetches ahead
  constexpr bool kOffsetsAhead = R < 4;    // the next item's offsets are loaded during the current item
  extern __shared__ __attribute__((aligned(16))) float slots[];     // (K + K / 8) * R floats
  const int tid = threadIdx.x, nthr = blockDim.x;
  const int lane = tid & 63, n_waves = nthr >> 6;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint16_t* x = xs.p[blockIdx.y];
  const int row0 = blockIdx.x * rows_per_block;
  const int row_end = min(rows, row0 + rows_per_block);
  const int chunks8 = K / 8;               // staging granularity: one 16-byte load
  const int chunks = K / C;
  const int wave_chunks = (chunks + 63) >> 6;
  // Candidates that repeat an earlier order are left out.  Lane c works out whether candidate c does (one
  // load); the answer is used after the first rows have been requested (see below).
  int same_as_lane = lane;
  if (differs && lane < n_cand) same_as_lane = first_same_order(differs, lane);
  const float T = t_arg.dev ? *t_arg.dev : t_arg.value;           // uniform
  const float encT = (FMT == kNvfp4) ? nv4_enc_scale(T) : 0.0f;
  // The offsets are used as LDS addresses as they are: the staged rows are the kernel's only LDS object and
  // start at address 0 (adding a base would cost one instruction per gathered channel).  Should a
  // toolchain ever place them elsewhere, every partial sum of the launch is made a NaN.
  typedef const __attribute__((address_space(3))) vec_t* lds_vec_ptr;
  const bool lds_at_zero = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) float*)slots == 0u;

  // rows past the end count as zero rows: error 0
  auto fetch_row = [&](int r, int c) {
    uint4 p = make_uint4(0u, 0u, 0u, 0u);
    if (r < row_end) p = *reinterpret_cast<const uint4*>(x + (int64_t)r * K + (int64_t)c * 8);
    return p;
  };
  double v_sq = 0.0;                       // NVFP4: this thread's share of the sum of squares of the rows
  auto put = [&](int c, const uint4 (&p)[R]) {
    float v[R][8];
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
      v[rr][0] = bf16_lo(p[rr].x); v[rr][1] = bf16_hi(p[rr].x); v[rr][2] = bf16_lo(p[rr].y); v[rr][3] = bf16_hi(p[rr].y);
      v[rr][4] = bf16_lo(p[rr].z); v[rr][5] = bf16_hi(p[rr].z); v[rr][6] = bf16_lo(p[rr].w); v[rr][7] = bf16_hi(p[rr].w);
      if constexpr (FMT == kNvfp4) {
#pragma unroll
        for (int j = 0; j < 8; ++j) v_sq = fma((double)v[rr][j], (double)v[rr][j], v_sq);
      }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      vec_t o;
      if constexpr (R == 1) o = v[0][j];
      else {
#pragma unroll
        for (int rr = 0; rr < R; ++rr) o[rr] = v[rr][j];
      }
      *reinterpret_cast<vec_t*>(slots + (size_t)(9 * c + j) * R) = o;
    }
  };
  uint4 ahead[PF][R];
  auto fetch_ahead = [&](int rg) {
#pragma unroll
    for (int f = 0; f < PF; ++f) {
      const int c = tid + f * nthr;
#pragma unroll
      for (int rr = 0; rr < R; ++rr) ahead[f][rr] = c < chunks8 ? fetch_row(rg + rr, c) : make_uint4(0u, 0u, 0u, 0u);
    }
  };

  // the slot offsets of the C channels of work item (cand, blk) of this lane
  auto load_offsets = [&](int cand, int blk, int (&o)[C]) {
    const int c_lane = blk * 64 + lane;
    const int c = c_lane < chunks ? c_lane : 0;
    if (!(identity_first && cand == 0)) {
      const int4* po = reinterpret_cast<const int4*>(offs + (int64_t)(cand - identity_first) * K + c * C);
#pragma unroll
      for (int j = 0; j < C; j += 4) {
        const int4 q = po[j / 4];
        o[j] = q.x; o[j + 1] = q.y; o[j + 2] = q.z; o[j + 3] = q.w;
      }
    } else {
      const int base = c * (C / 8 * 9) * qe_slot_bytes(R);
#pragma unroll
      for (int j = 0; j < C; ++j) o[j] = base + ((j / 8) * 9 + (j & 7)) * qe_slot_bytes(R);
    }
  };

  double acc = 0.0;
  fetch_ahead(row0);
  // the orders to evaluate, four bits each (at most 16 candidates); the work items run over that list
  unsigned long long order_list = 0;
  int n_orders = 0;
  {
    const unsigned long long keep = __ballot(lane < n_cand && same_as_lane == lane);     // uniform
    for (int c = 0; c < n_cand; ++c) {
      if (!((keep >> c) & 1ull)) continue;
      order_list |= (unsigned long long)c << (4 * n_orders);
      ++n_orders;
    }
  }
  const int n_items = n_orders * wave_chunks;
  const int per_wave = (n_items + n_waves - 1) / n_waves;
  const int it0 = wave * per_wave, it1 = min(n_items, it0 + per_wave);
  const int ord0 = it0 / wave_chunks, blk0 = it0 - ord0 * wave_chunks;       // uniform over the wave
  auto cand_of = [&](int ord) { return (int)((order_list >> (4 * ord)) & 15u); };
  for (int rg = row0; rg < row_end; rg += R) {
    __syncthreads();                       // the previous rows have been read by every wave
#pragma unroll
    for (int f = 0; f < PF; ++f) {
      const int c = tid + f * nthr;
      if (c < chunks8) put(c, ahead[f]);
    }
    for (int c = tid + PF * nthr; c < chunks8; c += nthr) {     // wider rows than the registers hold ahead
      uint4 p[R];
#pragma unroll
      for (int rr = 0; rr < R; ++rr) p[rr] = fetch_row(rg + rr, c);
      put(c, p);
    }
    __syncthreads();
    // Loads return in issue order, so the order below matters: the offsets of the first item go out
    // before the rows fetched ahead (they are needed at once), those of every later item while the item
    // before it is evaluated (at its start when four rows are resident: the registers do not hold both
    // then, and a second workgroup of the compute unit covers the wait), by which time the rows have
    // long arrived.
    int ord = ord0, blk = blk0;
    int cand = cand_of(ord);
    int o_ahead[kOffsetsAhead ? C : 1];
    if constexpr (kOffsetsAhead) {
      if (it0 < it1) load_offsets(cand, blk, o_ahead);
    }
    if (rg + R < row_end) fetch_ahead(rg + R);     // in flight during the evaluation below
    double run = 0.0;                      // this lane's error of the current candidate
    for (int it = it0; it < it1; ++it) {
      // every lane runs the group reduction; a lane past the last chunk (its whole group is, K being a
      // multiple of the group size) works on chunk 0 and its result is dropped
      const bool live = blk * 64 + lane < chunks;
      int o[C];
      if constexpr (kOffsetsAhead) {
#pragma unroll
        for (int j = 0; j < C; ++j) o[j] = o_ahead[j];
      } else {
        load_offsets(cand, blk, o);
      }
      float v[R][C];
#pragma unroll
      for (int j = 0; j < C; ++j) {
        const vec_t g = *(lds_vec_ptr)(uintptr_t)(uint32_t)o[j];
        if constexpr (R == 1) v[0][j] = g;
        else {
#pragma unroll
          for (int rr = 0; rr < R; ++rr) v[rr][j] = g[rr];
        }
      }
      const bool cand_done = blk + 1 == wave_chunks || it + 1 == it1;     // uniform
      if constexpr (kOffsetsAhead) {
        if (it + 1 < it1) load_offsets(cand_done ? cand_of(ord + 1) : cand, cand_done ? 0 : blk + 1, o_ahead);
      }
      double errs[R];                               // one chain per resident row
#pragma unroll
      for (int rr = 0; rr < R; ++rr) errs[rr] = 0.0;
      constexpr bool kRows4 = FMT != kNvfp4 && R == 4 && G >= 32;    // scales shared out over a quad
      float amax[R];
#pragma unroll
      for (int rr = 0; rr < R; ++rr) {
        float a = 0.0f;
#pragma unroll
        for (int j = 0; j < C; ++j) a = fmaxf(a, fabsf(v[rr][j]));
        amax[rr] = kRows4 ? a : group_max<G / C>(a);
      }
      if constexpr (FMT == kNvfp4) {
        // A group's error is sum (v - q d)^2 = sum v^2 - 2 d A + d^2 B with A = sum v q and B = sum q^2
        // (q = +-E2M1 value, d = block scale x tensor scale).  sum v^2 does not depend on the order: it is
        // added once per row (v_sq below); the lane accumulates A and B in fp32, which is exact: an element
        // with q != 0 has |v| > d / 4, so every product v q is a multiple of U > d 2^-11 (bf16 v, q a
        // multiple of 1/2), and |A| <= 16 * 6 * amax < 2^24 U as long as amax <= 48 d -- true unless the block
        // scale saturated far beyond its largest value (a tensor scale much too small for the data: the
        // wave then takes the element-wise fp64 sum instead).  B <= 16 * 36 in steps of 1/4.
        Nv4Scale s[R];
        nv4_scales<R>(amax, T, encT, s);
        bool far_saturated = false;
#pragma unroll
        for (int rr = 0; rr < R; ++rr) far_saturated = far_saturated || amax[rr] * encT > 6.0f * 448.0f * 7.0f;
        const bool exact_sums = !__any(far_saturated);          // uniform
        // eight elements on the conversion unit (a byte of `codes` per pair), decoded again
        auto quantize8 = [&](const float* x, float inv, float (&q)[8]) {
          uint32_t codes = 0u;
          codes = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(codes, x[0] * inv, x[1] * inv, 1.0f, 0);
          codes = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(codes, x[2] * inv, x[3] * inv, 1.0f, 1);
          codes = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(codes, x[4] * inv, x[5] * inv, 1.0f, 2);
          codes = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(codes, x[6] * inv, x[7] * inv, 1.0f, 3);
          const auto q0 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes, 1.0f, 0);
          const auto q1 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes, 1.0f, 1);
          const auto q2 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes, 1.0f, 2);
          const auto q3 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes, 1.0f, 3);
          q[0] = q0[0]; q[1] = q0[1]; q[2] = q1[0]; q[3] = q1[1];
          q[4] = q2[0]; q[5] = q2[1]; q[6] = q3[0]; q[7] = q3[1];
        };
        if (__builtin_expect(exact_sums, 1)) {
#pragma unroll
          for (int rr = 0; rr < R; ++rr) {
            float A = 0.0f, B = 0.0f;
#pragma unroll
            for (int j = 0; j < C; j += 8) {
              float q[8];
              quantize8(&v[rr][j], s[rr].inv, q);
#pragma unroll
              for (int u = 0; u < 8; ++u) {
                A = __builtin_fmaf(v[rr][j + u], q[u], A);
                B = __builtin_fmaf(q[u], q[u], B);
              }
            }
            // - 2 d A + d^2 B = d (d B - 2 A): d (4 + 24 bits) is exact, so are d B (+ 10 bits) and the
            // difference; one rounding in the last product
            const double d = (double)s[rr].value * (double)T;
            errs[rr] = d * fma(d, (double)B, -2.0 * (double)A);
          }
        } else {
#pragma unroll
          for (int rr = 0; rr < R; ++rr) {
            const double d = (double)s[rr].value * (double)T;
#pragma unroll
            for (int j = 0; j < C; j += 8) {
              float q[8];
              quantize8(&v[rr][j], s[rr].inv, q);
#pragma unroll
              for (int u = 0; u < 8; ++u) {
                const double x = (double)v[rr][j + u];
                const double e = fma(-(double)q[u], d, x);      // product exact: 2 + 28 bits
                errs[rr] = fma(e, e, errs[rr]);
                errs[rr] = fma(-x, x, errs[rr]);                // the part counted by v_sq
              }
            }
          }
        }
      } else {
        IntScale s[R];
        if constexpr (kRows4) int_scales_rows4<FMT, G / C>(amax, lane, s);
        else int_scales<FMT, R>(amax, s);
#pragma unroll
        for (int rr = 0; rr < R; ++rr) {
#pragma unroll
          for (int j = 0; j < C; ++j) {
            // The clip of the quantizer cannot act here: amax is the true maximum of the group, so
            // |x * inv| <= Q (1 + 3 * 2^-24) < Q + 1/2 and the rounding already lands on +-Q
            // (inv = 0 gives 0).  v_rndne_f32 rounds to the nearest integer, ties to even.
            const float t = __builtin_rintf(v[rr][j] * s[rr].inv);
            // v - s t is exact in binary32: for t != 0 both terms are multiples of the last place
            // of s and the difference is at most about s / 2, so it needs no more than 24 bits;
            // the fused multiply-add returns it unrounded
            const float e32 = __builtin_fmaf(-s[rr].s, t, v[rr][j]);
            const double e = (double)e32;
            errs[rr] = fma(e, e, errs[rr]);
          }
        }
      }
      double err = errs[0];
#pragma unroll
      for (int rr = 1; rr < R; ++rr) err += errs[rr];
      run += live ? err : 0.0;
      ++blk;
      if (cand_done) {                               // the candidate's last item of this wave
        const double total = wave_sum(run);          // fixed xor-tree order
        if (lane == cand) acc += total;
        run = 0.0;
        blk = 0;
        ++ord;
        cand = cand_of(ord);
      }
    }
  }
  if constexpr (FMT == kNvfp4) {
    // every candidate's error contains the rows' sum of squares: the wave's share goes to each
    const double share = wave_sum(v_sq);
    if (lane < n_cand) acc += share;
  }
  if (!lds_at_zero) acc = __builtin_nan("");
  if (lane < n_cand)
    part[((int64_t)blockIdx.y * n_cand + lane) * ((int64_t)gridDim.x * n_waves) + (int64_t)blockIdx.x * n_waves + wave] = acc;
}

// offs[i] = byte offset of channel perm[i]'s slot for R resident rows (the error evaluation of one given order)
__global__ __launch_bounds__(256) void perm_to_offsets_kernel(const int32_t* __restrict__ perm, int K, int slot_bytes,
                                                              int32_t* __restrict__ offs) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= K) return;
  const int e = perm[i];
  offs[i] = (e + (e >> 3)) * slot_bytes;
}

// out[seg][c] = sum over the rows of segment seg of row_err[r][c]; one workgroup per
// (candidate, segment), fixed order.  Segments are consecutive runs of seg_rows rows.  not_below_zero: a
// sum that comes out negative (NVFP4's error of data the format holds exactly is zero up to the rounding
// of a difference) is returned as zero.
__global__ __launch_bounds__(256) void reduce_rows_kernel(const double* __restrict__ row_err,
                                                          int64_t seg_rows, int n_cand, int out_stride,
                                                          int not_below_zero, double* __restrict__ out) {
  __shared__ double red[256];
  const int c = blockIdx.x;
  const double* base = row_err + (int64_t)blockIdx.y * seg_rows * n_cand;
  double s = 0.0;
  for (int64_t r = threadIdx.x; r < seg_rows; r += 256) s += base[r * n_cand + c];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int st = 128; st > 0; st >>= 1) {
    if (threadIdx.x < st) red[threadIdx.x] += red[threadIdx.x + st];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[(int64_t)blockIdx.y * out_stride + c] = not_below_zero && red[0] < 0.0 ? 0.0 : red[0];
}

// Everything the host needs for the decision, in one launch.  Workgroup b of the grid computes
// one fixed-order sum (per-thread strided partial sums, then a binary tree) into out[]:
//   b <  n_cand * n_batches         error of candidate b % n_cand on calibration batch b / n_cand
//                                   -> out[batch * kMaxCand + cand]
//   next n_cand                     error of the candidate on the weights -> out[n_batches * kMaxCand + cand]
//   next 2                          sum of act_sumsq, sum of w_sumsq      -> out[(n_batches + 1) * kMaxCand + 0 / 1]
//   next n_alpha                    number of channels candidate j moves  -> out[... + 2 + j] (as a double)
struct TailArgs {
  const double* x_part;     // [n_batches][n_cand][x_parts]
  const double* w_part;     // [n_cand][w_parts]
  const double* act_sumsq;
  const double* w_sumsq;
  const int32_t* cands;     // [n_alpha][K]
  const uint32_t* differs;  // per alpha: which earlier candidates differ; a repeated order takes the first one's sums
  int64_t x_parts, w_parts, K;
  int n_cand, n_batches, n_alpha;
};

// s + p[i0] + p[i0 + stride] + ... (i < n), in that order, with eight loads in flight at a time (a plain
// loop waits out one memory latency per element)
__device__ __forceinline__ double strided_sum(const double* __restrict__ p, int64_t i0, int64_t n, int64_t stride) {
  double s = 0.0;
  int64_t i = i0;
  for (; i + 7 * stride < n; i += 8 * stride) {
    double v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = p[i + u * stride];
#pragma unroll
    for (int u = 0; u < 8; ++u) s += v[u];
  }
  for (; i < n; i += stride) s += p[i];
  return s;
}

__global__ __launch_bounds__(256) void select_tail_kernel(TailArgs a, double* __restrict__ out) {
  __shared__ double red[256];
  const int n_x = a.n_cand * a.n_batches;
  int b = blockIdx.x;
  double s = 0.0;
  int64_t dst;
  if (b < n_x + a.n_cand) {
    const bool is_w = b >= n_x;
    const int seg = is_w ? 0 : b / a.n_cand, c = is_w ? b - n_x : b % a.n_cand;
    const int64_t n = is_w ? a.w_parts : a.x_parts;
    const double* base = is_w ? a.w_part : a.x_part + (int64_t)seg * n * a.n_cand;
    s = strided_sum(base + (int64_t)first_same_order(a.differs, c) * n, threadIdx.x, n, 256);
    dst = (int64_t)(is_w ? a.n_batches : seg) * kMaxCand + c;
  } else if (b < n_x + a.n_cand + 2) {
    const int which = b - n_x - a.n_cand;
    const double* p = which ? a.w_sumsq : a.act_sumsq;
    s = strided_sum(p, threadIdx.x, a.K, 256);
    dst = (int64_t)(a.n_batches + 1) * kMaxCand + which;
  } else {
    const int j = b - n_x - a.n_cand - 2;
    const int32_t* p = a.cands + (int64_t)j * a.K;
    int n = 0;
    int64_t i = threadIdx.x;
    for (; i + 7 * 256 < a.K; i += 8 * 256) {
      int32_t v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = p[i + u * 256];
#pragma unroll
      for (int u = 0; u < 8; ++u) n += (v[u] != (int32_t)(i + u * 256));
    }
    for (; i < a.K; i += 256) n += (p[i] != (int32_t)i);
    s = (double)n;                                    // small integers: every sum below is exact
    dst = (int64_t)(a.n_batches + 1) * kMaxCand + 2 + j;
  }
  red[threadIdx.x] = s;
  __syncthreads();
  for (int st = 128; st > 0; st >>= 1) {
    if (threadIdx.x < st) red[threadIdx.x] += red[threadIdx.x + st];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[dst] = red[0];
}

// Launch shape of the error evaluation of n_cand orders for `rows` rows per tensor of width K.
struct QeShape {
  int r;                 // rows resident in LDS together (1, 2 or 4)
  int threads;
  int rows_per_block;
  int blocks;            // per tensor
  size_t shmem;
  int parts() const { return blocks * (threads / 64); }    // partial sums per tensor and candidate
};

static QeShape qe_shape(pq_format fmt, int64_t rows, int64_t K, int n_tensors, int n_cand) {
  QeShape q;
  const bool nv = fmt == PQ_FMT_NVFP4;
  const int chunk = nv ? QeChunk<kNvfp4>::value : QeChunk<kInt4>::value;
  const size_t slot_floats = (size_t)(K + K / 8);
  q.r = slot_floats * 16 <= 64 * 1024 ? 4 : slot_floats * 8 <= 128 * 1024 ? 2 : 1;
  q.shmem = slot_floats * q.r * sizeof(float);
  // waves: the work items of a set of resident rows (candidate x block of 64 chunks) are shared out
  // evenly; take the fewest waves that need the fewest turns.  Two workgroups share a compute unit when
  // their rows fit its LDS twice (one stages while the other computes): half of the waves the unit's
  // registers hold each then (the NVFP4 instances need up to 128 registers a lane: sixteen waves a unit;
  // the integer ones up to 96: twenty), sixteen otherwise.
  const int items = n_cand * (int)((K / chunk + 63) / 64);
  const int max_waves = 2 * q.shmem <= 160 * 1024 ? (nv ? 8 : 10) : kQeMaxWaves;
  const int turns = (items + max_waves - 1) / max_waves;
  q.threads = 64 * ((items + turns - 1) / turns);
  // Rows per workgroup: the workgroups run in rounds of as many as the chip holds at once (256 compute
  // units, one or two each), every round lasts about as long as a workgroup's rows plus a fixed start-up
  // (taken as half a row); among kQeMinRowsPerBlock .. 64 rows take the smallest size whose total is
  // within 2 % of the shortest (smaller workgroups even out better when their times differ).
  const int64_t resident = (2 * q.shmem <= 160 * 1024 ? 2 : 1) * 256;
  const int64_t lo = (kQeMinRowsPerBlock + q.r - 1) / q.r * q.r;
  auto cost_of = [&](int64_t rpb) {
    const int64_t wgs = (rows + rpb - 1) / rpb * n_tensors;
    return (double)((wgs + resident - 1) / resident) * ((double)rpb + 0.5);
  };
  double best_cost = cost_of(lo);
  for (int64_t rpb = lo; rpb <= 64; rpb += q.r) best_cost = cost_of(rpb) < best_cost ? cost_of(rpb) : best_cost;
  int64_t best_rpb = lo;
  while (cost_of(best_rpb) > 1.02 * best_cost) best_rpb += q.r;
  q.rows_per_block = (int)best_rpb;
  q.blocks = (int)((rows + best_rpb - 1) / best_rpb);
  return q;
}

template <int FMT, int G, int R>
static int launch_qe_r(const TensorList& xs, int n_tensors, int64_t rows, int K, const QeShape& q,
                       const int32_t* offs, int n_cand, int identity_first, ScaleArg T, const uint32_t* same_as,
                       double* part, hipStream_t st) {
  auto kern = quant_error_kernel<FMT, G, R>;
  // the attribute is per kernel instance and device; it is raised once per instance to the most any
  // launch may ask for, not on every call
  static std::atomic<bool> raised[kMaxDevicesSeen];
  int dev = 0;
  (void)hipGetDevice(&dev);
  if (q.shmem > 48 * 1024 && (dev < 0 || dev >= kMaxDevicesSeen || !raised[dev].load(std::memory_order_acquire))) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
    if (e != hipSuccess) return check_hip(e, "hipFuncSetAttribute(quant_error_kernel)");
    if (dev >= 0 && dev < kMaxDevicesSeen) raised[dev].store(true, std::memory_order_release);
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)q.blocks, (unsigned)n_tensors), dim3(q.threads), q.shmem, st, xs,
                     (int)rows, K, offs, n_cand, identity_first, T, q.rows_per_block, same_as, part);
  return check_hip(hipGetLastError(), "quant_error_kernel");
}

template <int FMT, int G>
static int launch_qe(const TensorList& xs, int n_tensors, int64_t rows, int K, const QeShape& q,
                     const int32_t* offs, int n_cand, int identity_first, ScaleArg T, const uint32_t* same_as,
                     double* part, hipStream_t st) {
  switch (q.r) {
    case 4: return launch_qe_r<FMT, G, 4>(xs, n_tensors, rows, K, q, offs, n_cand, identity_first, T, same_as, part, st);
    case 2: return launch_qe_r<FMT, G, 2>(xs, n_tensors, rows, K, q, offs, n_cand, identity_first, T, same_as, part, st);
    default: return launch_qe_r<FMT, G, 1>(xs, n_tensors, rows, K, q, offs, n_cand, identity_first, T, same_as, part, st);
  }
}

// part: [n_tensors][n_cand][q.parts()]; offs: the candidate orders as slot offsets for q.r resident rows
static int launch_quant_error(pq_format fmt, int group, const TensorList& x, int n_tensors, int64_t rows,
                              int K, const QeShape& q, const int32_t* offs, int n_cand,
                              int identity_first, ScaleArg T, const uint32_t* same_as, double* part,
                              hipStream_t st) {
  if (rows > 0x7FFFFFFF) return fail(PQ_ERR_SHAPE, "too many rows");
  if (q.shmem > 150 * 1024) return fail(PQ_ERR_SHAPE, "K=%d too large for the LDS-resident row", K);   // the entry points refuse this earlier
  if (fmt == PQ_FMT_NVFP4)
    return launch_qe<kNvfp4, 16>(x, n_tensors, rows, K, q, offs, n_cand, identity_first, T, same_as, part, st);
#define PQ_INT_CASE(F, FE)                                                                                  \
  if (fmt == F) {                                                                                           \
    switch (group) {                                                                                        \
      case 32: return launch_qe<FE, 32>(x, n_tensors, rows, K, q, offs, n_cand, identity_first, T, same_as, part, st);   \
      case 64: return launch_qe<FE, 64>(x, n_tensors, rows, K, q, offs, n_cand, identity_first, T, same_as, part, st);   \
      case 128: return launch_qe<FE, 128>(x, n_tensors, rows, K, q, offs, n_cand, identity_first, T, same_as, part, st); \
      case 256: return launch_qe<FE, 256>(x, n_tensors, rows, K, q, offs, n_cand, identity_first, T, same_as, part, st); \
    }                                                                                                       \
  }
  PQ_INT_CASE(PQ_FMT_INT4, kInt4)
  PQ_INT_CASE(PQ_FMT_INT3, kInt3)
#undef PQ_INT_CASE
  return fail(PQ_ERR_FORMAT, "unsupported (format, group) = (%d, %d)", (int)fmt, group);
}

// ------------------------------------------------------------------------- workspace layout
struct SelectWs {
  double* keys;      // [PQ_MAX_ALPHAS][K]
  int32_t* cands;    // [PQ_MAX_ALPHAS][K]
  int32_t* rank;     // [PQ_MAX_ALPHAS][K] position of every channel in the sorted order
  int32_t* offs;     // [PQ_MAX_ALPHAS][K] the candidates as LDS slot offsets of the error evaluation
  uint32_t* same_as; // [PQ_MAX_ALPHAS] per alpha: a bit per earlier candidate whose order differs (same_order_kernel)
  double* row_err;   // partial error sums: [n_batches][n_cand][parts(M)], then [n_cand][parts(N)]
  double* sums;      // [(n_batches + 1) * kMaxCand + 2 + PQ_MAX_ALPHAS]: per-batch errors, weight
                     // errors, |X|^2, |W|^2, moved-channel counts
};

static int rank_chunks(int64_t K) { return (int)((K + kRankChunk - 1) / kRankChunk); }

static size_t carve_select(void* base, int64_t M, int64_t N, int64_t K, int n_batches, SelectWs* w) {
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off = align_up(off + bytes, 256);
    return o;
  };
  size_t o_keys = take((size_t)PQ_MAX_ALPHAS * K * 8);
  size_t o_cands = take((size_t)PQ_MAX_ALPHAS * K * 4);
  size_t o_rank = take((size_t)PQ_MAX_ALPHAS * K * 4);
  size_t o_offs = take((size_t)PQ_MAX_ALPHAS * K * 4);
  size_t o_same = take((size_t)kMaxCand * 4);
  // a workgroup covers at least kQeMinRowsPerBlock rows with at most kQeMaxWaves waves: no more
  // partial sums than kQeParts(rows) per tensor
  size_t o_rowerr = take((size_t)((int64_t)n_batches * kQeParts(M) + kQeParts(N)) * kMaxCand * 8);
  size_t o_sums = take(((size_t)(n_batches + 1) * kMaxCand + 2 + PQ_MAX_ALPHAS) * 8);
  if (w) {
    char* b = (char*)base;
    w->keys = (double*)(b + o_keys);
    w->cands = (int32_t*)(b + o_cands);
    w->rank = (int32_t*)(b + o_rank);
    w->offs = (int32_t*)(b + o_offs);
    w->same_as = (uint32_t*)(b + o_same);
    w->row_err = (double*)(b + o_rowerr);
    w->sums = (double*)(b + o_sums);
  }
  return off;
}

size_t select_workspace_bytes(int64_t M, int64_t N, int64_t K, int n_batches) {
  return carve_select(nullptr, M, N, K, n_batches, nullptr);
}

// partial sums, then the given order as slot offsets
size_t quant_error_workspace_bytes(int64_t rows, int64_t K) {
  return align_up((size_t)kQeParts(rows) * 8, 256) + align_up((size_t)K * 4, 256);
}

int run_quant_error(pq_format fmt, int group, const void* x, int64_t rows, int64_t K,
                    const int32_t* perm, float ts, double* err_out, void* ws, hipStream_t st) {
  double* part = (double*)ws;
  TensorList tl;
  for (int b = 0; b < kMaxMomentBatches; ++b) tl.p[b] = (const uint16_t*)x;
  const QeShape q = qe_shape(fmt, rows, K, 1, 1);
  int32_t* offs = nullptr;
  if (perm) {
    offs = (int32_t*)((char*)ws + align_up((size_t)kQeParts(rows) * 8, 256));
    hipLaunchKernelGGL(perm_to_offsets_kernel, dim3((unsigned)((K + 255) / 256)), dim3(256), 0, st, perm, (int)K,
                       qe_slot_bytes(q.r), offs);
  }
  int rc = launch_quant_error(fmt, group, tl, 1, rows, (int)K, q, offs, 1, perm ? 0 : 1, ScaleArg{ts, nullptr},
                              nullptr, part, st);
  if (rc) return rc;
  hipLaunchKernelGGL(reduce_rows_kernel, dim3(1, 1), dim3(256), 0, st, part, (int64_t)q.parts(), 1, 1,
                     fmt == PQ_FMT_NVFP4 ? 1 : 0, err_out);
  return check_hip(hipGetLastError(), "reduce_rows_kernel");
}

// The candidate orders of the alpha grid (joint score, descending stable sort) into
// cands[n_alpha][K]; keys [PQ_MAX_ALPHAS][K] doubles and rank [PQ_MAX_ALPHAS][K] ints are scratch.
// With offs ([n_alpha][K]), the same orders are also written as slot offsets of slot_bytes a slot.
int launch_candidate_orders(const double* act_sumsq, const double* w_sumsq, int64_t K, const double* alphas,
                            int n_alpha, double* keys, int32_t* rank, int32_t* cands, hipStream_t st,
                            int32_t* offs, int slot_bytes, uint32_t* differs) {
  const unsigned kb = (unsigned)((K + 255) / 256);
  const int chunks = rank_chunks(K);
  AlphaList al;
  for (int j = 0; j < PQ_MAX_ALPHAS; ++j) al.a[j] = j < n_alpha ? alphas[j] : 0.0;
  hipLaunchKernelGGL(key_kernel, dim3(kb, n_alpha), dim3(256), 0, st, act_sumsq, w_sumsq, K, al, keys, rank, differs);
  hipLaunchKernelGGL(rank_count_kernel, dim3(kb, chunks, n_alpha), dim3(256), 0, st, keys, (int)K, rank);
  hipLaunchKernelGGL(rank_scatter_kernel, dim3(kb, n_alpha), dim3(256), 0, st, rank, (int)K, cands, offs,
                     slot_bytes);
  if (differs)          // which orders repeat an earlier candidate (or the original order)
    hipLaunchKernelGGL(same_order_kernel, dim3(kb, n_alpha), dim3(256), 0, st, cands, (int)K, differs);
  return check_hip(hipGetLastError(), "key/rank kernels");
}

// ---- orders of the ablation (paper Tab. 2a) that are not a sort by a statistic
// round-robin: rank r of `order` goes to group r mod (K / g), slot r div (K / g)
__global__ __launch_bounds__(256) void round_robin_kernel(const int32_t* __restrict__ order, int K, int g,
                                                         int32_t* __restrict__ perm) {
  const int r = blockIdx.x * 256 + threadIdx.x;
  if (r >= K) return;
  const int n_groups = K / g;
  perm[(r % n_groups) * g + r / n_groups] = order[r];
}

// random: key[i] = -(splitmix64(seed + i) >> 11) as a double (53 bits: exact), so that the descending
// stable sort used for the scores gives ascending hashes with ties in ascending channel order
__global__ __launch_bounds__(256) void random_key_kernel(uint64_t seed, int K, double* __restrict__ keys,
                                                        int32_t* __restrict__ rank) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= K) return;
  uint64_t z = seed + (uint64_t)i + 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  z = z ^ (z >> 31);
  keys[i] = -(double)(z >> 11);
  rank[i] = 0;
}

int launch_round_robin(const int32_t* order, int64_t K, int group, int32_t* perm, hipStream_t st) {
  hipLaunchKernelGGL(round_robin_kernel, dim3((unsigned)((K + 255) / 256)), dim3(256), 0, st, order, (int)K, group, perm);
  return check_hip(hipGetLastError(), "round_robin_kernel");
}

size_t random_order_workspace_bytes(int64_t K) { return align_up((size_t)K * 8, 256) + align_up((size_t)K * 4, 256); }

int launch_random_order(uint64_t seed, int64_t K, int32_t* perm, void* ws, hipStream_t st) {
  double* keys = (double*)ws;
  int32_t* rank = (int32_t*)((char*)ws + align_up((size_t)K * 8, 256));
  const unsigned kb = (unsigned)((K + 255) / 256);
  hipLaunchKernelGGL(random_key_kernel, dim3(kb), dim3(256), 0, st, seed, (int)K, keys, rank);
  hipLaunchKernelGGL(rank_count_kernel, dim3(kb, rank_chunks(K), 1), dim3(256), 0, st, keys, (int)K, rank);
  hipLaunchKernelGGL(rank_scatter_kernel, dim3(kb, 1), dim3(256), 0, st, rank, (int)K, perm,
                     (int32_t*)nullptr, 0);
  return check_hip(hipGetLastError(), "random order kernels");
}

int launch_identity_order(int32_t* perm, int64_t K, hipStream_t st) {
  hipLaunchKernelGGL(iota_kernel, dim3((unsigned)((K + 255) / 256)), dim3(256), 0, st, perm, (int)K);
  return check_hip(hipGetLastError(), "iota_kernel");
}

// A pinned host buffer of at least n doubles that the calling thread keeps until it ends
// (a device-to-host copy into pageable memory goes through a staging copy and costs some 10 us
// more).  Grown, never shrunk; nullptr when the allocation fails.
struct PinnedBuffer {
  double* buf = nullptr;
  size_t cap = 0;
  ~PinnedBuffer() {                      // runs when the owning thread ends
    if (buf) (void)hipHostFree(buf);
  }
};
double* pinned_doubles(size_t n) {
  thread_local PinnedBuffer pb;
  if (n > pb.cap) {
    if (pb.buf) (void)hipHostFree(pb.buf);
    pb.buf = nullptr;
    pb.cap = 0;
    const size_t want = n < 512 ? 512 : n;
    void* p = nullptr;
    if (hipHostMalloc(&p, want * sizeof(double), hipHostMallocDefault) != hipSuccess) {
      (void)hipGetLastError();
      return nullptr;
    }
    pb.buf = (double*)p;
    pb.cap = want;
  }
  return pb.buf;
}

int run_select(pq_format fmt, int group, const double* act_sumsq, const double* w_sumsq, int64_t K,
               const void* const* x_calib, int n_batches, int64_t M, const void* w, int64_t N,
               float act_ts, float w_ts, const float* act_ts_dev, const float* w_ts_dev, const double* alphas,
               int n_alpha, double tau, int32_t* perm_out, pq_select_report* report, void* ws, hipStream_t st) {
  SelectWs W;
  carve_select(ws, M, N, K, n_batches, &W);
  const int n_cand = n_alpha + 1;            // candidate 0 is the original order
  int rc;
  // activations: all batches of a launch share one grid (up to kMaxMomentBatches per launch)
  const QeShape qa = qe_shape(fmt, M, K, n_batches < kMaxMomentBatches ? n_batches : kMaxMomentBatches, n_cand);
  const QeShape qw = qe_shape(fmt, N, K, 1, n_cand);       // the same resident rows (a function of K): one set of offsets
  if ((rc = launch_candidate_orders(act_sumsq, w_sumsq, K, alphas, n_alpha, W.keys, W.rank, W.cands, st, W.offs,
                                    qe_slot_bytes(qa.r), W.same_as)))
    return rc;
  double* sums = W.sums;
  for (int b0 = 0; b0 < n_batches; b0 += kMaxMomentBatches) {
    const int nb = n_batches - b0 < kMaxMomentBatches ? n_batches - b0 : kMaxMomentBatches;
    TensorList tl;
    for (int b = 0; b < kMaxMomentBatches; ++b) tl.p[b] = (const uint16_t*)x_calib[b0 + (b < nb ? b : 0)];
    rc = launch_quant_error(fmt, group, tl, nb, M, (int)K, qa, W.offs, n_cand, 1, ScaleArg{act_ts, act_ts_dev},
                            W.same_as, W.row_err + (size_t)b0 * qa.parts() * n_cand, st);
    if (rc) return rc;
  }
  double* w_part = W.row_err + (size_t)n_batches * qa.parts() * n_cand;
  TensorList wl;
  for (int b = 0; b < kMaxMomentBatches; ++b) wl.p[b] = (const uint16_t*)w;
  rc = launch_quant_error(fmt, group, wl, 1, N, (int)K, qw, W.offs, n_cand, 1, ScaleArg{w_ts, w_ts_dev}, W.same_as,
                          w_part, st);
  if (rc) return rc;
  TailArgs ta{W.row_err, w_part, act_sumsq, w_sumsq, W.cands, W.same_as, qa.parts(), qw.parts(), K, n_cand, n_batches,
              n_alpha};
  hipLaunchKernelGGL(select_tail_kernel, dim3((unsigned)(n_cand * (n_batches + 1) + 2 + n_alpha)), dim3(256), 0,
                     st, ta, sums);
  if ((rc = check_hip(hipGetLastError(), "select_tail_kernel"))) return rc;

  const size_t n_tot = (size_t)(n_batches + 1) * kMaxCand;      // offset of the two totals
  const size_t n_sums = n_tot + 2 + (size_t)n_alpha;
  double* h = pinned_doubles(n_sums);
  if (!h) return fail(PQ_ERR_HIP, "pq_select_perm: no pinned host memory for %zu sums", n_sums);
  if ((rc = check_hip(hipMemcpyAsync(h, sums, n_sums * 8, hipMemcpyDeviceToHost, st), "copy sums"))) return rc;
  if ((rc = check_hip(hipStreamSynchronize(st), "hipStreamSynchronize"))) return rc;

  const double sum_x2 = h[n_tot], sum_w2 = h[n_tot + 1];
  double E[kMaxCand];
  for (int c = 0; c < n_cand; ++c) {
    double ex = 0.0;
    for (int b = 0; b < n_batches; ++b) ex += h[(size_t)b * kMaxCand + c];
    double ew = h[(size_t)n_batches * kMaxCand + c];
    if (fmt == PQ_FMT_NVFP4) {
      // NVFP4 errors are differences known to about 1e-15 of the tensor's sum of squares: below 1e-13 of it
      // they are not told from zero (data the format holds exactly), and are reported as zero
      if (ex < 1e-13 * sum_x2) ex = 0.0;
      if (ew < 1e-13 * sum_w2) ew = 0.0;
    }
    E[c] = ex / sum_x2 + ew / sum_w2;
  }
  int best = 0;
  for (int j = 1; j < n_alpha; ++j)
    if (E[1 + j] < E[1 + best]) best = j;         // first minimum: smallest alpha on ties
  const double e_orig = E[0], e_best = E[1 + best];
  const bool accepted = h[n_tot + 2 + best] != 0.0 && e_orig > 0.0 && ((e_orig - e_best) / e_orig > tau);
  memset(report, 0, sizeof(*report));
  report->accepted = accepted ? 1 : 0;
  report->alpha_index = best;
  report->e_orig = e_orig;
  report->e_best = e_best;
  for (int j = 0; j < n_alpha; ++j) report->e_cand[j] = E[1 + j];
  report->sum_x2 = sum_x2;
  report->sum_w2 = sum_w2;
  if (accepted) {
    rc = check_hip(hipMemcpyAsync(perm_out, W.cands + (int64_t)best * K, (size_t)K * 4,
                                  hipMemcpyDeviceToDevice, st), "copy permutation");
  } else {
    rc = launch_identity_order(perm_out, K, st);
  }
  return rc;
}

}  // namespace pq
