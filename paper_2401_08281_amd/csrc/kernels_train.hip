// Training kernels (Sec. 4.1 "The k-means vector quantizer"; Sec. 5.1 "Encoding
// residuals"): the update step of Lloyd's iteration and the residual sub-vectors the
// sub-quantizers are trained on.  The assignment step is the library's k-nearest-rows
// routine with k = 1.
#include <algorithm>

#include "common.hpp"
#include "internal.hpp"

namespace {

constexpr int64_t kBlock = 4096;   // vectors per summation block (a multiple of every batch below)

// One wavefront per (centroid j, block of kBlock vectors).  order[off[j] .. off[j + 1])
// lists the vectors assigned to centroid j in ascending order; they are summed in float64 in
// blocks of kBlock: a block from 0 in the list's order, the block sums in block order -- a
// fixed order, so the sum has one value however the kernels are scheduled, and the blocks of
// a large cluster run side by side (sixteen centroids over millions of sub-vectors would
// otherwise be sixteen chains).  A centroid of one block stores sum / count rounded to fp32
// directly; the others store their block sums to `partial` (block bk of centroid j at slot
// off[j] / kBlock + j + bk: the slots of different centroids never overlap) and
// segmented_mean_finish_kernel adds them up.  A centroid without vectors is left as it is.
// Lane t adds up dimensions t, t + 64, ...; dimensions are taken 64 * NC at a time (NC = 1,
// 2 or 4).
// The chain of a large cluster is long (it sets the kernel's time), so the memory latency
// is taken off it: 64 / NC vectors at a time, their numbers come in with one load, their
// rows are all requested before the first is added, and the additions then run in the
// list's order.
template <int NC>
__global__ __launch_bounds__(256) void segmented_mean_kernel(const float* __restrict__ x, int d,
                                                             const int32_t* __restrict__ order,
                                                             const int64_t* __restrict__ off, int K,
                                                             float* __restrict__ centroids,
                                                             double* __restrict__ partial) {
  constexpr int NB = 64 / NC;
  const int wave = threadIdx.x >> 6, lane = lane_id();
  const int64_t j = blockIdx.x * 4ll + wave;
  if (j >= K) return;
  const int64_t b0 = off[j], e0 = off[j + 1];
  if (b0 == e0) return;
  const double count = (double)(e0 - b0);
  const int64_t nblk = (e0 - b0 + kBlock - 1) / kBlock;
  for (int64_t bk = blockIdx.y; bk < nblk; bk += gridDim.y)
  for (int t0 = 0; t0 < d; t0 += 64 * NC) {
    const int64_t b = b0 + bk * kBlock, e = min(e0, b + kBlock);
    double acc[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) acc[c] = 0.0;
    int64_t i = b;
    for (; i + NB <= e; i += NB) {
      const int32_t mine = order[i + (lane & (NB - 1))];
      float v[NB][NC];
#pragma unroll
      for (int u = 0; u < NB; ++u) {
        const float* __restrict__ row = x + (int64_t)__shfl(mine, u) * d + t0;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
          const int t = lane + 64 * c;
          v[u][c] = t0 + t < d ? row[t] : 0.f;
        }
      }
#pragma unroll
      for (int u = 0; u < NB; ++u)
#pragma unroll
        for (int c = 0; c < NC; ++c) acc[c] += (double)v[u][c];
    }
    for (; i < e; ++i) {
      const float* __restrict__ row = x + (int64_t)order[i] * d + t0;
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        const int t = lane + 64 * c;
        if (t0 + t < d) acc[c] += (double)row[t];
      }
    }
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const int t = t0 + lane + 64 * c;
      if (t < d) {
        if (nblk == 1) centroids[j * d + t] = (float)(acc[c] / count);
        else partial[(b0 / kBlock + j + bk) * d + t] = acc[c];
      }
    }
  }
}

// The same for rows of at most 32 floats (the sub-vectors of a product quantizer), where one
// row per load instruction would leave most lanes idle: lane (s, t) = (lane / DP, lane % DP)
// reads dimension t of every (64 / DP)-th vector, so one load instruction fetches 64 / DP
// rows and a batch of 16 instructions 16 * 64 / DP vectors; the chain of dimension t then
// takes the values in the list's order through cross-lane reads (it is kept in every group
// s alike).  DP: d rounded up to 8, 16 or 32.
template <int DP>
__global__ __launch_bounds__(256) void segmented_mean_small_kernel(const float* __restrict__ x, int d,
                                                                   const int32_t* __restrict__ order,
                                                                   const int64_t* __restrict__ off, int K,
                                                                   float* __restrict__ centroids,
                                                                   double* __restrict__ partial) {
  constexpr int VPL = 64 / DP, NU = 16, NBV = NU * VPL;          // vectors per load, loads and vectors per batch
  constexpr int NO = (NBV + 63) / 64;                            // registers of vector numbers per batch
  static_assert(kBlock % NBV == 0, "whole batches per block");
  const int wave = threadIdx.x >> 6, lane = lane_id();
  const int s = lane / DP, t = lane % DP;
  const int64_t j = blockIdx.x * 4ll + wave;
  if (j >= K) return;
  const int64_t b0 = off[j], e0 = off[j + 1];
  if (b0 == e0) return;
  const double count = (double)(e0 - b0);
  const int64_t nblk = (e0 - b0 + kBlock - 1) / kBlock;
  for (int64_t bk = blockIdx.y; bk < nblk; bk += gridDim.y) {
  const int64_t b = b0 + bk * kBlock, e = min(e0, b + kBlock);
  double acc = 0.0;
  int64_t i = b;
  for (; i + NBV <= e; i += NBV) {
    int32_t mine[NO];
#pragma unroll
    for (int o = 0; o < NO; ++o) mine[o] = (64 * o + lane) < NBV ? order[i + 64 * o + lane] : 0;
    float v[NU];
#pragma unroll
    for (int u = 0; u < NU; ++u) {
      const int w = u * VPL + s;                                 // this lane's vector of load u: number w of the batch
      const int32_t r = __shfl(mine[(u * VPL) / 64], w & 63);    // (a load's vectors sit in one register of numbers)
      v[u] = t < d ? x[(int64_t)r * d + t] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < NU; ++u)
#pragma unroll
      for (int s2 = 0; s2 < VPL; ++s2) acc += (double)__shfl(v[u], s2 * DP + t);
  }
  for (; i < e; ++i)                                             // the rest, one vector at a time
    if (t < d) acc += (double)x[(int64_t)order[i] * d + t];
  if (s == 0 && t < d) {
    if (nblk == 1) centroids[j * d + t] = (float)(acc / count);
    else partial[(b0 / kBlock + j + bk) * d + t] = acc;
  }
  }
}

// Centroids of more than one block: the block sums in block order, then the mean.
__global__ __launch_bounds__(256) void segmented_mean_finish_kernel(const double* __restrict__ partial,
                                                                    int d,
                                                                    const int64_t* __restrict__ off, int K,
                                                                    float* __restrict__ centroids) {
  const int wave = threadIdx.x >> 6, lane = lane_id();
  const int64_t j = blockIdx.x * 4ll + wave;
  if (j >= K) return;
  const int64_t b0 = off[j], e0 = off[j + 1];
  const int64_t nblk = (e0 - b0 + kBlock - 1) / kBlock;
  if (nblk <= 1) return;
  const double count = (double)(e0 - b0);
  const double* __restrict__ src = partial + (b0 / kBlock + j) * d;
  for (int t = lane; t < d; t += VS_WAVE) {
    double total = 0.0;
    for (int64_t bk = 0; bk < nblk; ++bk) total += src[bk * d + t];
    centroids[j * d + t] = (float)(total / count);
  }
}

// out[m][i][u] = x[i][m * dsub + u] - centroids[list_of[i]][m * dsub + u]: the residual of
// every vector (one fp32 subtraction per component), regrouped into M contiguous matrices
// of sub-vectors.
__global__ __launch_bounds__(256) void residual_slices_kernel(const float* __restrict__ x, int64_t n,
                                                              int d, int dsub,
                                                              const float* __restrict__ centroids,
                                                              const int32_t* __restrict__ list_of,
                                                              float* __restrict__ out) {
  const int64_t total = n * d, stride = (int64_t)gridDim.x * 256;   // grid-stride: n * d may exceed 2^32
  for (int64_t e = blockIdx.x * 256ll + threadIdx.x; e < total; e += stride) {
    const int64_t i = e / d;
    const int t = (int)(e - i * d);
    const int m = t / dsub, u = t - m * dsub;
    out[((int64_t)m * n + i) * dsub + u] = x[e] - centroids[(int64_t)list_of[i] * d + t];
  }
}

}  // namespace

size_t segmented_mean_partial_bytes(int64_t n, int d, int K, int64_t largest) {
  if (largest <= kBlock) return 0;
  return (size_t)(n / kBlock + K + 1) * d * sizeof(double);
}

void launch_segmented_mean(const float* x, int d, const int32_t* order, const int64_t* off, int K,
                           int64_t largest, float* centroids, double* partial, hipStream_t st) {
  if (K <= 0) return;
  // `largest` = size of the largest cluster (the host counted): its number of blocks is the grid's second dimension
  const int64_t nblk = std::max<int64_t>(1, (largest + kBlock - 1) / kBlock);
  const dim3 grid((unsigned)((K + 3) / 4), (unsigned)std::min<int64_t>(nblk, 65535)), block(256);
  if (d <= 8) hipLaunchKernelGGL((segmented_mean_small_kernel<8>), grid, block, 0, st, x, d, order, off, K, centroids, partial);
  else if (d <= 16) hipLaunchKernelGGL((segmented_mean_small_kernel<16>), grid, block, 0, st, x, d, order, off, K, centroids, partial);
  else if (d <= 32) hipLaunchKernelGGL((segmented_mean_small_kernel<32>), grid, block, 0, st, x, d, order, off, K, centroids, partial);
  else if (d <= 64) hipLaunchKernelGGL((segmented_mean_kernel<1>), grid, block, 0, st, x, d, order, off, K, centroids, partial);
  else if (d <= 128) hipLaunchKernelGGL((segmented_mean_kernel<2>), grid, block, 0, st, x, d, order, off, K, centroids, partial);
  else hipLaunchKernelGGL((segmented_mean_kernel<4>), grid, block, 0, st, x, d, order, off, K, centroids, partial);
  if (nblk > 1)
    hipLaunchKernelGGL(segmented_mean_finish_kernel, dim3((unsigned)((K + 3) / 4)), block, 0, st, partial, d, off, K,
                       centroids);
}

void launch_residual_slices(const float* x, int64_t n, int d, int dsub, const float* centroids,
                            const int32_t* list_of, float* out, hipStream_t st) {
  if (n <= 0) return;
  hipLaunchKernelGGL(residual_slices_kernel,
                     dim3((unsigned)std::min<int64_t>(1 << 22, (n * d + 255) / 256)), dim3(256), 0, st,
                     x, n, d, dsub, centroids, list_of, out);
}
