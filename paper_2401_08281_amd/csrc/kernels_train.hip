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

// ---- bookkeeping of a k-means round on the device -----------------------------------
// The update needs, for every centroid, the numbers of its vectors in ascending order: a
// stable counting sort of the assignment idx [n] by centroid.  The vectors are cut into at
// most 256 chunks of consecutive vectors:
//   km_hist_kernel     per chunk, how many vectors go to each centroid        mat [nchunk][K]
//   km_colscan_kernel  per centroid, exclusive running sum down the chunks (in place) and the total
//   km_offsets_kernel  exclusive sum of the totals = first slot of each centroid, off [K + 1];
//                      the largest total
//   km_scatter_kernel  one wavefront per chunk walks over its vectors in order, 64 at a time:
//                      lanes with the same centroid are ranked by lane number (ballot), so
//                      every vector gets slot off[j] + (vectors of j in earlier chunks) +
//                      (earlier vectors of j in this chunk): the stable order.
// K <= 16384 (one counter per centroid in LDS); the host does the same sort otherwise.
__global__ __launch_bounds__(256) void km_hist_kernel(const int32_t* __restrict__ idx, int64_t n, int K,
                                                      int64_t chunk, int32_t* __restrict__ mat,
                                                      int* __restrict__ bad) {
  extern __shared__ int km_lds[];
  for (int j = threadIdx.x; j < K; j += 256) km_lds[j] = 0;
  __syncthreads();
  const int64_t i0 = blockIdx.x * chunk, i1 = min(n, i0 + chunk);
  for (int64_t i = i0 + threadIdx.x; i < i1; i += 256) {
    const int32_t j = idx[i];
    if (j < 0 || j >= K) *bad = 1;
    else atomicAdd(&km_lds[j], 1);
  }
  __syncthreads();
  for (int j = threadIdx.x; j < K; j += 256) mat[(int64_t)blockIdx.x * K + j] = km_lds[j];
}

__global__ __launch_bounds__(256) void km_colscan_kernel(int32_t* __restrict__ mat, int nchunk, int K,
                                                         int64_t* __restrict__ cnt) {
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= K) return;
  int32_t run = 0;
  for (int c = 0; c < nchunk; ++c) {
    const int32_t v = mat[(int64_t)c * K + j];
    mat[(int64_t)c * K + j] = run;
    run += v;
  }
  cnt[j] = run;
}

// one workgroup: lane t owns centroids [t * per, (t + 1) * per)
__global__ __launch_bounds__(256) void km_offsets_kernel(const int64_t* __restrict__ cnt, int K,
                                                         int64_t* __restrict__ off,
                                                         int64_t* __restrict__ largest) {
  __shared__ int64_t part[256], big[256];
  const int t = threadIdx.x, per = (K + 255) / 256;
  const int j0 = min(K, t * per), j1 = min(K, j0 + per);
  int64_t sum = 0, mx = 0;
  for (int j = j0; j < j1; ++j) { sum += cnt[j]; mx = max(mx, cnt[j]); }
  part[t] = sum; big[t] = mx;
  __syncthreads();
  int64_t base = 0;
  for (int u = 0; u < t; ++u) base += part[u];
  for (int j = j0; j < j1; ++j) { off[j] = base; base += cnt[j]; }
  if (t == 255) {
    int64_t total = 0, m = 0;
    for (int u = 0; u < 256; ++u) { total += part[u]; m = max(m, big[u]); }
    off[K] = total;
    *largest = m;
  }
}

__global__ __launch_bounds__(64) void km_scatter_kernel(const int32_t* __restrict__ idx, int64_t n, int K,
                                                        int64_t chunk, const int32_t* __restrict__ mat,
                                                        const int64_t* __restrict__ off,
                                                        int32_t* __restrict__ order) {
  extern __shared__ int km_lds[];                       // next slot of every centroid for this chunk
  const int lane = lane_id();
  for (int j = lane; j < K; j += VS_WAVE) km_lds[j] = (int)(off[j] + mat[(int64_t)blockIdx.x * K + j]);
  wave_lds_sync();
  const int64_t i0 = blockIdx.x * chunk, i1 = min(n, i0 + chunk);
  for (int64_t g = i0; g < i1; g += VS_WAVE) {
    const int64_t i = g + lane;
    const bool valid = i < i1;
    int32_t key = valid ? idx[i] : -1;
    if (key >= K) key = -1;                             // (flagged by km_hist_kernel; never stored)
    u64 todo = __builtin_amdgcn_ballot_w64(key >= 0);
    while (todo != 0) {                                 // one round per distinct centroid among the 64
      const int leader = __builtin_ctzll(todo);
      const int32_t k = __shfl(key, leader);
      const u64 same = __builtin_amdgcn_ballot_w64(key == k);
      const int base = km_lds[k];
      if (key == k) order[base + __popcll(same & ((1ull << lane) - 1ull))] = (int32_t)i;
      wave_lds_sync();                                  // everyone has read the slot before it moves
      if (lane == leader) km_lds[k] = base + __popcll(same);
      wave_lds_sync();
      todo &= ~same;
    }
  }
}

// Sum of val [n] in float64 in a fixed order: workgroup w sums a contiguous slice (lane-strided,
// then a fixed tree), the host adds the 256 partial sums in order.
__global__ __launch_bounds__(256) void km_objective_kernel(const float* __restrict__ val, int64_t n,
                                                           double* __restrict__ partial) {
  __shared__ double red[256];
  const int64_t per = (n + gridDim.x - 1) / gridDim.x;
  const int64_t i0 = blockIdx.x * per, i1 = min(n, i0 + per);
  double acc = 0.0;
  for (int64_t i = i0 + threadIdx.x; i < i1; i += 256) acc += (double)val[i];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) partial[blockIdx.x] = red[0];
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

size_t kmeans_sort_bytes(int64_t n, int K) {
  (void)n;
  return (size_t)256 * K * sizeof(int32_t) + (size_t)K * sizeof(int64_t) + 256 * sizeof(double) + 64;
}

// work: kmeans_sort_bytes(n, K); out: order [n], off [K + 1]; in the work space afterwards:
// scal[0] = the largest cluster (int64), scal[1] = 1 if an assignment was out of range,
// partial [256] doubles whose sum is the sum of val.
void launch_kmeans_sort(const int32_t* idx, const float* val, int64_t n, int K, char* work, int32_t* order,
                        int64_t* off, int64_t** scal_out, double** partial_out, hipStream_t st) {
  int32_t* mat = reinterpret_cast<int32_t*>(work);
  int64_t* cnt = reinterpret_cast<int64_t*>(work + (size_t)256 * K * sizeof(int32_t));
  double* partial = reinterpret_cast<double*>(cnt + K);
  int64_t* scal = reinterpret_cast<int64_t*>(partial + 256);
  *scal_out = scal; *partial_out = partial;
  const int64_t chunk = std::max<int64_t>(2048, ((n + 255) / 256 + 63) / 64 * 64);
  const int nchunk = (int)((n + chunk - 1) / chunk);
  const size_t lds = (size_t)K * sizeof(int);
  if (lds > 48 * 1024) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&km_hist_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&km_scatter_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  }
  launch_fill_u64(reinterpret_cast<u64*>(scal), 2, 0ull, st);
  hipLaunchKernelGGL(km_hist_kernel, dim3((unsigned)nchunk), dim3(256), lds, st, idx, n, K, chunk, mat,
                     reinterpret_cast<int*>(scal + 1));
  hipLaunchKernelGGL(km_colscan_kernel, dim3((unsigned)((K + 255) / 256)), dim3(256), 0, st, mat, nchunk, K, cnt);
  hipLaunchKernelGGL(km_offsets_kernel, dim3(1), dim3(256), 0, st, cnt, K, off, scal);
  hipLaunchKernelGGL(km_scatter_kernel, dim3((unsigned)nchunk), dim3(64), lds, st, idx, n, K, chunk, mat, off, order);
  hipLaunchKernelGGL(km_objective_kernel, dim3(256), dim3(256), 0, st, val, n, partial);
}

void launch_residual_slices(const float* x, int64_t n, int d, int dsub, const float* centroids,
                            const int32_t* list_of, float* out, hipStream_t st) {
  if (n <= 0) return;
  hipLaunchKernelGGL(residual_slices_kernel,
                     dim3((unsigned)std::min<int64_t>(1 << 22, (n * d + 255) / 256)), dim3(256), 0, st,
                     x, n, d, dsub, centroids, list_of, out);
}
