// Training kernels (Sec. 4.1 "The k-means vector quantizer"; Sec. 5.1 "Encoding
// residuals"): the update step of Lloyd's iteration and the residual sub-vectors the
// sub-quantizers are trained on.  The assignment step is the library's k-nearest-rows
// routine with k = 1.
#include <algorithm>

#include "common.hpp"
#include "internal.hpp"

namespace {

// One wavefront per centroid j.  order[off[j] .. off[j + 1]) lists the vectors assigned to
// it in ascending order; lane t adds up dimensions t, t + 64, ... of those vectors in
// float64, in that order -- a fixed order, so the sum has one value however the kernel is
// scheduled -- and stores sum / count rounded to fp32.  A centroid without vectors is left
// as it is.  Dimensions are taken 256 at a time.
__global__ __launch_bounds__(256) void segmented_mean_kernel(const float* __restrict__ x, int d,
                                                             const int32_t* __restrict__ order,
                                                             const int64_t* __restrict__ off, int K,
                                                             float* __restrict__ centroids) {
  const int wave = threadIdx.x >> 6, lane = lane_id();
  const int64_t j = blockIdx.x * 4ll + wave;
  if (j >= K) return;
  const int64_t b = off[j], e = off[j + 1];
  if (b == e) return;
  const double count = (double)(e - b);
  for (int t0 = 0; t0 < d; t0 += 256) {
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll 4
    for (int64_t i = b; i < e; ++i) {
      const float* __restrict__ row = x + (int64_t)order[i] * d + t0;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int t = lane + 64 * c;
        if (t0 + t < d) acc[c] += (double)row[t];
      }
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int t = t0 + lane + 64 * c;
      if (t < d) centroids[j * d + t] = (float)(acc[c] / count);
    }
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

void launch_segmented_mean(const float* x, int d, const int32_t* order, const int64_t* off, int K,
                           float* centroids, hipStream_t st) {
  if (K <= 0) return;
  hipLaunchKernelGGL(segmented_mean_kernel, dim3((unsigned)((K + 3) / 4)), dim3(256), 0, st, x, d,
                     order, off, K, centroids);
}

void launch_residual_slices(const float* x, int64_t n, int d, int dsub, const float* centroids,
                            const int32_t* list_of, float* out, hipStream_t st) {
  if (n <= 0) return;
  hipLaunchKernelGGL(residual_slices_kernel,
                     dim3((unsigned)std::min<int64_t>(1 << 22, (n * d + 255) / 256)), dim3(256), 0, st,
                     x, n, d, dsub, centroids, list_of, out);
}
