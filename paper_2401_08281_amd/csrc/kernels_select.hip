// k-selection over rows of a distance matrix, and key -> result conversion.
#include "common.hpp"
#include "internal.hpp"

namespace {

__global__ void fill_u64_kernel(u64* p, int64_t n, u64 v) {
  const int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// One workgroup (4 wavefronts) per row.  Each wavefront selects over a
// quarter of the columns with its own WaveSelect; the four sorted results and
// the row's previous best k (when the row continues an earlier chunk) are then
// merged by ranking.  The previous k-th best key seeds every wavefront's
// threshold, so that nearly all columns are rejected by a single compare.
template <int R>
__global__ __launch_bounds__(256) void row_select_kernel(const float* __restrict__ mat, int64_t ld,
                                                         int64_t ncols, u32 col_base, int metric,
                                                         int k, int tot, u64* __restrict__ keys,
                                                         int first, int last, SelectOut out) {
  extern __shared__ u64 slots[];  // 5 * tot: four wavefronts, then the previous best k
  const int wave = threadIdx.x >> 6, lane = lane_id();
  const int64_t row = blockIdx.x;
  const float* __restrict__ m = mat + row * ld;
  const u64* kr = first ? nullptr : keys + row * (int64_t)k;
  u64* prev = slots + 4 * tot;

  WaveSelect<R> ws;
  ws.init(slots + wave * tot, tot, k);
  for (int j = threadIdx.x; j < k; j += 256) prev[j] = first ? KEY_EMPTY : kr[j];
  if (!first) ws.thresh = kr[k - 1];            // may be KEY_EMPTY: then nothing is rejected
  for (int64_t c0 = wave * VS_WAVE; c0 < ncols; c0 += 4 * VS_WAVE) {
    const int64_t c = c0 + lane;
    const bool valid = c < ncols;
    const float v = valid ? m[c] : 0.f;
    ws.push(valid, make_key(v, col_base + (u32)c, metric));
  }
  ws.finish();
  __syncthreads();
  KeySink sink;
  sink.keys = last ? nullptr : keys;
  sink.val = last ? out.val : nullptr;
  sink.id64 = last ? out.id64 : nullptr;
  sink.idx32 = last ? out.idx32 : nullptr;
  sink.idmap = nullptr;
  sink.metric = metric;
  block_rank_merge(slots, tot, 5, k, sink, row * (int64_t)k);
}

__global__ void keys_to_results_kernel(const u64* __restrict__ keys, int64_t n, int metric,
                                       float* __restrict__ out_dist, int64_t* __restrict__ out_ids,
                                       const int64_t* __restrict__ idmap) {
  const int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i >= n) return;
  const u64 key = keys[i];
  if (key == KEY_EMPTY) {
    out_dist[i] = metric ? -__builtin_inff() : __builtin_inff();
    out_ids[i] = -1;
  } else {
    out_dist[i] = key_value(key, metric);
    const u32 idx = key_index(key);
    out_ids[i] = idmap ? idmap[idx] : (int64_t)idx;
  }
}

__global__ void keys_to_probes_kernel(const u64* __restrict__ keys, int64_t n, int metric,
                                      int32_t* __restrict__ out_idx, float* __restrict__ out_val) {
  const int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i >= n) return;
  const u64 key = keys[i];
  if (key == KEY_EMPTY) {
    out_idx[i] = -1;
    if (out_val) out_val[i] = metric ? -__builtin_inff() : __builtin_inff();
  } else {
    out_idx[i] = (int32_t)key_index(key);
    if (out_val) out_val[i] = key_value(key, metric);
  }
}

}  // namespace

void launch_fill_u64(u64* p, int64_t n, u64 v, hipStream_t st) {
  if (n <= 0) return;
  hipLaunchKernelGGL(fill_u64_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, n, v);
}

void launch_row_select(const float* mat, int64_t ld, int64_t nrows, int64_t ncols, u32 col_base,
                       int metric, int k, u64* keys, bool first, bool last, const SelectOut& out,
                       hipStream_t st) {
  if (nrows <= 0) return;
  const int tot = select_slots_for_k(k);
  const size_t shmem = (size_t)5 * tot * sizeof(u64);
  const dim3 grid((unsigned)nrows), block(256);
#define LAUNCH(RR)                                                                                 \
  do {                                                                                             \
    if (shmem > 48 * 1024)                                                                         \
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&row_select_kernel<RR>),             \
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);           \
    hipLaunchKernelGGL((row_select_kernel<RR>), grid, block, shmem, st, mat, ld, ncols, col_base,  \
                       metric, k, tot, keys, first ? 1 : 0, last ? 1 : 0, out);                    \
  } while (0)
  switch (select_regs_for_slots(tot)) {
    case 2: LAUNCH(2); break;
    case 4: LAUNCH(4); break;
    default: LAUNCH(0); break;
  }
#undef LAUNCH
}

void launch_keys_to_results(const u64* keys, int64_t n, int metric, float* out_dist,
                            int64_t* out_ids, const int64_t* idmap, hipStream_t st) {
  if (n <= 0) return;
  hipLaunchKernelGGL(keys_to_results_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                     keys, n, metric, out_dist, out_ids, idmap);
}

void launch_keys_to_probes(const u64* keys, int64_t n, int metric, int32_t* out_idx,
                           float* out_val, hipStream_t st) {
  if (n <= 0) return;
  hipLaunchKernelGGL(keys_to_probes_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                     keys, n, metric, out_idx, out_val);
}

void launch_keys_to_index32(const u64* keys, int64_t n, int32_t* out_idx, hipStream_t st) {
  launch_keys_to_probes(keys, n, 0, out_idx, nullptr, st);
}
