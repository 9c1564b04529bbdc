// Placement of newly added vectors into the inverted lists (Sec. 5.1 "Inverted files": the vectors
// of a cluster are stored contiguously), entirely on the device.
// Input: the list of every new vector, list_of [n].  Output: for every new vector its slot in the
// grown store, dest [n] -- behind the entries its list already holds and behind the new vectors of
// the same list that come earlier in the batch (add order is kept inside a list) -- and the grown
// lists' offsets new_off [nlist + 1].
// The order inside a list needs a STABLE sort of the batch by list.  It is a radix sort by list
// number, least significant digit first, 12 bits per pass (one pass up to 4096 lists, two up to
// 16.7M); every pass is a counting sort that keeps equal digits in input order:
//   place_hist_kernel     per chunk of consecutive positions, the count of every digit   mat [nchunk][4096]
//   place_colscan_kernel  per digit, exclusive running sum down the chunks (in place) and its total
//   place_digit_offsets_kernel  exclusive sum of the totals: first slot of every digit
//   place_scatter_kernel  one wavefront per chunk walks over its positions in order, 64 at a
//                         time; lanes with the same digit are ranked by lane number (ballot)
// then per-list counts (atomics: a count does not depend on order), two prefix sums over the
// lists, and dest from each vector's rank in the sorted batch.
#include <algorithm>

#include "common.hpp"
#include "internal.hpp"

namespace {

constexpr int kDigitBits = 12;
constexpr int kBuckets = 1 << kDigitBits;
constexpr int kMaxChunks = 1024;

__device__ __forceinline__ int digit_of(int32_t key, int shift) { return (key >> shift) & (kBuckets - 1); }

// position p of the pass holds vector perm[p] (or p itself when perm is null)
__global__ __launch_bounds__(256) void place_hist_kernel(const int32_t* __restrict__ keys,
                                                         const int32_t* __restrict__ perm, int64_t n, int nlist,
                                                         int shift, int64_t chunk, int32_t* __restrict__ mat,
                                                         int* __restrict__ bad) {
  __shared__ int h[kBuckets];
  for (int j = threadIdx.x; j < kBuckets; j += 256) h[j] = 0;
  __syncthreads();
  const int64_t p0 = blockIdx.x * chunk, p1 = min(n, p0 + chunk);
  for (int64_t p = p0 + threadIdx.x; p < p1; p += 256) {
    const int32_t key = keys[perm ? perm[p] : p];
    if (key < 0 || key >= nlist) *bad = 1;
    else atomicAdd(&h[digit_of(key, shift)], 1);
  }
  __syncthreads();
  for (int j = threadIdx.x; j < kBuckets; j += 256) mat[(int64_t)blockIdx.x * kBuckets + j] = h[j];
}

__global__ __launch_bounds__(256) void place_colscan_kernel(int32_t* __restrict__ mat, int nchunk,
                                                            int64_t* __restrict__ cnt) {
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= kBuckets) return;
  int32_t run = 0;
  for (int c = 0; c < nchunk; ++c) {
    const int32_t v = mat[(int64_t)c * kBuckets + j];
    mat[(int64_t)c * kBuckets + j] = run;
    run += v;
  }
  cnt[j] = run;
}

// one workgroup of 256: thread t owns digits [16 t, 16 t + 16)
__global__ __launch_bounds__(256) void place_digit_offsets_kernel(const int64_t* __restrict__ cnt,
                                                                  int64_t* __restrict__ off) {
  __shared__ int64_t part[256];
  constexpr int per = kBuckets / 256;
  const int t = threadIdx.x;
  int64_t sum = 0;
  for (int j = t * per; j < (t + 1) * per; ++j) sum += cnt[j];
  part[t] = sum;
  __syncthreads();
  int64_t base = 0;
  for (int u = 0; u < t; ++u) base += part[u];
  for (int j = t * per; j < (t + 1) * per; ++j) { off[j] = base; base += cnt[j]; }
}

__global__ __launch_bounds__(64) void place_scatter_kernel(const int32_t* __restrict__ keys,
                                                           const int32_t* __restrict__ perm, int64_t n, int nlist,
                                                           int shift, int64_t chunk, const int32_t* __restrict__ mat,
                                                           const int64_t* __restrict__ off,
                                                           int32_t* __restrict__ out) {
  __shared__ int next[kBuckets];                        // next slot of every digit for this chunk
  const int lane = lane_id();
  for (int j = lane; j < kBuckets; j += VS_WAVE) next[j] = (int)(off[j] + mat[(int64_t)blockIdx.x * kBuckets + j]);
  wave_lds_sync();
  const int64_t p0 = blockIdx.x * chunk, p1 = min(n, p0 + chunk);
  for (int64_t g = p0; g < p1; g += VS_WAVE) {
    const int64_t p = g + lane;
    int32_t i = -1, dg = -1;
    if (p < p1) {
      i = perm ? perm[p] : (int32_t)p;
      const int32_t key = keys[i];
      if (key >= 0 && key < nlist) dg = digit_of(key, shift);   // (others were flagged by the histogram pass)
    }
    u64 todo = __builtin_amdgcn_ballot_w64(dg >= 0);
    while (todo != 0) {                                 // one round per distinct digit among the 64
      const int leader = __builtin_ctzll(todo);
      const int32_t k = __shfl(dg, leader);
      const u64 same = __builtin_amdgcn_ballot_w64(dg == k);
      const int base = next[k];
      if (dg == k) out[base + __popcll(same & ((1ull << lane) - 1ull))] = i;
      wave_lds_sync();                                  // everyone has read the slot before it moves
      if (lane == leader) next[k] = base + __popcll(same);
      wave_lds_sync();
      todo &= ~same;
    }
  }
}

__global__ __launch_bounds__(256) void place_zero_kernel(int32_t* __restrict__ p, int64_t n) {
  const int64_t i = blockIdx.x * 256ll + threadIdx.x;
  if (i < n) p[i] = 0;
}

__global__ __launch_bounds__(256) void place_count_kernel(const int32_t* __restrict__ keys, int64_t n, int nlist,
                                                          int32_t* __restrict__ cnt) {
  const int64_t i = blockIdx.x * 256ll + threadIdx.x;
  if (i >= n) return;
  const int32_t l = keys[i];
  if (l >= 0 && l < nlist) atomicAdd(&cnt[l], 1);
}

// One workgroup of 1024: thread t owns lists [t * per, (t + 1) * per).
//   first_new[l] = number of new vectors in lists before l (their first rank in the sorted batch)
//   new_off[l]   = first slot of list l in the grown store = sum over lists before l of old size + new count
__global__ __launch_bounds__(1024) void place_list_offsets_kernel(const int32_t* __restrict__ cnt,
                                                                  const int64_t* __restrict__ old_off, int nlist,
                                                                  int64_t* __restrict__ first_new,
                                                                  int64_t* __restrict__ new_off) {
  __shared__ int64_t part_new[1024], part_all[1024];
  const int t = threadIdx.x, per = (nlist + 1023) / 1024;
  const int l0 = min(nlist, t * per), l1 = min(nlist, l0 + per);
  int64_t s_new = 0, s_all = 0;
  for (int l = l0; l < l1; ++l) {
    s_new += cnt[l];
    s_all += cnt[l] + (old_off[l + 1] - old_off[l]);
  }
  part_new[t] = s_new; part_all[t] = s_all;
  __syncthreads();
  int64_t b_new = 0, b_all = 0;
  for (int u = 0; u < t; ++u) { b_new += part_new[u]; b_all += part_all[u]; }
  for (int l = l0; l < l1; ++l) {
    first_new[l] = b_new; new_off[l] = b_all;
    b_new += cnt[l];
    b_all += cnt[l] + (old_off[l + 1] - old_off[l]);
  }
  if (l1 == nlist && l0 < nlist) new_off[nlist] = b_all;   // (the thread that owns the last list)
  if (nlist == 0 && t == 0) new_off[0] = 0;
}

// the vector at rank p of the sorted batch goes behind its list's old entries and the p -
// first_new[l] new ones before it
__global__ __launch_bounds__(256) void place_dest_kernel(const int32_t* __restrict__ order,
                                                         const int32_t* __restrict__ keys, int64_t n, int nlist,
                                                         const int64_t* __restrict__ first_new,
                                                         const int64_t* __restrict__ new_off,
                                                         const int64_t* __restrict__ old_off,
                                                         int64_t* __restrict__ dest) {
  const int64_t p = blockIdx.x * 256ll + threadIdx.x;
  if (p >= n) return;
  const int32_t i = order[p];
  const int32_t l = keys[i];
  if (l < 0 || l >= nlist) return;
  dest[i] = new_off[l] + (old_off[l + 1] - old_off[l]) + (p - first_new[l]);
}

struct PlaceWork {
  int32_t *order_a, *order_b, *mat, *cnt_new;
  int64_t *digit_cnt, *digit_off, *first_new;
  int* bad;
  size_t bytes;
};
PlaceWork carve(char* base, int64_t n, int nlist) {
  PlaceWork w;
  size_t o = 0;
  auto take = [&](size_t b) { const size_t at = o; o += (b + 255) & ~(size_t)255; return base ? base + at : nullptr; };
  w.order_a = reinterpret_cast<int32_t*>(take((size_t)n * sizeof(int32_t)));
  w.order_b = reinterpret_cast<int32_t*>(take((size_t)n * sizeof(int32_t)));
  w.mat = reinterpret_cast<int32_t*>(take((size_t)kMaxChunks * kBuckets * sizeof(int32_t)));
  w.cnt_new = reinterpret_cast<int32_t*>(take(((size_t)nlist + 1) * sizeof(int32_t)));
  w.digit_cnt = reinterpret_cast<int64_t*>(take((size_t)kBuckets * sizeof(int64_t)));
  w.digit_off = reinterpret_cast<int64_t*>(take((size_t)kBuckets * sizeof(int64_t)));
  w.first_new = reinterpret_cast<int64_t*>(take(((size_t)nlist + 1) * sizeof(int64_t)));
  w.bad = reinterpret_cast<int*>(take(sizeof(int64_t)));
  w.bytes = o;
  return w;
}

}  // namespace

size_t ivf_place_work_bytes(int64_t n, int nlist) { return carve(nullptr, n, nlist).bytes; }

int* launch_ivf_place(const int32_t* list_of, int64_t n, int nlist, const int64_t* old_off, char* work,
                      int64_t* dest, int64_t* new_off, hipStream_t st) {
  const PlaceWork w = carve(work, n, nlist);
  launch_fill_u64(reinterpret_cast<u64*>(w.bad), 1, 0ull, st);
  const int64_t chunk = std::max<int64_t>(1024, ((n + kMaxChunks - 1) / kMaxChunks + 63) / 64 * 64);
  const int nchunk = (int)((n + chunk - 1) / chunk);
  const int32_t* perm = nullptr;
  int32_t* out = w.order_a;
  for (int shift = 0; shift == 0 || (nlist - 1) >> shift != 0; shift += kDigitBits) {
    hipLaunchKernelGGL(place_hist_kernel, dim3((unsigned)nchunk), dim3(256), 0, st, list_of, perm, n, nlist, shift,
                       chunk, w.mat, w.bad);
    hipLaunchKernelGGL(place_colscan_kernel, dim3(kBuckets / 256), dim3(256), 0, st, w.mat, nchunk, w.digit_cnt);
    hipLaunchKernelGGL(place_digit_offsets_kernel, dim3(1), dim3(256), 0, st, w.digit_cnt, w.digit_off);
    hipLaunchKernelGGL(place_scatter_kernel, dim3((unsigned)nchunk), dim3(64), 0, st, list_of, perm, n, nlist, shift,
                       chunk, w.mat, w.digit_off, out);
    perm = out;
    out = out == w.order_a ? w.order_b : w.order_a;
  }
  hipLaunchKernelGGL(place_zero_kernel, dim3((unsigned)((nlist + 255) / 256)), dim3(256), 0, st, w.cnt_new,
                     (int64_t)nlist);
  hipLaunchKernelGGL(place_count_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, list_of, n, nlist,
                     w.cnt_new);
  hipLaunchKernelGGL(place_list_offsets_kernel, dim3(1), dim3(1024), 0, st, w.cnt_new, old_off, nlist, w.first_new,
                     new_off);
  hipLaunchKernelGGL(place_dest_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, perm, list_of, n, nlist,
                     w.first_new, new_off, old_off, dest);
  return w.bad;
}
