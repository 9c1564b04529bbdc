// Exact re-ranking of a shortlist (Sec. 3.5 "Refining"): a first, approximate search
// returns kc candidate ids per query; here the canon fp32 distance between the query and
// each candidate's stored vector is computed and the k best are kept, best first, ties to
// the smaller id.  Reads kc rows of d floats per query, each row by one lane (a row is a
// run of consecutive bytes, so every fetched sector is used), which is all the traffic:
// the kernel is bound by those gathers.
#include "common.hpp"
#include "internal.hpp"

namespace {

// Four wavefronts per workgroup, one query per wavefront; no workgroup-wide barrier.
template <int R, int METRIC>
__global__ __launch_bounds__(256) void refine_kernel(const float* __restrict__ x, int64_t nb,
                                                     const float* __restrict__ q, int64_t nq, int d,
                                                     const int64_t* __restrict__ cand, int kc, int k,
                                                     int tot, float* __restrict__ out_dist,
                                                     int64_t* __restrict__ out_ids) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int wave = threadIdx.x >> 6, lane = lane_id();
  const int64_t qi = blockIdx.x * 4ll + wave;
  if (qi >= nq) return;
  const size_t per_wave = (size_t)tot * sizeof(u64) + (size_t)((d + 3) / 4 * 4) * sizeof(float);
  u64* slots = reinterpret_cast<u64*>(smem + wave * per_wave);
  float* qs = reinterpret_cast<float*>(slots + tot);
  for (int t = lane; t < d; t += VS_WAVE) qs[t] = q[qi * d + t];
  WaveSelect<R> ws;
  ws.init(slots, tot, k);
  wave_lds_sync();
  const bool vec = (d & 3) == 0;
  const int64_t* __restrict__ c = cand + qi * (int64_t)kc;
  for (int j0 = 0; j0 < kc; j0 += VS_WAVE) {
    const int j = j0 + lane;
    const int64_t id = j < kc ? c[j] : -1;
    const bool valid = id >= 0 && id < nb;          // empty slots of the first stage are skipped
    const float val = valid ? canon_row<METRIC>(qs, x + id * d, d, vec) : 0.f;
    ws.push(valid, make_key(val, (u32)id, METRIC));
  }
  ws.finish();
  for (int j = lane; j < k; j += VS_WAVE) {
    const u64 key = ws.s[j];
    const bool empty = key == KEY_EMPTY;
    out_dist[qi * k + j] = empty ? (METRIC ? -__builtin_inff() : __builtin_inff()) : key_value(key, METRIC);
    out_ids[qi * k + j] = empty ? -1 : (int64_t)key_index(key);
  }
}

}  // namespace

size_t refine_lds_bytes(int d, int k) {
  return 4 * ((size_t)select_slots_for_k(k) * sizeof(u64) + (size_t)((d + 3) / 4 * 4) * sizeof(float));
}

void launch_refine(const float* x, int64_t nb, const float* q, int64_t nq, int d, int metric,
                   const int64_t* cand, int kc, int k, float* out_dist, int64_t* out_ids,
                   hipStream_t st) {
  if (nq <= 0) return;
  const int tot = select_slots_for_k(k);
  const size_t shmem = refine_lds_bytes(d, k);
  const dim3 grid((unsigned)((nq + 3) / 4)), block(256);
#define GO(RR, MET)                                                                              \
  do {                                                                                           \
    auto kern = &refine_kernel<RR, MET>;                                                         \
    if (shmem > 48 * 1024)                                                                       \
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                             \
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);         \
    hipLaunchKernelGGL(kern, grid, block, shmem, st, x, nb, q, nq, d, cand, kc, k, tot, out_dist, \
                       out_ids);                                                                 \
  } while (0)
  switch (select_regs_for_slots(tot)) {
    case 2: if (metric == 0) GO(2, 0); else GO(2, 1); break;
    case 4: if (metric == 0) GO(4, 0); else GO(4, 1); break;
    default: if (metric == 0) GO(0, 0); else GO(0, 1); break;
  }
#undef GO
}
