// IVF-Flat: inverted lists that store the vectors themselves (Sec. 5.1 "Inverted files";
// App. A.3 "GPU Faiss" lists it among the GPU indexes).  The coarse quantizer, the probe
// splits, the k-selection and the merge are the IVF-PQ ones; the scan computes the canon
// fp32 distance between the query and every stored vector of the probed lists -- the same
// chain as the flat search, so a vector's value here equals its value there bit for bit.
// The lists are streamed once: rows [ntotal, d] fp32, list-contiguous; the kernel is bound
// by that stream (d * 4 bytes per visited vector).
#include "common.hpp"
#include "internal.hpp"

namespace {

// storage of a grown index: old entries keep their order inside their list, new entries
// follow them at dest[i]; one lane per fp32 element
__global__ void flat_move_old_kernel(const float* __restrict__ old_rows,
                                     const int64_t* __restrict__ old_ids, int64_t old_total, int d,
                                     const int64_t* __restrict__ old_off,
                                     const int64_t* __restrict__ new_off, int nlist,
                                     float* __restrict__ rows, int64_t* __restrict__ ids) {
  const int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (e >= old_total * d) return;
  const int64_t p = e / d;
  const int t = (int)(e - p * d);
  const int l = list_of_position(old_off, nlist, p);
  const int64_t np = new_off[l] + (p - old_off[l]);
  rows[np * d + t] = old_rows[e];
  if (t == 0) ids[np] = old_ids[p];
}

__global__ void flat_scatter_new_kernel(const float* __restrict__ x,
                                        const int64_t* __restrict__ new_ids, int64_t id_base,
                                        const int64_t* __restrict__ dest, int64_t n, int d,
                                        float* __restrict__ rows, int64_t* __restrict__ ids) {
  const int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (e >= n * d) return;
  const int64_t i = e / d;
  const int t = (int)(e - i * d);
  const int64_t p = dest[i];
  rows[p * d + t] = x[e];
  if (t == 0) ids[p] = new_ids ? new_ids[i] : id_base + i;
}

// One workgroup (4 wavefronts) per (query, probe split).  The query sits in LDS and is read
// as broadcasts; every lane takes one stored vector at a time and walks it with 16-byte
// loads (a row is a run of consecutive bytes: every fetched sector is used).  Candidates go
// through the wavefront's WaveSelect with a workgroup-shared bound; the four results are
// merged by ranking.
template <int R, int METRIC>
__global__ __launch_bounds__(256) void ivfflat_scan_kernel(
    const float* __restrict__ q, int d, const int32_t* __restrict__ probes, int nprobe, int ppb,
    int nsplit, const int64_t* __restrict__ list_off, const float* __restrict__ rows, int k, int tot,
    KeySink sink) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  u64* slots = reinterpret_cast<u64*>(smem);                    // 4 * tot
  u64* bound = slots + 4 * tot;                                 // workgroup bound (+ pad)
  float* qs = reinterpret_cast<float*>(bound + 2);              // d
  const int64_t qi = blockIdx.x / nsplit;
  const int split = blockIdx.x % nsplit;
  const int wave = threadIdx.x >> 6;
  const int p_begin = split * ppb;
  const int p_end = min(nprobe, p_begin + ppb);
  const bool vec = (d & 3) == 0;

  for (int t = threadIdx.x; t < d; t += 256) qs[t] = q[qi * d + t];
  if (threadIdx.x == 0) *bound = KEY_EMPTY;
  WaveSelect<R> ws;
  ws.init(slots + wave * tot, tot, k, bound);
  __syncthreads();
  for (int p = p_begin; p < p_end; ++p) {
    const int l = probes[qi * nprobe + p];
    if (l < 0) continue;
    const int64_t begin = list_off[l], end = list_off[l + 1];
    for (int64_t i0 = begin; i0 < end; i0 += 256) {              // uniform trip count
      const int64_t i = i0 + threadIdx.x;
      const bool valid = i < end;
      const float val = valid ? canon_row<METRIC>(qs, rows + i * d, d, vec) : 0.f;
      ws.push(valid, make_key(val, (u32)i, METRIC), true);
    }
  }
  ws.finish();
  __syncthreads();
  block_rank_merge(slots, tot, 4, k, sink, ((int64_t)qi * nsplit + split) * k);
}

}  // namespace

void launch_ivfflat_relayout(int d, int nlist, const float* old_rows, const int64_t* old_ids,
                             int64_t old_total, const int64_t* old_off, const int64_t* new_off,
                             const float* x, const int64_t* new_ids_or_null, int64_t id_base,
                             const int64_t* dest, int64_t n_new, float* rows, int64_t* ids,
                             hipStream_t st) {
  if (old_total > 0)
    hipLaunchKernelGGL(flat_move_old_kernel, dim3((unsigned)((old_total * d + 255) / 256)), dim3(256), 0,
                       st, old_rows, old_ids, old_total, d, old_off, new_off, nlist, rows, ids);
  if (n_new > 0)
    hipLaunchKernelGGL(flat_scatter_new_kernel, dim3((unsigned)((n_new * d + 255) / 256)), dim3(256), 0,
                       st, x, new_ids_or_null, id_base, dest, n_new, d, rows, ids);
}

size_t ivfflat_scan_lds_bytes(int d, int k) {
  return (size_t)(4 * select_slots_for_k(k) + 2) * sizeof(u64) + (size_t)d * sizeof(float);
}

void launch_ivfflat_scan(int d, int metric, const float* q, int64_t nq, const int32_t* probes,
                         int nprobe, int nsplit, const int64_t* list_off, const float* rows, int k,
                         u64* partial, const int64_t* ids, float* out_dist, int64_t* out_ids,
                         hipStream_t st) {
  if (nq <= 0) return;
  KeySink sink;
  sink.metric = metric;
  sink.idx32 = nullptr;
  if (nsplit == 1) { sink.keys = nullptr; sink.val = out_dist; sink.id64 = out_ids; sink.idmap = ids; }
  else             { sink.keys = partial; sink.val = nullptr; sink.id64 = nullptr; sink.idmap = nullptr; }
  const int ppb = (nprobe + nsplit - 1) / nsplit;
  const int tot = select_slots_for_k(k);
  const size_t shmem = ivfflat_scan_lds_bytes(d, k);
  const dim3 grid((unsigned)(nq * nsplit)), block(256);
#define GO(RR, MET)                                                                              \
  do {                                                                                           \
    auto kern = &ivfflat_scan_kernel<RR, MET>;                                                   \
    if (shmem > 48 * 1024)                                                                       \
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                             \
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);         \
    hipLaunchKernelGGL(kern, grid, block, shmem, st, q, d, probes, nprobe, ppb, nsplit, list_off, \
                       rows, k, tot, sink);                                                      \
  } while (0)
  switch (select_regs_for_slots(tot)) {
    case 2: if (metric == 0) GO(2, 0); else GO(2, 1); break;
    case 4: if (metric == 0) GO(4, 0); else GO(4, 1); break;
    default: if (metric == 0) GO(0, 0); else GO(0, 1); break;
  }
#undef GO
}
