// IVF-Flat: inverted lists that store the vectors themselves (Sec. 5.1 "Inverted files";
// App. A.3 "GPU Faiss" lists it among the GPU indexes).  The coarse quantizer, the probe
// splits, the k-selection and the merge are the IVF-PQ ones; the scan computes the canon
// fp32 distance between the query and every stored vector of the probed lists -- the same
// chain as the flat search, so a vector's value here equals its value there bit for bit.
// The lists are streamed once: rows [ntotal, d] fp32, list-contiguous; the kernel is bound
// by that stream (d * 4 bytes per visited vector).
#include <algorithm>

#include "common.hpp"
#include "internal.hpp"

namespace {

// storage of a grown index: old entries keep their order inside their list, new entries
// follow them at dest[i]; one lane per fp32 element, grid-stride (a launch cannot hold more
// than 2^32 - 1 work-items and 100M rows of 96 floats are 9.6e9 elements)
__global__ void flat_move_old_kernel(const float* __restrict__ old_rows,
                                     const int64_t* __restrict__ old_ids, int64_t old_total, int d,
                                     const int64_t* __restrict__ old_off,
                                     const int64_t* __restrict__ new_off, int nlist,
                                     float* __restrict__ rows, int64_t* __restrict__ ids) {
  const int64_t total = old_total * d, stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; e < total; e += stride) {
    const int64_t p = e / d;
    const int t = (int)(e - p * d);
    const int l = list_of_position(old_off, nlist, p);
    const int64_t np = new_off[l] + (p - old_off[l]);
    rows[np * d + t] = old_rows[e];
    if (t == 0) ids[np] = old_ids[p];
  }
}

__global__ void flat_scatter_new_kernel(const float* __restrict__ x,
                                        const int64_t* __restrict__ new_ids, int64_t id_base,
                                        const int64_t* __restrict__ dest, int64_t n, int d,
                                        float* __restrict__ rows, int64_t* __restrict__ ids) {
  const int64_t total = n * d, stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; e < total; e += stride) {
    const int64_t i = e / d;
    const int t = (int)(e - i * d);
    const int64_t p = dest[i];
    rows[p * d + t] = x[e];
    if (t == 0) ids[p] = new_ids ? new_ids[i] : id_base + i;
  }
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

// The same scan with the rows staged through LDS, for d a multiple of 32.  Reading one row
// per lane straight from memory makes every load instruction touch 64 cache lines; here a
// tile of 256 rows x 32 dimensions is fetched with 8 lanes per row (128 consecutive bytes of
// a row per request), written to LDS with a row stride of 36 floats (16-byte aligned and
// conflict-free for the 16-byte reads that follow), and lane r then continues the canon
// chain of row r over those 32 dimensions.  The next tile chunk is in flight (registers)
// while the current one is summed; one LDS barrier per chunk.
template <int R, int METRIC>
__global__ __launch_bounds__(256) void ivfflat_scan_tiled_kernel(
    const float* __restrict__ q, int d, const int32_t* __restrict__ probes, int nprobe, int ppb,
    int nsplit, const int64_t* __restrict__ list_off, const float* __restrict__ rows, int k, int tot,
    KeySink sink) {
  constexpr int DC = 32, LD = 36, TR = 256;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  u64* slots = reinterpret_cast<u64*>(smem);                    // 4 * tot
  u64* bound = slots + 4 * tot;                                 // workgroup bound (+ pad)
  float* qs = reinterpret_cast<float*>(bound + 2);              // d
  float* tile = qs + d;                                         // 2 x TR x LD
  const int64_t qi = blockIdx.x / nsplit;
  const int split = blockIdx.x % nsplit;
  const int tid = threadIdx.x, wave = tid >> 6;
  const int p_end = min(nprobe, split * ppb + ppb);
  const int r_ld = tid >> 3, c_ld = tid & 7;                    // fetch: 8 lanes per row, 32 rows per pass

  for (int t = tid; t < d; t += 256) qs[t] = q[qi * d + t];
  if (tid == 0) *bound = KEY_EMPTY;
  WaveSelect<R> ws;
  ws.init(slots + wave * tot, tot, k, bound);

  // position in the sequence of (list, tile of 256 rows, chunk of 32 dimensions): all uniform
  struct Pos { int p; int64_t i0, end; int c0; bool ok; };
  auto first_row_from = [&](int p) {                            // first non-empty list at or after p
    Pos s{p, 0, 0, 0, false};
    for (; s.p < p_end; ++s.p) {
      const int l = probes[qi * nprobe + s.p];
      if (l < 0) continue;
      s.i0 = list_off[l]; s.end = list_off[l + 1];
      if (s.i0 < s.end) { s.ok = true; break; }
    }
    return s;
  };
  auto next_of = [&](const Pos& c) {
    Pos n = c;
    n.c0 += DC;
    if (n.c0 < d) return n;
    n.c0 = 0;
    n.i0 += TR;
    if (n.i0 < n.end) return n;
    return first_row_from(c.p + 1);
  };
  u32x4 stg[8];   // (an ext-vector type: HIP's float4 arrays end up in scratch memory)
#define FETCH(S)                                                                                  \
  do {                                                                                            \
    _Pragma("unroll") for (int j_ = 0; j_ < 8; ++j_) {                                            \
      const int64_t row_ = min((S).i0 + j_ * 32 + r_ld, (S).end - 1);   /* rows past the end: masked later */ \
      stg[j_] = *reinterpret_cast<const u32x4*>(rows + row_ * d + (S).c0 + c_ld * 4);            \
    }                                                                                             \
  } while (0)
#define STASH(BUF)                                                                                \
  do {                                                                                            \
    _Pragma("unroll") for (int j_ = 0; j_ < 8; ++j_)                                              \
      *reinterpret_cast<u32x4*>(tile + ((BUF) * TR + j_ * 32 + r_ld) * LD + c_ld * 4) = stg[j_]; \
  } while (0)

  Pos cur = first_row_from(split * ppb);
  if (cur.ok) { FETCH(cur); STASH(0); }
  __syncthreads();                                              // query, bound and the first chunk
  int buf = 0;
  float acc = 0.f;
  while (cur.ok) {
    const Pos nxt = next_of(cur);
    if (nxt.ok) FETCH(nxt);                                     // in flight during the arithmetic
    const float* __restrict__ tr = tile + (buf * TR + tid) * LD;
    const float* __restrict__ qc = qs + cur.c0;
#pragma unroll
    for (int c = 0; c < DC / 4; ++c) {
      const float4 xv = *reinterpret_cast<const float4*>(tr + c * 4);
      const float4 qv = *reinterpret_cast<const float4*>(qc + c * 4);
      const float xs[4] = {xv.x, xv.y, xv.z, xv.w}, qq[4] = {qv.x, qv.y, qv.z, qv.w};
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (METRIC == 0) { const float diff = qq[u] - xs[u]; acc = __builtin_fmaf(diff, diff, acc); }
        else acc = __builtin_fmaf(qq[u], xs[u], acc);
      }
    }
    if (cur.c0 + DC >= d) {                                     // the row is complete
      const int64_t i = cur.i0 + tid;
      ws.push(i < cur.end, make_key(acc, (u32)i, METRIC), true);
      acc = 0.f;
    }
    if (nxt.ok) STASH(buf ^ 1);
    block_sync_lds();
    cur = nxt;
    buf ^= 1;
  }
#undef FETCH
#undef STASH
  ws.finish();
  block_sync_lds();
  block_rank_merge(slots, tot, 4, k, sink, ((int64_t)qi * nsplit + split) * k);
}

// ---------------------------------------------------------------------------
// IVF-SQ8: the entries of the lists are 8-bit scalar-quantizer codes of the vectors
// (Sec. 4.1 "Scalar quantizers"; App. A.3 lists the index among the GPU ones).  Component t
// of a vector falls into one of 256 cells of width step[t] starting at vmin[t]; its code is
// the cell number, its reconstruction the middle of the cell: fma(code + 0.5, step, vmin).
// The scan evaluates the distance to the reconstruction from the code bytes directly.
// ---------------------------------------------------------------------------
__global__ void sq8_encode_kernel(const float* __restrict__ x, int64_t n, int d,
                                  const float* __restrict__ vmin, const float* __restrict__ step,
                                  uint8_t* __restrict__ codes) {
  const int64_t total = n * d, stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; e < total; e += stride) {
    const int t = (int)(e % d);
    const float u = (x[e] - vmin[t]) / step[t];
    codes[e] = u < 0.f ? (uint8_t)0 : (u >= 256.f ? (uint8_t)255 : (uint8_t)(int)u);
  }
}

// Per-query terms that fold the reconstruction x'_t = vmin_t + (code + 0.5) step_t into the
// distance chain (same value up to fp32 rounding, 3 resp. 2 vector instructions per component
// instead of 5):  L2: q_t - x'_t = a_t - code * step_t with a_t = q_t - (vmin_t + step_t / 2);
// IP: q_t x'_t = q_t (vmin_t + step_t / 2) + code * b_t with b_t = q_t step_t, the first terms
// summed once per query.  qs: [0, d) a_t or b_t, [d, 2d) step_t (L2 only).
template <int METRIC>
__device__ __forceinline__ float sq8_step(float acc, float ab, float code, float st) {
  if (METRIC == 0) { const float diff = __builtin_fmaf(-code, st, ab); return __builtin_fmaf(diff, diff, acc); }
  return __builtin_fmaf(code, ab, acc);
}

// fills qs for query qi and returns the constant of the inner-product form (0 for L2);
// call with all 256 lanes, followed by a barrier
template <int METRIC>
__device__ __forceinline__ void sq8_query_terms(const float* __restrict__ q, int64_t qi, int d,
                                                const float* __restrict__ vmin,
                                                const float* __restrict__ step, float* qs,
                                                float* ip0) {
  for (int t = threadIdx.x; t < d; t += 256) {
    const float mid = __builtin_fmaf(0.5f, step[t], vmin[t]);
    if (METRIC == 0) { qs[t] = q[qi * d + t] - mid; qs[d + t] = step[t]; }
    else { qs[t] = q[qi * d + t] * step[t]; qs[d + t] = q[qi * d + t] * mid; }
  }
  if (METRIC == 1) {
    __syncthreads();
    if (threadIdx.x == 0) {
      float s0 = 0.f;
      for (int t = 0; t < d; ++t) s0 += qs[d + t];
      *ip0 = s0;
    }
  }
}

// any d: one stored code per lane, read straight from memory
template <int R, int METRIC>
__global__ __launch_bounds__(256) void ivfsq8_scan_kernel(
    const float* __restrict__ q, int d, const float* __restrict__ vmin, const float* __restrict__ step,
    const int32_t* __restrict__ probes, int nprobe, int ppb, int nsplit,
    const int64_t* __restrict__ list_off, const uint8_t* __restrict__ codes, int k, int tot,
    KeySink sink) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  u64* slots = reinterpret_cast<u64*>(smem);
  u64* bound = slots + 4 * tot;
  float* qs = reinterpret_cast<float*>(bound + 2);              // per-query terms, 2 d floats (+ 1)
  const int64_t qi = blockIdx.x / nsplit;
  const int split = blockIdx.x % nsplit;
  const int wave = threadIdx.x >> 6;
  const int p_end = min(nprobe, split * ppb + ppb);
  sq8_query_terms<METRIC>(q, qi, d, vmin, step, qs, qs + 2 * d);
  if (threadIdx.x == 0) *bound = KEY_EMPTY;
  WaveSelect<R> ws;
  ws.init(slots + wave * tot, tot, k, bound);
  __syncthreads();
  const float acc0 = METRIC == 1 ? qs[2 * d] : 0.f;
  for (int p = split * ppb; p < p_end; ++p) {
    const int l = probes[qi * nprobe + p];
    if (l < 0) continue;
    const int64_t begin = list_off[l], end = list_off[l + 1];
    for (int64_t i0 = begin; i0 < end; i0 += 256) {
      const int64_t i = i0 + threadIdx.x;
      const bool valid = i < end;
      float acc = acc0;
      if (valid) {
        const uint8_t* __restrict__ c = codes + i * d;
        for (int t = 0; t < d; ++t) acc = sq8_step<METRIC>(acc, qs[t], (float)c[t], qs[d + t]);
      }
      ws.push(valid, make_key(acc, (u32)i, METRIC), true);
    }
  }
  ws.finish();
  __syncthreads();
  block_rank_merge(slots, tot, 4, k, sink, ((int64_t)qi * nsplit + split) * k);
}

// d a multiple of DC (64 or 32): tiles of 256 codes x DC components staged through LDS with
// DC / 16 lanes per code (runs of DC consecutive bytes per request), rows padded by 16 bytes
// (conflict-free 16-byte reads); structure as ivfflat_scan_tiled_kernel.
template <int R, int METRIC, int DC>
__global__ __launch_bounds__(256) void ivfsq8_scan_tiled_kernel(
    const float* __restrict__ q, int d, const float* __restrict__ vmin, const float* __restrict__ step,
    const int32_t* __restrict__ probes, int nprobe, int ppb, int nsplit,
    const int64_t* __restrict__ list_off, const uint8_t* __restrict__ codes, int k, int tot,
    KeySink sink) {
  constexpr int LDB = DC + 16, TR = 256, LPR = DC / 16, NPASS = TR * LPR / 256;   // lanes per row, passes
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  u64* slots = reinterpret_cast<u64*>(smem);
  u64* bound = slots + 4 * tot;
  float* qs = reinterpret_cast<float*>(bound + 2);              // per-query terms, 2 d floats (+ 4)
  unsigned char* tile = reinterpret_cast<unsigned char*>(qs + 2 * d + 4);   // 2 x TR x LDB bytes
  const int64_t qi = blockIdx.x / nsplit;
  const int split = blockIdx.x % nsplit;
  const int tid = threadIdx.x, wave = tid >> 6;
  const int p_end = min(nprobe, split * ppb + ppb);
  const int r_ld = tid / LPR, c_ld = tid % LPR;

  sq8_query_terms<METRIC>(q, qi, d, vmin, step, qs, qs + 2 * d);
  if (tid == 0) *bound = KEY_EMPTY;
  WaveSelect<R> ws;
  ws.init(slots + wave * tot, tot, k, bound);

  struct Pos { int p; int64_t i0, end; int c0; bool ok; };
  auto first_row_from = [&](int p) {
    Pos s{p, 0, 0, 0, false};
    for (; s.p < p_end; ++s.p) {
      const int l = probes[qi * nprobe + s.p];
      if (l < 0) continue;
      s.i0 = list_off[l]; s.end = list_off[l + 1];
      if (s.i0 < s.end) { s.ok = true; break; }
    }
    return s;
  };
  auto next_of = [&](const Pos& c) {
    Pos n = c;
    n.c0 += DC;
    if (n.c0 < d) return n;
    n.c0 = 0;
    n.i0 += TR;
    if (n.i0 < n.end) return n;
    return first_row_from(c.p + 1);
  };
  u32x4 stg[NPASS];
#define FETCH(S)                                                                                  \
  do {                                                                                            \
    _Pragma("unroll") for (int j_ = 0; j_ < NPASS; ++j_) {                                        \
      const int64_t row_ = min((S).i0 + j_ * (256 / LPR) + r_ld, (S).end - 1);                    \
      stg[j_] = *reinterpret_cast<const u32x4*>(codes + row_ * d + (S).c0 + c_ld * 16);           \
    }                                                                                             \
  } while (0)
#define STASH(BUF)                                                                                \
  do {                                                                                            \
    _Pragma("unroll") for (int j_ = 0; j_ < NPASS; ++j_)                                          \
      *reinterpret_cast<u32x4*>(tile + ((BUF) * TR + j_ * (256 / LPR) + r_ld) * LDB + c_ld * 16) = stg[j_]; \
  } while (0)

  Pos cur = first_row_from(split * ppb);
  if (cur.ok) { FETCH(cur); STASH(0); }
  __syncthreads();
  const float acc0 = METRIC == 1 ? qs[2 * d] : 0.f;
  int buf = 0;
  float acc = acc0;
  while (cur.ok) {
    const Pos nxt = next_of(cur);
    if (nxt.ok) FETCH(nxt);
    const unsigned char* __restrict__ tr = tile + (buf * TR + tid) * LDB;
    const float* __restrict__ qc = qs + cur.c0;
#pragma unroll
    for (int c = 0; c < DC / 16; ++c) {
      const u32x4 w = *reinterpret_cast<const u32x4*>(tr + c * 16);
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float4 ab = *reinterpret_cast<const float4*>(qc + c * 16 + g * 4);
        float4 st = ab;
        if (METRIC == 0) st = *reinterpret_cast<const float4*>(qc + d + c * 16 + g * 4);
        const u32 word = w[g];
        acc = sq8_step<METRIC>(acc, ab.x, (float)(word & 0xFFu), st.x);
        acc = sq8_step<METRIC>(acc, ab.y, (float)((word >> 8) & 0xFFu), st.y);
        acc = sq8_step<METRIC>(acc, ab.z, (float)((word >> 16) & 0xFFu), st.z);
        acc = sq8_step<METRIC>(acc, ab.w, (float)(word >> 24), st.w);
      }
    }
    if (cur.c0 + DC >= d) {
      const int64_t i = cur.i0 + tid;
      ws.push(i < cur.end, make_key(acc, (u32)i, METRIC), true);
      acc = acc0;
    }
    if (nxt.ok) STASH(buf ^ 1);
    block_sync_lds();
    cur = nxt;
    buf ^= 1;
  }
#undef FETCH
#undef STASH
  ws.finish();
  block_sync_lds();
  block_rank_merge(slots, tot, 4, k, sink, ((int64_t)qi * nsplit + split) * k);
}

}  // namespace

void launch_ivfflat_relayout(int d, int nlist, const float* old_rows, const int64_t* old_ids,
                             int64_t old_total, const int64_t* old_off, const int64_t* new_off,
                             const float* x, const int64_t* new_ids_or_null, int64_t id_base,
                             const int64_t* dest, int64_t n_new, float* rows, int64_t* ids,
                             hipStream_t st) {
  constexpr int64_t kMaxBlocks = 1 << 22;   // 2^30 work-items per launch; the kernels stride
  if (old_total > 0)
    hipLaunchKernelGGL(flat_move_old_kernel,
                       dim3((unsigned)std::min(kMaxBlocks, (old_total * d + 255) / 256)), dim3(256), 0,
                       st, old_rows, old_ids, old_total, d, old_off, new_off, nlist, rows, ids);
  if (n_new > 0)
    hipLaunchKernelGGL(flat_scatter_new_kernel,
                       dim3((unsigned)std::min(kMaxBlocks, (n_new * d + 255) / 256)), dim3(256), 0,
                       st, x, new_ids_or_null, id_base, dest, n_new, d, rows, ids);
}

// d a multiple of 32 takes the tiled kernel (two tile buffers of 256 x 36 floats on top)
size_t ivfflat_scan_lds_bytes(int d, int k) {
  const size_t base = (size_t)(4 * select_slots_for_k(k) + 2) * sizeof(u64) + (size_t)d * sizeof(float);
  return d % 32 == 0 ? base + (size_t)2 * 256 * 36 * sizeof(float) : base;
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
    auto kern = d % 32 == 0 ? &ivfflat_scan_tiled_kernel<RR, MET> : &ivfflat_scan_kernel<RR, MET>; \
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

void launch_sq8_encode(const float* x, int64_t n, int d, const float* vmin, const float* step,
                       uint8_t* codes, hipStream_t st) {
  if (n <= 0) return;
  hipLaunchKernelGGL(sq8_encode_kernel, dim3((unsigned)std::min<int64_t>(1 << 22, (n * d + 255) / 256)),
                     dim3(256), 0, st, x, n, d, vmin, step, codes);
}

static int sq8_chunk(int d) { return d % 64 == 0 ? 64 : (d % 32 == 0 ? 32 : 0); }

size_t ivfsq8_scan_lds_bytes(int d, int k) {
  const size_t base = (size_t)(4 * select_slots_for_k(k) + 2) * sizeof(u64) + ((size_t)2 * d + 4) * sizeof(float);
  const int dc = sq8_chunk(d);
  return dc ? base + (size_t)2 * 256 * (dc + 16) : base;
}

void launch_ivfsq8_scan(int d, int metric, const float* q, int64_t nq, const float* vmin,
                        const float* step, const int32_t* probes, int nprobe, int nsplit,
                        const int64_t* list_off, const uint8_t* codes, int k, u64* partial,
                        const int64_t* ids, float* out_dist, int64_t* out_ids, hipStream_t st) {
  if (nq <= 0) return;
  KeySink sink;
  sink.metric = metric;
  sink.idx32 = nullptr;
  if (nsplit == 1) { sink.keys = nullptr; sink.val = out_dist; sink.id64 = out_ids; sink.idmap = ids; }
  else             { sink.keys = partial; sink.val = nullptr; sink.id64 = nullptr; sink.idmap = nullptr; }
  const int ppb = (nprobe + nsplit - 1) / nsplit;
  const int tot = select_slots_for_k(k);
  const size_t shmem = ivfsq8_scan_lds_bytes(d, k);
  const int dc = sq8_chunk(d);
  const dim3 grid((unsigned)(nq * nsplit)), block(256);
#define GO(RR, MET)                                                                              \
  do {                                                                                           \
    auto kern = dc == 64 ? &ivfsq8_scan_tiled_kernel<RR, MET, 64>                                \
                         : (dc == 32 ? &ivfsq8_scan_tiled_kernel<RR, MET, 32> : &ivfsq8_scan_kernel<RR, MET>); \
    if (shmem > 48 * 1024)                                                                       \
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                             \
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);         \
    hipLaunchKernelGGL(kern, grid, block, shmem, st, q, d, vmin, step, probes, nprobe, ppb, nsplit, \
                       list_off, codes, k, tot, sink);                                           \
  } while (0)
  switch (select_regs_for_slots(tot)) {
    case 2: if (metric == 0) GO(2, 0); else GO(2, 1); break;
    case 4: if (metric == 0) GO(4, 0); else GO(4, 1); break;
    default: if (metric == 0) GO(0, 0); else GO(0, 1); break;
  }
#undef GO
}
