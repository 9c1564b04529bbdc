// MFMA shortlist + exact re-rank for k-nearest rows (coarse quantizer, flat search).
//
// Sec. 3.2 of the paper: with large query batches distances are computed through
// the matrix-multiplication decomposition ||q||^2 + ||x||^2 - 2<q, x>.  Here the
// contraction runs on the gfx950 matrix cores in bf16 (v_mfma_f32_32x32x16_bf16):
// every fp32 operand is split into a bf16 head and a bf16 tail, and
//     <q, x> ~ <qh, xh> + <qh, xl> + <ql, xh>
// (one pass when both operands are exactly representable in bf16).  The result is
// only used to SHORTLIST: the kp > k best rows by approximate value.  The
// shortlisted rows are then re-evaluated with the canon fp32 chain (the arithmetic
// every bit-exact decision of the library is defined in) and the k best of those
// are returned.  A row's answer is provably the canon answer when
//     t' - eps > v_k        (L2; mirrored for the inner product)
// where t' is the kp-th best approximate value (every row outside the shortlist
// is at least that far), v_k the k-th best canon value inside it, and eps a
// bound on |approximate - canon| for that row.  Rows that fail the test are
// recomputed by canon_rows_kernel over all columns, so the output never depends
// on the approximation.
#include <algorithm>

#include "common.hpp"
#include "internal.hpp"

// rows recomputed by the exact fallback since the last read (statistics only)
__device__ unsigned long long g_fallback_total;

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ unsigned short bf16_rn_bits(float f) {
  u32 u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);   // round to nearest even (inputs are finite)
  return (unsigned short)(u >> 16);
}
__device__ __forceinline__ float bf16_bits_to_f32(unsigned short b) {
  return __uint_as_float(((u32)b) << 16);
}

// ---------------------------------------------------------------------------
// Operand preparation: bf16 head / tail planes, fp32 squared norms, and the
// facts needed to bound the approximation error (PrepInfo).
// One lane per 8 consecutive elements (d % 8 == 0), 256 lanes per workgroup,
// RB = 2048 / d ... rows per workgroup; row sums are added in a fixed order.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void prep_kernel(const float* __restrict__ x, int64_t n, int d,
                                                   int rows_per_block,
                                                   unsigned short* __restrict__ hi,
                                                   unsigned short* __restrict__ lo,
                                                   float* __restrict__ norm,
                                                   PrepInfo* __restrict__ info) {
  __shared__ float part[256];
  __shared__ u32 flags[2];
  const int cpr = d / 8;                               // chunks per row
  const int64_t row0 = (int64_t)blockIdx.x * rows_per_block;
  const int tid = threadIdx.x;
  if (tid < 2) flags[tid] = 1u;
  __syncthreads();
  const int r = tid / cpr, c = tid - r * cpr;
  float ss = 0.f;
  bool is_int = true, is_bf16 = true;
  if (r < rows_per_block && row0 + r < n) {
    const int64_t off = (row0 + r) * d + c * 8;
    float v[8];
    const float4 a = *reinterpret_cast<const float4*>(x + off);
    const float4 b = *reinterpret_cast<const float4*>(x + off + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    unsigned short h[8], l[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      h[t] = bf16_rn_bits(v[t]);
      const float rem = v[t] - bf16_bits_to_f32(h[t]);      // exact in fp32
      l[t] = bf16_rn_bits(rem);
      is_bf16 = is_bf16 && rem == 0.f;
      is_int = is_int && v[t] == __builtin_rintf(v[t]);
      ss = __builtin_fmaf(v[t], v[t], ss);
    }
    uint4 hv, lv;
    hv.x = h[0] | ((u32)h[1] << 16); hv.y = h[2] | ((u32)h[3] << 16);
    hv.z = h[4] | ((u32)h[5] << 16); hv.w = h[6] | ((u32)h[7] << 16);
    lv.x = l[0] | ((u32)l[1] << 16); lv.y = l[2] | ((u32)l[3] << 16);
    lv.z = l[4] | ((u32)l[5] << 16); lv.w = l[6] | ((u32)l[7] << 16);
    *reinterpret_cast<uint4*>(hi + off) = hv;
    *reinterpret_cast<uint4*>(lo + off) = lv;
  }
  part[tid] = ss;
  if (!is_int) flags[0] = 0u;
  if (!is_bf16) flags[1] = 0u;
  __syncthreads();
  if (tid < rows_per_block && row0 + tid < n) {
    float s = 0.f;
    for (int j = 0; j < cpr; ++j) s += part[tid * cpr + j];
    norm[row0 + tid] = s;
    atomicMax(&info->max_norm_bits, __float_as_uint(s));    // s >= 0: bit order = value order
  }
  if (tid == 0) {
    if (!flags[0]) atomicAnd(&info->all_int, 0u);
    if (!flags[1]) atomicAnd(&info->all_bf16, 0u);
  }
}

__global__ void prep_info_init_kernel(PrepInfo* info) {
  info->all_int = 1u; info->all_bf16 = 1u; info->max_norm_bits = 0u; info->pad = 0u;
}

// ---------------------------------------------------------------------------
// Approximate kp-best rows of B for each row of A.
// Workgroup = 4 wavefronts = (32 * RB rows of A) x (a range of B rows, 256 per step).
// Each wavefront holds the A fragments of ALL the workgroup's rows in registers
// for the whole kernel and streams its own 64 B rows per step straight from
// memory into MFMA operand registers (no LDS for operands: lane l of a 32x32x16
// tile needs 16 contiguous bytes of row l % 32).  The 32*RB x 256 tile of
// approximate values is staged in LDS; then every wavefront runs the
// threshold-filtered WaveSelect for the rows it owns (one select state per row,
// kept in LDS).  B fragments of the next step are requested right after the
// MFMAs of this step have been issued, so they fly during staging and selection.
// ---------------------------------------------------------------------------
template <int KSTEPS, int RB, int R, int METRIC>
__global__ __launch_bounds__(256)
void mfma_knn_kernel(const unsigned short* __restrict__ Ahi, const unsigned short* __restrict__ Alo,
                     const float* __restrict__ Anorm, const PrepInfo* __restrict__ Ainfo, int64_t na,
                     const unsigned short* __restrict__ Bhi, const unsigned short* __restrict__ Blo,
                     const float* __restrict__ Bnorm, const PrepInfo* __restrict__ Binfo, int64_t nb,
                     int nsplit, int64_t cols_per_split, int kp, int cap,
                     u64* __restrict__ shortlist) {
  constexpr int D = KSTEPS * 16, BM = 32 * RB, LD = 256 + 4, ROWS_PER_WAVE = BM / 4;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float* stage = reinterpret_cast<float*>(smem);                       // BM x LD
  u64* slots = reinterpret_cast<u64*>(stage + BM * LD);                // BM x cap
  u64* thr = slots + (size_t)BM * cap;                                 // BM
  int* cnts = reinterpret_cast<int*>(thr + BM);                        // BM

  const int tid = threadIdx.x, wave = tid >> 6, lane = lane_id();
  const int64_t rt = blockIdx.x / nsplit;
  const int split = blockIdx.x % nsplit;
  const int64_t row0 = rt * BM;
  const int64_t c_begin = (int64_t)split * cols_per_split;
  const int64_t c_end = min(nb, c_begin + cols_per_split);
  const bool three = !(Ainfo->all_bf16 && Binfo->all_bf16);            // uniform

  // A fragments: lane holds row (l % 32) of each 32-row block, dims 8 * (l / 32) .. + 7 of each k-step
  bf16x8 ah[RB][KSTEPS], al[RB][KSTEPS];
  float an[RB][16];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int64_t ar = min(row0 + rb * 32 + (lane & 31), na - 1);
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk) {
      const int64_t off = ar * D + kk * 16 + 8 * (lane >> 5);
      ah[rb][kk] = *reinterpret_cast<const bf16x8*>(Ahi + off);
      al[rb][kk] = *reinterpret_cast<const bf16x8*>(Alo + off);
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int64_t r = min(row0 + rb * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3), na - 1);
      an[rb][v] = METRIC == 0 ? Anorm[r] : 0.f;
    }
  }
  for (int i = tid; i < BM; i += 256) { thr[i] = KEY_EMPTY; cnts[i] = 0; }
  for (int i = tid; i < BM * kp; i += 256) slots[(size_t)(i / kp) * cap + (i % kp)] = KEY_EMPTY;
  block_sync_lds();

  bf16x8 bh[2][KSTEPS], bl[2][KSTEPS];
  float bn[2];
  auto load_b = [&](int64_t ct) {
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
      const int64_t col = min(ct + wave * 64 + cb * 32 + (lane & 31), nb - 1);
#pragma unroll
      for (int kk = 0; kk < KSTEPS; ++kk) {
        const int64_t off = col * D + kk * 16 + 8 * (lane >> 5);
        bh[cb][kk] = *reinterpret_cast<const bf16x8*>(Bhi + off);
        if (three) bl[cb][kk] = *reinterpret_cast<const bf16x8*>(Blo + off);
      }
      bn[cb] = METRIC == 0 ? Bnorm[col] : 0.f;
    }
  };
  if (c_begin < c_end) load_b(c_begin);

  for (int64_t ct = c_begin; ct < c_end; ct += 256) {
    floatx16 acc[RB][2];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[rb][cb][v] = 0.f;
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk)
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
          acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[rb][kk], bh[cb][kk], acc[rb][cb], 0, 0, 0);
    if (three) {
#pragma unroll
      for (int kk = 0; kk < KSTEPS; ++kk)
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
          for (int cb = 0; cb < 2; ++cb) {
            acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[rb][kk], bl[cb][kk], acc[rb][cb], 0, 0, 0);
            acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[rb][kk], bh[cb][kk], acc[rb][cb], 0, 0, 0);
          }
    }
    const float bn0 = bn[0], bn1 = bn[1];
    if (ct + 256 < c_end) load_b(ct + 256);     // in flight during staging and selection

    // stage the tile: value (row i, col j) at stage[i][j]
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int i = rb * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
          const int j = wave * 64 + cb * 32 + (lane & 31);
          float val = acc[rb][cb][v];
          if (METRIC == 0) val = (an[rb][v] + (cb ? bn1 : bn0)) - 2.f * val;
          stage[i * LD + j] = val;
        }
    block_sync_lds();

    // selection: this wavefront owns rows wave * ROWS_PER_WAVE ..
    for (int rr = 0; rr < ROWS_PER_WAVE; ++rr) {
      const int i = wave * ROWS_PER_WAVE + rr;
      const u64 th = thr[i];
      u64 key[4];
      bool any = false;
#pragma unroll
      for (int c4 = 0; c4 < 4; ++c4) {
        const int64_t col = ct + c4 * 64 + lane;
        key[c4] = col < c_end ? make_key(stage[i * LD + c4 * 64 + lane], (u32)col, METRIC) : KEY_EMPTY;
        any = any || key[c4] < th;
      }
      if (__ballot(any) == 0) continue;          // nothing in this row beats its kp-th best
      WaveSelect<R> ws;
      ws.attach(slots + (size_t)i * cap, cap, kp, cnts[i], th);
#pragma unroll
      for (int c4 = 0; c4 < 4; ++c4) ws.push(key[c4] != KEY_EMPTY, key[c4]);
      if (lane == 0) { cnts[i] = ws.cnt; thr[i] = ws.thresh; }
    }
    block_sync_lds();
  }

  // flush: sorted kp best per owned row
  for (int rr = 0; rr < ROWS_PER_WAVE; ++rr) {
    const int i = wave * ROWS_PER_WAVE + rr;
    WaveSelect<R> ws;
    ws.attach(slots + (size_t)i * cap, cap, kp, cnts[i], thr[i]);
    ws.finish();
    if (row0 + i < na) {
      u64* out = shortlist + ((row0 + i) * nsplit + split) * (int64_t)kp;
      for (int j = lane; j < kp; j += VS_WAVE) out[j] = ws.s[j];
    }
  }
}

// ---------------------------------------------------------------------------
// Exact re-rank: one wavefront per row of A.
// ---------------------------------------------------------------------------
template <int METRIC>
__device__ __forceinline__ float canon_row(const float* __restrict__ qs, const float* __restrict__ b,
                                           int d, bool vec) {
  float acc = 0.f;
  if (vec) {
    for (int t = 0; t < d; t += 4) {
      const float4 bv = *reinterpret_cast<const float4*>(b + t);
      const float bb[4] = {bv.x, bv.y, bv.z, bv.w};
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (METRIC == 0) { const float diff = qs[t + u] - bb[u]; acc = __builtin_fmaf(diff, diff, acc); }
        else acc = __builtin_fmaf(qs[t + u], bb[u], acc);
      }
    }
  } else {
    for (int t = 0; t < d; ++t) {
      if (METRIC == 0) { const float diff = qs[t] - b[t]; acc = __builtin_fmaf(diff, diff, acc); }
      else acc = __builtin_fmaf(qs[t], b[t], acc);
    }
  }
  return acc;
}

template <int R, int METRIC>
__global__ __launch_bounds__(64) void rerank_kernel(
    const u64* __restrict__ shortlist, int nsplit, int kp, const float* __restrict__ A,
    const float* __restrict__ B, int d, int k, const float* __restrict__ Anorm,
    const PrepInfo* __restrict__ Ainfo, const PrepInfo* __restrict__ Binfo, float eps_scale,
    SelectOut out, int* __restrict__ fb_count, int* __restrict__ fb_rows) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  u64* slots = reinterpret_cast<u64*>(smem);                    // 64 * R
  float* qs = reinterpret_cast<float*>(slots + 64 * R);         // d
  const int64_t row = blockIdx.x;
  const int lane = lane_id();
  const bool vec = (d & 3) == 0;
  for (int t = lane; t < d; t += VS_WAVE) qs[t] = A[row * d + t];

  // global kp best approximate keys of this row
  WaveSelect<R> ws;
  ws.init(slots, 64 * R, kp);
  const u64* __restrict__ src = shortlist + row * (int64_t)nsplit * kp;
  const int n = nsplit * kp;
  for (int j0 = 0; j0 < n; j0 += VS_WAVE) {
    const int j = j0 + lane;
    const u64 key = j < n ? src[j] : KEY_EMPTY;
    ws.push(j < n && key != KEY_EMPTY, key);
  }
  ws.finish();
  const u64 tkey = ws.s[kp - 1];                                // kp-th best approximate key

  // canon value of every shortlisted row, then an exact sort
  u64 v[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int e = lane * R + r;
    const u64 ak = e < kp ? ws.s[e] : KEY_EMPTY;
    if (ak == KEY_EMPTY) { v[r] = KEY_EMPTY; continue; }
    const u32 idx = key_index(ak);
    v[r] = make_key(canon_row<METRIC>(qs, B + (int64_t)idx * d, d, vec), idx, METRIC);
  }
  wave_sort_regs<R>(v);
  wave_lds_sync();
#pragma unroll
  for (int r = 0; r < R; ++r) slots[lane * R + r] = v[r];
  wave_lds_sync();
  const lds_u64_ptr sorted = to_lds(slots);
  const u64 vk = sorted[k - 1];                                 // k-th best canon key

  // is the shortlist provably sufficient?
  bool ok = true;
  if (tkey != KEY_EMPTY && vk != KEY_EMPTY) {
    const float na2 = Anorm[row], nb2 = __uint_as_float(Binfo->max_norm_bits);
    const bool exact = Ainfo->all_int && Binfo->all_int && Ainfo->all_bf16 && Binfo->all_bf16 &&
                       (__uint_as_float(Ainfo->max_norm_bits) + nb2 < 16777216.f);
    const bool three = !(Ainfo->all_bf16 && Binfo->all_bf16);
    // |approx - canon| <= eps: bf16 head/tail split drops terms below 2^-15 |q||x| per product;
    // fp32 accumulation and the canon chain each stay below d 2^-22 (|q|^2 + |x|^2)
    const float coef = (three ? 6.2e-5f : 0.f) + (float)d * 4.8e-7f;
    const float eps = exact ? 0.f : eps_scale * coef * (na2 + nb2);
    const float tv = key_value(tkey, METRIC), kv = key_value(vk, METRIC);
    ok = METRIC == 0 ? (tv - eps > kv) : (tv + eps < kv);
  } else if (tkey != KEY_EMPTY && vk == KEY_EMPTY) {
    ok = true;   // cannot happen: kp >= k candidates exist
  }
  if (eps_scale < 0.f) ok = false;                              // test hook: force the fallback
  if (!ok && lane == 0) {
    const int f = atomicAdd(fb_count, 1);
    fb_rows[f] = (int)row;
  }
  for (int j = lane; j < k; j += VS_WAVE) {
    const u64 key = sorted[j];
    const bool empty = key == KEY_EMPTY;
    const int64_t at = row * (int64_t)k + j;
    if (out.val) out.val[at] = empty ? (METRIC ? -__builtin_inff() : __builtin_inff()) : key_value(key, METRIC);
    if (out.id64) out.id64[at] = empty ? -1 : (int64_t)key_index(key);
    if (out.idx32) out.idx32[at] = empty ? -1 : (int32_t)key_index(key);
  }
}

// Canon over ALL columns for the rows listed in fb_rows (persistent workgroups).
template <int R, int METRIC>
__global__ __launch_bounds__(256) void canon_rows_kernel(const float* __restrict__ A,
                                                         const float* __restrict__ B, int64_t nb,
                                                         int d, int k, int tot, SelectOut out,
                                                         const int* __restrict__ fb_count,
                                                         const int* __restrict__ fb_rows) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  u64* slots = reinterpret_cast<u64*>(smem);                    // 4 * tot
  float* qs = reinterpret_cast<float*>(slots + 4 * tot);        // d
  const int wave = threadIdx.x >> 6;
  const bool vec = (d & 3) == 0;
  const int count = *fb_count;
  if (blockIdx.x == 0 && threadIdx.x == 0 && count > 0)
    atomicAdd(&g_fallback_total, (unsigned long long)count);
  for (int f = blockIdx.x; f < count; f += gridDim.x) {
    const int64_t row = fb_rows[f];
    __syncthreads();
    for (int t = threadIdx.x; t < d; t += 256) qs[t] = A[row * d + t];
    WaveSelect<R> ws;
    ws.init(slots + wave * tot, tot, k);
    __syncthreads();
    for (int64_t c0 = 0; c0 < nb; c0 += 256) {
      const int64_t c = c0 + threadIdx.x;
      const bool valid = c < nb;
      const float val = valid ? canon_row<METRIC>(qs, B + c * d, d, vec) : 0.f;
      ws.push(valid, make_key(val, (u32)c, METRIC));
    }
    ws.finish();
    __syncthreads();
    KeySink sink;
    sink.keys = nullptr; sink.val = out.val; sink.id64 = out.id64; sink.idx32 = out.idx32;
    sink.idmap = nullptr; sink.metric = METRIC;
    block_rank_merge(slots, tot, 4, k, sink, row * (int64_t)k);
  }
}

__global__ void zero_int_kernel(int* p) { *p = 0; }

}  // namespace

// ------------------------------------------------------------------ launchers

bool mfma_knn_supported(int d, int k) {
  return (d == 32 || d == 64 || d == 96 || d == 128) && k <= 150;
}

int mfma_knn_kp(int k) {
  int kp = k + std::max(16, k / 4);
  kp = (kp + 7) / 8 * 8;
  return std::min(kp, 192);
}

void launch_prep(const float* x, int64_t n, int d, unsigned short* hi, unsigned short* lo,
                 float* norm, PrepInfo* info, hipStream_t st) {
  hipLaunchKernelGGL(prep_info_init_kernel, dim3(1), dim3(1), 0, st, info);
  if (n <= 0) return;
  const int rpb = 2048 / d;                          // d <= 128 here, d % 8 == 0
  hipLaunchKernelGGL(prep_kernel, dim3((unsigned)((n + rpb - 1) / rpb)), dim3(256), 0, st, x, n, d, rpb,
                     hi, lo, norm, info);
}

size_t mfma_knn_shortlist_bytes(int64_t na, int64_t nb, int k, int* nsplit_out) {
  const int kp = mfma_knn_kp(k);
  const int BM = kp <= 64 ? 64 : 32;
  const int64_t row_tiles = (na + BM - 1) / BM;
  const int64_t col_steps = (nb + 255) / 256;
  int64_t nsplit = std::max<int64_t>(1, (768 + row_tiles - 1) / row_tiles);
  nsplit = std::min(nsplit, col_steps);
  nsplit = std::min<int64_t>(nsplit, 64);
  *nsplit_out = (int)nsplit;
  return (size_t)na * nsplit * kp * sizeof(u64);
}

template <int KSTEPS, int RB, int R, int METRIC>
static void launch_mfma_t(const MfmaOperand& A, const MfmaOperand& B, int nsplit, int kp,
                          u64* shortlist, hipStream_t st) {
  constexpr int BM = 32 * RB;
  const int cap = 64 * R;
  const size_t shmem = (size_t)BM * (256 + 4) * sizeof(float) + (size_t)BM * cap * sizeof(u64) +
                       (size_t)BM * (sizeof(u64) + sizeof(int)) + 16;
  auto kern = &mfma_knn_kernel<KSTEPS, RB, R, METRIC>;
  (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
  const int64_t row_tiles = (A.n + BM - 1) / BM;
  const int64_t col_steps = (B.n + 255) / 256;
  const int64_t cols_per_split = (col_steps + nsplit - 1) / nsplit * 256;
  hipLaunchKernelGGL(kern, dim3((unsigned)(row_tiles * nsplit)), dim3(256), shmem, st, A.hi, A.lo,
                     A.norm, A.info, A.n, B.hi, B.lo, B.norm, B.info, B.n, nsplit, cols_per_split, kp,
                     cap, shortlist);
}

template <int KSTEPS, int METRIC>
static void launch_mfma_k(const MfmaOperand& A, const MfmaOperand& B, int nsplit, int kp,
                          u64* shortlist, hipStream_t st) {
  if (kp <= 64) launch_mfma_t<KSTEPS, 2, 2, METRIC>(A, B, nsplit, kp, shortlist, st);
  else          launch_mfma_t<KSTEPS, 1, 4, METRIC>(A, B, nsplit, kp, shortlist, st);
}

void launch_mfma_shortlist(const MfmaOperand& A, const MfmaOperand& B, int d, int metric, int k,
                           int nsplit, u64* shortlist, hipStream_t st) {
  const int kp = mfma_knn_kp(k);
#define GO(KS)                                                                     \
  do {                                                                             \
    if (metric == 0) launch_mfma_k<KS, 0>(A, B, nsplit, kp, shortlist, st);        \
    else             launch_mfma_k<KS, 1>(A, B, nsplit, kp, shortlist, st);        \
  } while (0)
  switch (d / 16) {
    case 2: GO(2); break;
    case 4: GO(4); break;
    case 6: GO(6); break;
    default: GO(8); break;
  }
#undef GO
}

void launch_rerank(const MfmaOperand& A, const MfmaOperand& B, int d, int metric, int k, int nsplit,
                   const u64* shortlist, float eps_scale, const SelectOut& out, int* fb_count,
                   int* fb_rows, hipStream_t st) {
  const int kp = mfma_knn_kp(k);
  hipLaunchKernelGGL(zero_int_kernel, dim3(1), dim3(1), 0, st, fb_count);
  const int R = kp <= 64 ? 2 : 4;
  const size_t sh = (size_t)64 * R * sizeof(u64) + (size_t)d * sizeof(float);
#define RR(RV, MET)                                                                               \
  hipLaunchKernelGGL((rerank_kernel<RV, MET>), dim3((unsigned)A.n), dim3(64), sh, st, shortlist, nsplit, \
                     kp, A.x, B.x, d, k, A.norm, A.info, B.info, eps_scale, out, fb_count, fb_rows)
  if (R == 2) { if (metric == 0) RR(2, 0); else RR(2, 1); }
  else        { if (metric == 0) RR(4, 0); else RR(4, 1); }
#undef RR
  // rows whose shortlist could not be proven sufficient: canon over all columns
  const int tot = select_slots_for_k(k);
  const size_t sh2 = (size_t)4 * tot * sizeof(u64) + (size_t)d * sizeof(float);
  const int grid = (int)std::min<int64_t>(A.n, 1024);
#define CR(RV, MET)                                                                              \
  hipLaunchKernelGGL((canon_rows_kernel<RV, MET>), dim3(grid), dim3(256), sh2, st, A.x, B.x, B.n, d, k, \
                     tot, out, fb_count, fb_rows)
  const int R2 = select_regs_for_slots(tot);
  if (R2 == 2) { if (metric == 0) CR(2, 0); else CR(2, 1); }
  else         { if (metric == 0) CR(4, 0); else CR(4, 1); }
#undef CR
}

int read_fallback_total(unsigned long long* out) {
  unsigned long long zero = 0;
  if (hipMemcpyFromSymbol(out, HIP_SYMBOL(g_fallback_total), sizeof(zero)) != hipSuccess) return -1;
  if (hipMemcpyToSymbol(HIP_SYMBOL(g_fallback_total), &zero, sizeof(zero)) != hipSuccess) return -1;
  return 0;
}
