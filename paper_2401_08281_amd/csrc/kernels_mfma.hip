// MFMA shortlist + exact re-rank for k-nearest rows (coarse quantizer, flat search).
//
// Sec. 3.1 of the paper: with large query batches distances are computed through
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
// where t' is a lower bound on the approximate value of every row that was not
// re-ranked (the listing threshold, or the kp-th best listed value when more than
// kp rows were listed), v_k the k-th best canon value inside the shortlist, and
// eps a bound on |approximate - canon| for that row.  Rows that fail the test are
// recomputed by canon_rows_kernel over all columns, so the output never depends
// on the approximation.
#include <algorithm>
#include <cmath>

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
// fp16 image of a float, round to nearest even, subnormals kept (the matrix cores take them as
// they are)
__device__ __forceinline__ unsigned short f16_rn_bits(float f) {
  return __builtin_bit_cast(unsigned short, (_Float16)f);
}
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
// One matrix product on 16-byte operand fragments that hold eight bf16 or (F16) eight fp16 values.
template <bool F16>
__device__ __forceinline__ floatx16 mfma_32x32x16(bf16x8 a, bf16x8 b, floatx16 c) {
  if constexpr (F16)
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
// Operands whose values fit fp16 (|v| <= sqrt(max |row|^2) <= 2^15): their fp16 heads exist.
__device__ __forceinline__ bool f16_heads_ok(const PrepInfo* a, const PrepInfo* b) {
  return a->max_norm_bits <= 0x4E800000u && b->max_norm_bits <= 0x4E800000u;   // 2^30 as float bits
}
// Which operand-precision variant a call runs (every kernel of the call evaluates this on the
// same flags): 0 one product on the bf16 heads (both operands exactly bf16), 3 one product on the
// fp16 heads (the attempt on an index's own operand, see PrepInfo::heads_only), 1 two products
// (A exactly bf16, long A), 2 three products.
__device__ __forceinline__ int precision_variant(const PrepInfo* a, const PrepInfo* b, int hbit, bool allow_two) {
  const bool ea = a->all_bf16 != 0, eb = b->all_bf16 != 0;
  if (ea && eb) return 0;
  if ((b->heads_only & (u32)hbit) && f16_heads_ok(a, b)) return 3;
  return ea && allow_two ? 1 : 2;
}

// ---------------------------------------------------------------------------
// Operand preparation: bf16 head / tail planes, fp32 squared norms, and the
// facts needed to bound the approximation error (PrepInfo).
// One lane per 8 consecutive elements (d % 8 == 0), 256 lanes per workgroup,
// 2048 / d rows per group; a workgroup walks over groups and reports its flags
// and largest norm once at the end.  Row sums are added in a fixed order.
// The planes are [n_pad][d] row-major.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void prep_kernel(const float* __restrict__ x, int64_t n,
                                                   int64_t n_pad, int d, int rows_per_group,
                                                   unsigned short* __restrict__ hi,
                                                   unsigned short* __restrict__ lo,
                                                   float* __restrict__ norm,
                                                   PrepInfo* __restrict__ info) {
  __shared__ float part[2][256];                       // two buffers: one barrier per group
  __shared__ u32 flags[4];                             // all_int, all_bf16, all_nonneg, largest norm
  const int cpr = d / 8;                               // chunks per row
  const int tid = threadIdx.x;
  if (tid < 3) flags[tid] = 1u;
  if (tid == 3) flags[3] = 0u;
  const int r = tid / cpr, c = tid - r * cpr;
  bool is_int = true, is_bf16 = true, is_nonneg = true;
  u32 max_bits = 0u;
  const int64_t ngroups = (n_pad + rows_per_group - 1) / rows_per_group;
  int pb = 0;
  for (int64_t g = blockIdx.x; g < ngroups; g += gridDim.x, pb ^= 1) {
    const int64_t row0 = g * rows_per_group;
    float ss = 0.f;
    if (r < rows_per_group && row0 + r < n) {
      const int64_t off = (row0 + r) * d + c * 8;
      float v[8];
      const float4 a = *reinterpret_cast<const float4*>(x + off);
      const float4 b = *reinterpret_cast<const float4*>(x + off + 4);
      v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
      unsigned short h[8], l[8], f[8];
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        h[t] = bf16_rn_bits(v[t]);
        const float rem = v[t] - bf16_bits_to_f32(h[t]);      // exact in fp32
        l[t] = bf16_rn_bits(rem);
        f[t] = f16_rn_bits(v[t]);
        is_bf16 = is_bf16 && rem == 0.f;
        is_int = is_int && v[t] == __builtin_rintf(v[t]);
        is_nonneg = is_nonneg && v[t] >= 0.f;
        ss = __builtin_fmaf(v[t], v[t], ss);
      }
      uint4 hv, lv, fv;
      hv.x = h[0] | ((u32)h[1] << 16); hv.y = h[2] | ((u32)h[3] << 16);
      hv.z = h[4] | ((u32)h[5] << 16); hv.w = h[6] | ((u32)h[7] << 16);
      lv.x = l[0] | ((u32)l[1] << 16); lv.y = l[2] | ((u32)l[3] << 16);
      lv.z = l[4] | ((u32)l[5] << 16); lv.w = l[6] | ((u32)l[7] << 16);
      fv.x = f[0] | ((u32)f[1] << 16); fv.y = f[2] | ((u32)f[3] << 16);
      fv.z = f[4] | ((u32)f[5] << 16); fv.w = f[6] | ((u32)f[7] << 16);
      *reinterpret_cast<uint4*>(hi + off) = hv;
      *reinterpret_cast<uint4*>(lo + off) = lv;
      *reinterpret_cast<uint4*>(lo + n_pad * d + off) = fv;   // the fp16 heads: a third plane behind the tails
    } else if (r < rows_per_group && row0 + r < n_pad) {   // padding rows: zeros (never selected)
      const int64_t off = (row0 + r) * d + c * 8;
      const uint4 z = make_uint4(0u, 0u, 0u, 0u);
      *reinterpret_cast<uint4*>(hi + off) = z;
      *reinterpret_cast<uint4*>(lo + off) = z;
      *reinterpret_cast<uint4*>(lo + n_pad * d + off) = z;
    }
    part[pb][tid] = ss;
    // (the buffer written two groups later is safe: every lane passes the next group's
    // barrier only after its reads below)
    __syncthreads();
    if (tid < rows_per_group && row0 + tid < n) {
      float sum = 0.f;
      for (int j = 0; j < cpr; ++j) sum += part[pb][tid * cpr + j];
      norm[row0 + tid] = sum;
      max_bits = max(max_bits, __float_as_uint(sum));        // sum >= 0: bit order = value order
    } else if (tid < rows_per_group && row0 + tid < n_pad) {
      norm[row0 + tid] = 0.f;
    }
  }
  __syncthreads();
  if (!is_int) flags[0] = 0u;
  if (!is_bf16) flags[1] = 0u;
  if (!is_nonneg) flags[2] = 0u;
  if (max_bits) atomicMax(&flags[3], max_bits);
  __syncthreads();
  if (tid == 0) {
    // (a look first: hundreds of workgroups reporting the same fact to one address, one atomic
    // after the other, were most of the time of preparing a batch of queries)
    if (!flags[0] && __atomic_load_n(&info->all_int, __ATOMIC_RELAXED)) atomicAnd(&info->all_int, 0u);
    if (!flags[1] && __atomic_load_n(&info->all_bf16, __ATOMIC_RELAXED)) atomicAnd(&info->all_bf16, 0u);
    if (!flags[2] && __atomic_load_n(&info->all_nonneg, __ATOMIC_RELAXED)) atomicAnd(&info->all_nonneg, 0u);
    if (flags[3] > __atomic_load_n(&info->max_norm_bits, __ATOMIC_RELAXED)) atomicMax(&info->max_norm_bits, flags[3]);
  }
}

// The same preparation for the tiled kernel, which wants the planes as d / 16 panels of
// [n_pad][16]: elements k0 .. k0 + 15 of all rows lie together, so that a block of 32 rows x
// 16 elements -- one MFMA operand -- is 1 KB of consecutive memory.  A workgroup takes 32
// rows at a time: lane (r, s) = (tid % 32, tid / 32) converts chunks s, s + 8, ... of row r,
// so a wavefront writes one whole block (32 rows x 32 bytes, consecutive) per store and
// reads 64-byte runs of 32 rows; the eight partial sums of a row are added in a fixed order.
__global__ __launch_bounds__(256) void prep_panel_kernel(const float* __restrict__ x, int64_t n,
                                                         int64_t n_pad, int d,
                                                         unsigned short* __restrict__ hi,
                                                         unsigned short* __restrict__ lo,
                                                         float* __restrict__ norm,
                                                         PrepInfo* __restrict__ info) {
  __shared__ float part[2][8][32];
  __shared__ u32 flags[4];
  const int cpr = d / 8;
  const int tid = threadIdx.x, r = tid & 31, s = tid >> 5;
  if (tid < 3) flags[tid] = 1u;
  if (tid == 3) flags[3] = 0u;
  bool is_int = true, is_bf16 = true, is_nonneg = true;
  u32 max_bits = 0u;
  const int64_t nblocks = n_pad / 32;
  int pb = 0;
  for (int64_t b = blockIdx.x; b < nblocks; b += gridDim.x, pb ^= 1) {
    const int64_t row = b * 32 + r;
    float ss = 0.f;
    if (row < n) {
#pragma unroll 4
      for (int c = s; c < cpr; c += 8) {
        const int64_t off = row * d + c * 8;
        float v[8];
        const float4 a = *reinterpret_cast<const float4*>(x + off);
        const float4 bq = *reinterpret_cast<const float4*>(x + off + 4);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = bq.x; v[5] = bq.y; v[6] = bq.z; v[7] = bq.w;
        unsigned short h[8], l[8], f[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) {
          h[t] = bf16_rn_bits(v[t]);
          const float rem = v[t] - bf16_bits_to_f32(h[t]);      // exact in fp32
          l[t] = bf16_rn_bits(rem);
          f[t] = f16_rn_bits(v[t]);
          is_bf16 = is_bf16 && rem == 0.f;
          is_int = is_int && v[t] == __builtin_rintf(v[t]);
          is_nonneg = is_nonneg && v[t] >= 0.f;
          ss = __builtin_fmaf(v[t], v[t], ss);
        }
        uint4 hv, lv, fv;
        hv.x = h[0] | ((u32)h[1] << 16); hv.y = h[2] | ((u32)h[3] << 16);
        hv.z = h[4] | ((u32)h[5] << 16); hv.w = h[6] | ((u32)h[7] << 16);
        lv.x = l[0] | ((u32)l[1] << 16); lv.y = l[2] | ((u32)l[3] << 16);
        lv.z = l[4] | ((u32)l[5] << 16); lv.w = l[6] | ((u32)l[7] << 16);
        fv.x = f[0] | ((u32)f[1] << 16); fv.y = f[2] | ((u32)f[3] << 16);
        fv.z = f[4] | ((u32)f[5] << 16); fv.w = f[6] | ((u32)f[7] << 16);
        const int64_t out = ((int64_t)(c >> 1) * n_pad + row) * 16 + (c & 1) * 8;
        *reinterpret_cast<uint4*>(hi + out) = hv;
        *reinterpret_cast<uint4*>(lo + out) = lv;
        *reinterpret_cast<uint4*>(lo + n_pad * d + out) = fv;   // the fp16 heads: a third plane, same panels
      }
    } else {                                               // padding rows: zeros (never selected)
      const uint4 z = make_uint4(0u, 0u, 0u, 0u);
      for (int c = s; c < cpr; c += 8) {
        const int64_t out = ((int64_t)(c >> 1) * n_pad + row) * 16 + (c & 1) * 8;
        *reinterpret_cast<uint4*>(hi + out) = z;
        *reinterpret_cast<uint4*>(lo + out) = z;
        *reinterpret_cast<uint4*>(lo + n_pad * d + out) = z;
      }
    }
    part[pb][s][r] = ss;
    // (the buffer written two blocks later is safe: every lane passes the next block's
    // barrier only after its reads below)
    __syncthreads();
    if (tid < 32) {
      float sum = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) sum += part[pb][j][tid];
      const int64_t rr = b * 32 + tid;
      norm[rr] = rr < n ? sum : 0.f;
      if (rr < n) max_bits = max(max_bits, __float_as_uint(sum));   // sum >= 0: bit order = value order
    }
  }
  __syncthreads();
  if (!is_int) flags[0] = 0u;
  if (!is_bf16) flags[1] = 0u;
  if (!is_nonneg) flags[2] = 0u;
  if (max_bits) atomicMax(&flags[3], max_bits);
  __syncthreads();
  if (tid == 0) {
    // (a look first: hundreds of workgroups reporting the same fact to one address, one atomic
    // after the other, were most of the time of preparing a batch of queries)
    if (!flags[0] && __atomic_load_n(&info->all_int, __ATOMIC_RELAXED)) atomicAnd(&info->all_int, 0u);
    if (!flags[1] && __atomic_load_n(&info->all_bf16, __ATOMIC_RELAXED)) atomicAnd(&info->all_bf16, 0u);
    if (!flags[2] && __atomic_load_n(&info->all_nonneg, __ATOMIC_RELAXED)) atomicAnd(&info->all_nonneg, 0u);
    if (flags[3] > __atomic_load_n(&info->max_norm_bits, __ATOMIC_RELAXED)) atomicMax(&info->max_norm_bits, flags[3]);
  }
}

__global__ void prep_info_init_kernel(PrepInfo* info, u32 heads_only) {
  info->all_int = 1u; info->all_bf16 = 1u; info->max_norm_bits = 0u; info->all_nonneg = 1u;
  info->heads_only = heads_only ? 3u : 0u;
}

// ---------------------------------------------------------------------------
// Shortlist of at least kp approximately-best rows of B for each row of A.
//
// Tiling.  Workgroup = 4 wavefronts; wavefront w owns 32 * RB rows of A whose bf16
// fragments stay in its registers for the whole kernel.  The workgroup walks over a
// range of B in steps of 64 rows; each step's 64 x d bf16 tile is copied once from
// memory into LDS (double buffered, padded rows: conflict-free 128-bit reads) and is
// read by all four wavefronts, so one byte of B feeds 128 * RB rows of A.  Per step a
// wavefront issues 2 * RB * (d / 16) v_mfma_f32_32x32x16_bf16 (x3 when the operands
// need the head/tail split).
//
// Selection uses TWO sweeps over the columns instead of a running top-k, so that the
// inner loops carry no selection state beyond registers:
//   MODE 0 (minima): every accumulator position keeps the minimum of its values
//     m = |x|^2 - 2<q,x> (L2) or m = -<q,x> (IP) over a phase of the sweep and writes
//     it out at the end of the phase: a row gets G group minima, each attained by a
//     different column.  When B is long this sweep computes every S-th row of B only.
//   tau kernel: tau(row) = r-th smallest group minimum, so at least r columns of the
//     row have m <= tau.  With S = 1, r = kp.  With S > 1 the minima describe a 1/S
//     sample of the columns and r is chosen so that about r * S columns, and very
//     probably at least k, lie below tau; nothing is assumed about that number --
//     the re-rank test catches rows with too few or too many.
//   MODE 1 (collect): every tile is computed, with the accumulators started at the row
//     thresholds so that "m <= tau(row)" is a comparison of the finished accumulator with
//     a per-column number; every column that passes is appended to the row's list.  The
//     test is the same inequality as MODE 0's m, evaluated in a different rounding order.
// Every column that is NOT listed has m > tau, which is what the re-rank kernel's
// sufficiency test needs.
// ---------------------------------------------------------------------------
template <int KSTEPS, int RB, int METRIC, int MODE, int PREC>
__global__ __launch_bounds__(256, 2)
void mfma_sweep_kernel(const unsigned short* __restrict__ Ahi, const unsigned short* __restrict__ Alo,
                       const float* __restrict__ Anorm, const PrepInfo* __restrict__ Ainfo, int64_t na,
                       const unsigned short* __restrict__ Bhi, const unsigned short* __restrict__ Blo,
                       const float* __restrict__ Bnorm, const PrepInfo* __restrict__ Binfo, int64_t nb,
                       int nsplit, int64_t cols_per_split, int stride, int nphase,
                       int64_t cols_per_phase,
                       float* __restrict__ minima, int g_raw,       // MODE 0 out: [na][g_raw]
                       const float* __restrict__ tau,               // MODE 1 in:  [na]
                       int* __restrict__ cnt, u64* __restrict__ shortlist, int cap,    // MODE 1 out
                       int allow_two) {
  // PREC: which products the operands need.  0: both are exactly bf16 -- heads only.  1: A is
  // exact, B is not -- A's tails are zero, so head x head + head x tail (two passes; A's tail
  // plane is never read).  2: head x head + head x tail + tail x head (three passes).  3: one
  // product on the fp16 heads, which the host passes in place of the bf16 heads (Ahi, Bhi).
  constexpr bool THREE = PREC == 2, LOB = PREC == 1 || PREC == 2, F16 = PREC == 3;
  constexpr int D = KSTEPS * 16, BN = 64, LDB = D + 8;            // LDS row stride in bf16 elements
  constexpr int NPL = LOB ? 2 : 1;                                // planes of B in LDS
  constexpr int CHUNKS = BN * (D / 8);                            // 16-byte chunks per plane per step
  constexpr int CPT = (CHUNKS + 255) / 256;                       // chunks per lane
  constexpr float SCALE = METRIC == 0 ? -2.f : -1.f;
  // the variants that may be needed are all launched; those that do not match the operands'
  // flags leave at once (the two-pass variant is only enqueued for long A: allow_two)
  // allow_two: bit 0 = the two-pass variant was enqueued; bits 1.. = this call's bit of heads_only
  if (precision_variant(Ainfo, Binfo, allow_two >> 1, (allow_two & 1) != 0) != PREC) return;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned short* bt = reinterpret_cast<unsigned short*>(smem);   // [2 buffers][NPL][BN][LDB]
  float* bns = reinterpret_cast<float*>(bt + 2 * NPL * BN * LDB); // [2][BN] norms (+inf past the end)
  // MODE 1: per-row candidate counters of this workgroup and one candidate queue per wavefront
  int* cnt_s = reinterpret_cast<int*>(bns + 2 * BN);              // [128 * RB]
  u64* qkey = reinterpret_cast<u64*>(cnt_s + 128 * RB) + (threadIdx.x >> 6) * 128;   // [4][128]
  int* qrow = reinterpret_cast<int*>(reinterpret_cast<u64*>(cnt_s + 128 * RB) + 4 * 128) +
              (threadIdx.x >> 6) * 128;                           // [4][128]
  // |q|^2 of the workgroup's rows (L2 values of listed columns are formed from LDS only: a
  // read from memory there would wait behind the tile loads in flight)
  float* an_s = reinterpret_cast<float*>(reinterpret_cast<int*>(reinterpret_cast<u64*>(cnt_s + 128 * RB) +
                                                               4 * 128) + 4 * 128);   // [128 * RB]
  int qn = 0;                                                     // queue fill (wave-uniform)

  const int tid = threadIdx.x, wave = tid >> 6, lane = lane_id();
  // Work item = (split of B, row tile), numbered split first.  Workgroup ids go round the eight
  // XCDs, each with an L2 of its own: XCD x takes a run of consecutive items, so the workgroups
  // resident on it at a time are row tiles that walk through the SAME split of B in step, and a
  // tile of B comes from memory once per XCD instead of once per workgroup.
  const int64_t row_tiles = (na + 128 * RB - 1) / (128 * RB);
  const int64_t items = row_tiles * nsplit, per_xcd = (items + 7) / 8;
  const int64_t item = (int64_t)(blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if ((int64_t)(blockIdx.x >> 3) >= per_xcd || item >= items) return;
  const int split = (int)(item / row_tiles);
  const int64_t rt = item - (int64_t)split * row_tiles;
  const int64_t row0 = rt * (128 * RB) + wave * (32 * RB);        // this wavefront's first row
  const int64_t c_begin = (int64_t)split * cols_per_split;
  const int64_t c_end = min(nb, c_begin + cols_per_split);
  // A step covers 64 * stride rows of B and computes every stride-th of them (stride = 1:
  // all of them).  Rows past the padded end of B are read from its last row and masked.
  const int64_t col_step = (int64_t)BN * stride;
  const int64_t b_last = (nb + 63) / 64 * 64 - 1;

  // A fragments: lane holds row (l % 32) of each 32-row block, dims 8 * (l / 32) .. + 7 of each k-step
  bf16x8 ah[RB][KSTEPS], al[THREE ? RB : 1][THREE ? KSTEPS : 1];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int64_t ar = min(row0 + rb * 32 + (lane & 31), na - 1);
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk) {
      const int64_t off = ar * D + kk * 16 + 8 * (lane >> 5);
      ah[rb][kk] = *reinterpret_cast<const bf16x8*>(Ahi + off);
      if constexpr (THREE) al[rb][kk] = *reinterpret_cast<const bf16x8*>(Alo + off);
    }
  }
  // Per accumulator register: running minimum (MODE 0), or (MODE 1) the threshold in the
  // units of the contraction: m <= tau  <=>  <q,x> + tau / s >= b / s  with s = 2 (L2:
  // m = |x|^2 - 2 <q,x>, b = |x|^2) or s = 1 (IP: m = -<q,x>, b = 0).  The collect sweep
  // starts every accumulator at tau / s instead of 0, so its test is one comparison of the
  // finished accumulator with the column's b / s and costs no arithmetic per element.
  constexpr float INV_S = METRIC == 0 ? 0.5f : 1.f;
  float mn[RB][2][16];
  floatx16 tr[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int64_t r = row0 + rb * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
      // (rows past the end of A start from -inf: nothing of them passes the collect test)
      tr[rb][v] = MODE == 1 ? (r < na ? tau[r] * INV_S : -__builtin_inff()) : 0.f;
#pragma unroll
      for (int cb = 0; cb < 2; ++cb) mn[rb][cb][v] = __builtin_inff();
    }

  // global -> registers -> LDS staging of one 64-row B tile (spelled as macros so that the
  // staging registers stay registers).  B planes are padded to a multiple of 64 rows; tile
  // row r is row CT + r * stride of B.
  u32x4 stg[NPL][CPT];
  float stn = 0.f;
  int g_row[CPT], g_col[CPT], g_lin[CPT], l_off[CPT];
#pragma unroll
  for (int i = 0; i < CPT; ++i) {
    const int ch = tid + 256 * i;                                 // chunk ch of the tile
    g_lin[i] = ch * 8;
    g_row[i] = (ch / (D / 8)) * stride;
    g_col[i] = (ch % (D / 8)) * 8;
    l_off[i] = (ch / (D / 8)) * LDB + (ch % (D / 8)) * 8;
  }
#define FETCH_TILE(CT)                                                                           \
  do {                                                                                           \
    if constexpr (MODE == 1) {   /* every row: the tile is one contiguous block of memory */     \
      const unsigned short* __restrict__ th_ = Bhi + (CT) * D;                                   \
      const unsigned short* __restrict__ tl_ = Blo + (CT) * D;                                   \
      _Pragma("unroll") for (int i_ = 0; i_ < CPT; ++i_) {                                       \
        stg[0][i_] = *reinterpret_cast<const u32x4*>(th_ + g_lin[i_]);                           \
        if constexpr (LOB) stg[NPL - 1][i_] = *reinterpret_cast<const u32x4*>(tl_ + g_lin[i_]);   \
      }                                                                                          \
      stn = Bnorm[(CT) + (tid & 63)];                                                            \
    } else {                                                                                     \
      _Pragma("unroll") for (int i_ = 0; i_ < CPT; ++i_) {                                       \
        const int64_t o_ = min((CT) + g_row[i_], b_last) * D + g_col[i_];                        \
        stg[0][i_] = *reinterpret_cast<const u32x4*>(Bhi + o_);                                  \
        if constexpr (LOB) stg[NPL - 1][i_] = *reinterpret_cast<const u32x4*>(Blo + o_);         \
      }                                                                                          \
      stn = Bnorm[min((CT) + (int64_t)(tid & 63) * stride, b_last)];                             \
    }                                             /* stn is consumed only at the stash */        \
  } while (0)
#define STASH_TILE(BUF, CT)                                                                      \
  do {                                                                                           \
    _Pragma("unroll") for (int i_ = 0; i_ < CPT; ++i_) {                                         \
      _Pragma("unroll") for (int pl_ = 0; pl_ < NPL; ++pl_)                                      \
        *reinterpret_cast<u32x4*>(bt + ((BUF) * NPL + pl_) * BN * LDB + l_off[i_]) = stg[pl_][i_]; \
    }                                                                                            \
    if (tid < BN)                                                                                \
      bns[(BUF) * BN + tid] =                                                                    \
          (CT) + (int64_t)tid * stride < c_end                                                   \
              ? (METRIC == 0 ? (MODE == 1 ? stn * INV_S : stn) : 0.f) : __builtin_inff();        \
  } while (0)
  static_assert(CHUNKS % 256 == 0, "every lane stages the same number of chunks");

  if (MODE == 1)
    for (int i = tid; i < 128 * RB; i += 256) {
      cnt_s[i] = 0;
      an_s[i] = METRIC == 0 ? Anorm[min(rt * (128 * RB) + i, na - 1)] : 0.f;
    }
  // Takes n <= 64 queued candidates (the newest ones) and appends each to its row's list:
  // one LDS atomic per candidate for the position, all lanes in parallel.
  auto drain = [&](int n) {
    wave_lds_sync();
    const int e = qn - n + lane;
    if (lane < n) {
      const int rl = qrow[e];
      const u64 key = qkey[e];
      const int pos = atomicAdd(&cnt_s[rl], 1);
      const int64_t r = rt * (128 * RB) + rl;
      if (pos < cap) shortlist[(r * nsplit + split) * (int64_t)cap + pos] = key;
    }
    qn -= n;
    wave_lds_sync();
  };
  if (c_begin < c_end) { FETCH_TILE(c_begin); STASH_TILE(0, c_begin); }
  wait_all_global_loads();   // A fragments, thresholds and norms are in registers from here on
  block_sync_lds();
  int buf = 0;
  for (int64_t ct = c_begin; ct < c_end; ct += col_step, buf ^= 1) {
    const bool more = ct + col_step < c_end;
    if (more) FETCH_TILE(ct + col_step);                          // in flight during the MFMAs
    floatx16 m[RB][2];
    const unsigned short* __restrict__ bth = bt + (buf * NPL) * BN * LDB;
    // B fragments go through a ring of registers and are requested PF fragments ahead of
    // their use; the scheduling groups below pin that order (one LDS read per product group)
    constexpr int NF = KSTEPS * 2, PF = 4;
    static_assert(NF >= PF, "ring deeper than the tile");
    bf16x8 rh[PF], rl[LOB ? PF : 1];
#define FRAG_OFF(F) ((((F) & 1) * 32 + (lane & 31)) * LDB + ((F) >> 1) * 16 + 8 * (lane >> 5))
#pragma unroll
    for (int f = 0; f < PF; ++f) {
      rh[f] = *reinterpret_cast<const bf16x8*>(bth + FRAG_OFF(f));
      if constexpr (LOB) rl[f] = *reinterpret_cast<const bf16x8*>(bth + BN * LDB + FRAG_OFF(f));
    }
#pragma unroll
    for (int f = 0; f < NF; ++f) {
      const int kk = f >> 1, cb = f & 1;
      const bf16x8 ch = rh[f % PF];
      bf16x8 cl;
      if constexpr (LOB) cl = rl[f % PF];
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        // the first product starts from 0 (MODE 0) or from the row thresholds (MODE 1)
        m[rb][cb] = mfma_32x32x16<F16>(ah[rb][kk], ch, kk == 0 ? tr[rb] : m[rb][cb]);
        if constexpr (LOB) m[rb][cb] = mfma_32x32x16<false>(ah[rb][kk], cl, m[rb][cb]);
        if constexpr (THREE) m[rb][cb] = mfma_32x32x16<false>(al[rb][kk], ch, m[rb][cb]);
      }
      if (f + PF < NF) {
        rh[f % PF] = *reinterpret_cast<const bf16x8*>(bth + FRAG_OFF(f + PF));
        if constexpr (LOB) rl[f % PF] = *reinterpret_cast<const bf16x8*>(bth + BN * LDB + FRAG_OFF(f + PF));
      }
    }
#undef FRAG_OFF
    __builtin_amdgcn_sched_group_barrier(0x100, PF * NPL, 0);                       // LDS reads
#pragma unroll
    for (int f = 0; f < NF; ++f) {
      __builtin_amdgcn_sched_group_barrier(0x008, RB * (1 + (LOB ? 1 : 0) + (THREE ? 1 : 0)), 0);   // matrix products
      if (f + PF < NF) __builtin_amdgcn_sched_group_barrier(0x100, NPL, 0);
    }
    const float b0 = bns[buf * BN + (lane & 31)], b1 = bns[buf * BN + 32 + (lane & 31)];
    if (MODE == 0) {
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
          for (int v = 0; v < 16; ++v)
            mn[rb][cb][v] = fminf(mn[rb][cb][v], __builtin_fmaf(SCALE, m[rb][cb][v], cb ? b1 : b0));
      // end of a phase: flush the group minima (after the last step, also pad the phases left)
      const int ph = (int)((ct - c_begin) / cols_per_phase);
      const int ph_next = more ? (int)((ct + col_step - c_begin) / cols_per_phase) : nphase;
      for (int p2 = ph; p2 < ph_next; ++p2) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
          for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              const int64_t r = row0 + rb * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
              if (r < na)
                minima[r * g_raw + (split * nphase + p2) * 64 + cb * 32 + (lane & 31)] = mn[rb][cb][v];
              mn[rb][cb][v] = __builtin_inff();
            }
      }
    } else {
      // b0 / b1 hold b / s here.  Largest accumulator of each 32 x 32 block against the
      // column's bound: one v_max3 per two elements, one comparison per block.
      bool any[RB][2];
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
          float mx = m[rb][cb][0];
#pragma unroll
          for (int v = 1; v < 16; ++v) mx = fmaxf(mx, m[rb][cb][v]);
          any[rb][cb] = mx >= (cb ? b1 : b0);
        }
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
          if (__builtin_amdgcn_ballot_w64(any[rb][cb]) == 0) continue;   // nothing of this 32 x 32 block passes
          const float hb = cb ? b1 : b0;
          // rare path: narrow down by groups of four accumulators, then by element
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const float gm = fmaxf(fmaxf(m[rb][cb][4 * g], m[rb][cb][4 * g + 1]),
                                   fmaxf(m[rb][cb][4 * g + 2], m[rb][cb][4 * g + 3]));
            if (__builtin_amdgcn_ballot_w64(gm >= hb) == 0) continue;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
              const int v = 4 * g + u;
              const int rl = wave * (32 * RB) + rb * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
              const bool pass = m[rb][cb][v] >= hb;
              const u64 mask = __builtin_amdgcn_ballot_w64(pass);
              if (mask != 0) {
                if (pass) {
                  const int e = qn + __popcll(mask & ((1ull << lane) - 1ull));
                  // approximate value from the accumulator a = tau / s + <q,x>:
                  // L2: |q|^2 + |x|^2 - 2 <q,x> = |q|^2 + 2 (b / s - (a - tau / s));  IP: <q,x>
                  const float dotv = m[rb][cb][v] - tr[rb][v];
                  const float val = METRIC == 0 ? an_s[rl] + 2.f * (hb - dotv) : dotv;
                  qkey[e] = make_key(val, (u32)(ct + cb * 32 + (lane & 31)), METRIC);
                  qrow[e] = rl;
                }
                qn += __popcll(mask);
                if (qn >= 64) drain(64);
              }
            }
          }
        }
    }
    if (more) STASH_TILE(buf ^ 1, ct + col_step);
    block_sync_lds();
  }
#undef FETCH_TILE
#undef STASH_TILE
  if (MODE == 1) {
    if (qn > 0) drain(qn);
    block_sync_lds();
    for (int i = tid; i < 128 * RB; i += 256) {
      const int64_t r = rt * (128 * RB) + i;
      if (r < na) cnt[r * nsplit + split] = cnt_s[i];
    }
  }
  if (MODE == 0 && c_begin >= c_end) {                            // empty split: all its groups are +inf
    for (int ph = 0; ph < nphase; ++ph)
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int64_t r = row0 + rb * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
            if (r < na) minima[r * g_raw + (split * nphase + ph) * 64 + cb * 32 + (lane & 31)] = __builtin_inff();
          }
  }
}

// ---------------------------------------------------------------------------
// The same two sweeps for any d that is a multiple of 32 (up to 2048), where the fragments
// of a row block no longer fit in registers: a tiled contraction.  Workgroup = 8 wavefronts
// in a 4 x 2 grid over a 256 x 256 tile of (rows of A) x (rows of B); wavefront (wr, wc) owns
// rows 64 wr .. + 63 of the tile and the four 32-column blocks wc, wc + 2, wc + 4, wc + 6
// (interleaved, so that a short B still reaches all 64 group minima of a row) as 2 x 4 MFMA
// tiles (128 accumulators): one fragment read from LDS feeds 4 resp. 2 products.
// The operands come in the panel layout of prep_kernel: a block of 32 rows x 16 elements is
// 1 KB of consecutive memory.  The contraction runs over stages of 32 dimensions (two
// panels); the 16 row blocks of a stage are copied global -> LDS directly
// (global_load_lds_dwordx4: no staging registers, no LDS stores), one stage ahead of the
// products (two buffers).  A copy instruction moves one block: lane l fetches the 16 bytes
// of row (l & 31), elements 8 (l >> 5) .. + 7, and the hardware stores them at l * 16 of the
// block -- exactly the order in which the MFMA operand is read back, so fragment reads are
// 1 KB of consecutive LDS (conflict-free without padding).  The copies are not tracked by
// the compiler: every stage ends with an explicit wait for this wavefront's copies and a
// workgroup barrier, which is also what frees the other buffer for the next copies.
// The selection epilogue runs once per tile, after the last stage -- MODE 0 / MODE 1 exactly
// as in mfma_sweep_kernel.
// ---------------------------------------------------------------------------
template <int METRIC, int MODE, int PREC>   // PREC: 0, 2 or 3 as in mfma_sweep_kernel
__global__ __launch_bounds__(512)
void mfma_sweep_kc_kernel(const unsigned short* __restrict__ Ahi, const unsigned short* __restrict__ Alo,
                          const float* __restrict__ Anorm, const PrepInfo* __restrict__ Ainfo, int64_t na,
                          const unsigned short* __restrict__ Bhi, const unsigned short* __restrict__ Blo,
                          const float* __restrict__ Bnorm, const PrepInfo* __restrict__ Binfo, int64_t nb,
                          int d, int nsplit, int64_t cols_per_split, int stride, int nphase,
                          int64_t cols_per_phase, float* __restrict__ minima, int g_raw,
                          const float* __restrict__ tau, int* __restrict__ cnt,
                          u64* __restrict__ shortlist, int cap, int hbit) {
  constexpr int BM = 256, BN = 256, BLK = 1024;                  // BLK: bytes of a 32-row x 16-element block
  constexpr bool THREE = PREC == 2, F16 = PREC == 3;
  constexpr int NPL = THREE ? 2 : 1;
  constexpr int STAGE = NPL * 2 * 16 * BLK;                      // [plane][panel][8 A + 8 B blocks][BLK]
  constexpr float SCALE = METRIC == 0 ? -2.f : -1.f;
  constexpr float INV_S = METRIC == 0 ? 0.5f : 1.f;
  if (precision_variant(Ainfo, Binfo, hbit, false) != PREC) return;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* tiles = smem;                                           // [2][STAGE]
  float* bns = reinterpret_cast<float*>(tiles + 2 * STAGE);              // [2][BN]
  int* cnt_s = reinterpret_cast<int*>(bns + 2 * BN);                     // [BM]
  float* an_s = reinterpret_cast<float*>(cnt_s + BM);                    // [BM] |q|^2 of the rows
  float* tr_s = an_s + BM;                                               // [BM] row thresholds (MODE 1)
  u64* qkey = reinterpret_cast<u64*>(tr_s + BM) + (threadIdx.x >> 6) * 128;           // [8][128]
  int* qrow = reinterpret_cast<int*>(reinterpret_cast<u64*>(tr_s + BM) + 8 * 128) +
              (threadIdx.x >> 6) * 128;                                  // [8][128]
  int qn = 0;

  const int tid = threadIdx.x, wave = tid >> 6, lane = lane_id();
  const int wr = wave >> 1, wc = wave & 1;
  // Work item = (row tile, split of B), numbered row tile first.  Workgroup ids go round the
  // eight XCDs, each with an L2 of its own: XCD x takes a run of consecutive items, i.e. a few
  // row tiles with all their splits, so that its workgroups share their A and B tiles in L2
  // (with ids taken in order, no two workgroups of an XCD shared an A tile: 56 % L2 misses).
  const int64_t items = (na + BM - 1) / BM * nsplit, per_xcd = (items + 7) / 8;
  const int64_t item = (int64_t)(blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if ((int64_t)(blockIdx.x >> 3) >= per_xcd || item >= items) return;
  const int64_t rt = item / nsplit;
  const int split = (int)(item % nsplit);
  const int64_t row0 = rt * BM;
  const int64_t c_begin = (int64_t)split * cols_per_split;
  const int64_t c_end = min(nb, c_begin + cols_per_split);
  const int64_t col_step = (int64_t)BN * stride;
  const int64_t na_pad = (na + 63) / 64 * 64, nb_pad = (nb + 63) / 64 * 64;
  const int nst = d / 32;

  // running minima (MODE 0) of this wavefront's 64 rows; the row thresholds (MODE 1) sit in LDS
  float mn[2][16];
#pragma unroll
  for (int rb = 0; rb < 2; ++rb)
#pragma unroll
    for (int v = 0; v < 16; ++v) mn[rb][v] = __builtin_inff();

  // Copies: wavefront w moves row blocks 2w and 2w + 1 of every (plane, panel) of a stage;
  // blocks 0..7 are the 256 rows of A (wavefronts 0..3), 8..15 the 256 rows of B.
  const bool copies_a = wave < 4;
  const unsigned short* __restrict__ src_hi = copies_a ? Ahi : Bhi;
  const unsigned short* __restrict__ src_lo = copies_a ? Alo : Blo;
  const int64_t panel_elems = (copies_a ? na_pad : nb_pad) * 16;
  int64_t goff[2];                         // element offset of this lane's 16 bytes inside a panel
  auto set_rows = [&](int64_t ct) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int rl = ((wave & 3) * 2 + i) * 32 + (lane & 31);            // row of the tile, 0..255
      const int64_t g = copies_a ? min(row0 + rl, na_pad - 1) : min(ct + (int64_t)rl * stride, nb_pad - 1);
      goff[i] = g * 16 + 8 * (lane >> 5);
    }
  };
  // copy number c of a stage, c < 4 NPL: (plane, panel, row block) = (c / 4, (c / 2) % 2, c % 2)
  auto copy_one = [&](int buf, int st, int c) {
    const int pl = c >> 2, pp = (c >> 1) & 1, i = c & 1;
    const unsigned short* g = (pl ? src_lo : src_hi) + (int64_t)(st * 2 + pp) * panel_elems + goff[i];
    unsigned char* l = tiles + buf * STAGE + ((pl * 2 + pp) * 16 + wave * 2 + i) * BLK;
    __builtin_amdgcn_global_load_lds(g, l, 16, 0, 0);
  };
  auto copy_stage = [&](int buf, int st) {
#pragma unroll
    for (int c = 0; c < 4 * NPL; ++c) copy_one(buf, st, c);
  };
  float stn = 0.f;

  if (MODE == 1)
    for (int i = tid; i < BM; i += 512) {
      cnt_s[i] = 0;
      an_s[i] = METRIC == 0 ? Anorm[min(row0 + i, na - 1)] : 0.f;
      tr_s[i] = row0 + i < na ? tau[row0 + i] * INV_S : -__builtin_inff();
    }
  auto drain = [&](int n) {
    wave_lds_sync();
    const int e = qn - n + lane;
    if (lane < n) {
      const int rl = qrow[e];
      const u64 key = qkey[e];
      const int pos = atomicAdd(&cnt_s[rl], 1);
      const int64_t r = row0 + rl;
      if (pos < cap) shortlist[(r * nsplit + split) * (int64_t)cap + pos] = key;
    }
    qn -= n;
    wave_lds_sync();
  };

  if (c_begin < c_end) {
    set_rows(c_begin);
    copy_stage(0, 0);
    if (tid < BN) {
      const int64_t c = c_begin + (int64_t)tid * stride;
      stn = Bnorm[min(c, nb_pad - 1)];
      bns[tid] = c < c_end ? (METRIC == 0 ? (MODE == 1 ? stn * INV_S : stn) : 0.f) : __builtin_inff();
    }
  }
  wait_all_global_loads();
  block_sync_lds();
  int buf = 0;
  floatx16 m[2][4];
  const int ntiles = c_begin < c_end ? (int)((c_end - c_begin + col_step - 1) / col_step) : 0;
  for (int tile = 0; tile < ntiles; ++tile) {
    const int64_t ct = c_begin + tile * col_step;
    for (int st = 0; st < nst; ++st, buf ^= 1) {
      // the stage after this one: next stage of the same tile, or the first of the next tile
      const bool last_st = st + 1 == nst;
      const int64_t ct_n = last_st ? ct + col_step : ct;
      const bool more = !last_st || tile + 1 < ntiles;
      const int st_n = last_st ? 0 : st + 1;
      if (more) {
        if (last_st && !copies_a) set_rows(ct_n);
        copy_stage(buf ^ 1, st_n);
        if (last_st && tid < BN) stn = Bnorm[min(ct_n + (int64_t)tid * stride, nb_pad - 1)];
      }
      const unsigned char* __restrict__ tb = tiles + buf * STAGE;
      if (st == 0) {   // a new tile starts from 0 (MODE 0) / from the row thresholds (MODE 1)
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
          floatx16 t0;
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            float4 t4 = make_float4(0.f, 0.f, 0.f, 0.f);
            if (MODE == 1) t4 = *reinterpret_cast<const float4*>(tr_s + wr * 64 + rb * 32 + 8 * g + 4 * (lane >> 5));
            t0[4 * g] = t4.x; t0[4 * g + 1] = t4.y; t0[4 * g + 2] = t4.z; t0[4 * g + 3] = t4.w;
          }
#pragma unroll
          for (int cb = 0; cb < 4; ++cb) m[rb][cb] = t0;
        }
      }
#pragma unroll
      for (int pp = 0; pp < 2; ++pp) {
        bf16x8 ah[2], al[2], bh[4], bl[4];
#pragma unroll
        for (int x = 0; x < 2; ++x) {
          ah[x] = *reinterpret_cast<const bf16x8*>(tb + (pp * 16 + wr * 2 + x) * BLK + lane * 16);
          if constexpr (THREE)
            al[x] = *reinterpret_cast<const bf16x8*>(tb + ((2 + pp) * 16 + wr * 2 + x) * BLK + lane * 16);
        }
#pragma unroll
        for (int y = 0; y < 4; ++y) {
          bh[y] = *reinterpret_cast<const bf16x8*>(tb + (pp * 16 + 8 + 2 * y + wc) * BLK + lane * 16);
          if constexpr (THREE)
            bl[y] = *reinterpret_cast<const bf16x8*>(tb + ((2 + pp) * 16 + 8 + 2 * y + wc) * BLK + lane * 16);
        }
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
          for (int cb = 0; cb < 4; ++cb) {
            m[rb][cb] = mfma_32x32x16<F16>(ah[rb], bh[cb], m[rb][cb]);
            if constexpr (THREE) {
              m[rb][cb] = mfma_32x32x16<false>(ah[rb], bl[cb], m[rb][cb]);
              m[rb][cb] = mfma_32x32x16<false>(al[rb], bh[cb], m[rb][cb]);
            }
          }
      }
      if (last_st) {   // the tile is complete: selection epilogue
        float bt[4];
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) bt[cb] = bns[(tile & 1) * BN + (2 * cb + wc) * 32 + (lane & 31)];
        if (MODE == 0) {
#pragma unroll
          for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int cb = 0; cb < 4; ++cb)
#pragma unroll
              for (int v = 0; v < 16; ++v)
                mn[rb][v] = fminf(mn[rb][v], __builtin_fmaf(SCALE, m[rb][cb][v], bt[cb]));
          const int ph = (int)((ct - c_begin) / cols_per_phase);
          const int ph_next = tile + 1 < ntiles ? (int)((ct + col_step - c_begin) / cols_per_phase) : nphase;
          for (int p2 = ph; p2 < ph_next; ++p2) {
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
              for (int v = 0; v < 16; ++v) {
                const int64_t r = row0 + wr * 64 + rb * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (r < na)
                  minima[r * g_raw + (split * nphase + p2) * 64 + wc * 32 + (lane & 31)] = mn[rb][v];
                mn[rb][v] = __builtin_inff();
              }
          }
        } else {
          bool any[2][4];
#pragma unroll
          for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int cb = 0; cb < 4; ++cb) {
              float mx = m[rb][cb][0];
#pragma unroll
              for (int v = 1; v < 16; ++v) mx = fmaxf(mx, m[rb][cb][v]);
              any[rb][cb] = mx >= bt[cb];
            }
#pragma unroll
          for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int cb = 0; cb < 4; ++cb) {
              if (__builtin_amdgcn_ballot_w64(any[rb][cb]) == 0) continue;
              const float hb = bt[cb];
#pragma unroll
              for (int g = 0; g < 4; ++g) {   // rare path: by groups of four, then by element
                const float gm = fmaxf(fmaxf(m[rb][cb][4 * g], m[rb][cb][4 * g + 1]),
                                       fmaxf(m[rb][cb][4 * g + 2], m[rb][cb][4 * g + 3]));
                if (__builtin_amdgcn_ballot_w64(gm >= hb) == 0) continue;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                  const int v = 4 * g + u;
                  const int rl = wr * 64 + rb * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                  const bool pass = m[rb][cb][v] >= hb;
                  const u64 mask = __builtin_amdgcn_ballot_w64(pass);
                  if (mask != 0) {
                    if (pass) {
                      const int e = qn + __popcll(mask & ((1ull << lane) - 1ull));
                      const float dotv = m[rb][cb][v] - tr_s[rl];
                      const float val = METRIC == 0 ? an_s[rl] + 2.f * (hb - dotv) : dotv;
                      qkey[e] = make_key(val, (u32)(ct + (2 * cb + wc) * 32 + (lane & 31)), METRIC);
                      qrow[e] = rl;
                    }
                    qn += __popcll(mask);
                    if (qn >= 64) drain(64);
                  }
                }
              }
            }
        }
        if (more && tid < BN)   // column terms of the next tile (the other half of bns)
          bns[((tile + 1) & 1) * BN + tid] =
              ct_n + (int64_t)tid * stride < c_end
                  ? (METRIC == 0 ? (MODE == 1 ? stn * INV_S : stn) : 0.f) : __builtin_inff();
      }
      wait_all_global_loads();   // this wavefront's copies of the next stage have landed
      block_sync_lds();          // ... everyone's have, and everyone is done reading this stage
    }
  }
  if (MODE == 1) {
    if (qn > 0) drain(qn);
    block_sync_lds();
    for (int i = tid; i < BM; i += 512) {
      const int64_t r = row0 + i;
      if (r < na) cnt[r * nsplit + split] = cnt_s[i];
    }
  }
  if (MODE == 0 && c_begin >= c_end) {
    for (int ph = 0; ph < nphase; ++ph)
#pragma unroll
      for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int64_t r = row0 + wr * 64 + rb * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
          if (r < na) minima[r * g_raw + (split * nphase + ph) * 64 + wc * 32 + (lane & 31)] = __builtin_inff();
        }
  }
}

// tau(row) = kp-th smallest of the row's g_raw group minima (min-combined down to 64 * RG
// values first), or the largest finite one if fewer than kp are finite.
template <int RG>
__global__ __launch_bounds__(256) void tau_kernel(const float* __restrict__ minima, int g_raw,
                                                  int64_t na, int kp, float* __restrict__ tau,
                                                  int* __restrict__ zero_this) {
  // (also clears the count of rows that the re-rank, which runs later on the same stream, will
  // send to the exact fallback: one launch less per call)
  if (zero_this && blockIdx.x == 0 && threadIdx.x == 0) *zero_this = 0;
  const int64_t row = blockIdx.x * 4ll + (threadIdx.x >> 6);
  if (row >= na) return;
  const int lane = lane_id();
  const float* __restrict__ src = minima + row * g_raw;
  u32 v[RG];
#pragma unroll
  for (int r = 0; r < RG; ++r) v[r] = order_f32(__builtin_inff());
  // value j goes to slot j % (64 * RG): lane (j / RG) % 64, register j % RG
#pragma unroll 8
  for (int j0 = 0; j0 < g_raw; j0 += 64 * RG) {
#pragma unroll
    for (int r = 0; r < RG; ++r) {
      const int j = j0 + lane * RG + r;
      if (j < g_raw) { const u32 o = order_f32(src[j]); v[r] = o < v[r] ? o : v[r]; }
    }
  }
  wave_sort_regs(v);
  // With fewer than kp finite minima (a short B) the threshold is the largest finite one: any
  // threshold is valid for the re-rank test, and a finite one keeps the collect sweep's
  // accumulators (which start at the threshold) in a range where the products still register.
  int nfin = 0;
#pragma unroll
  for (int r = 0; r < RG; ++r) nfin += v[r] < order_f32(__builtin_inff()) ? 1 : 0;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) nfin += __shfl_xor(nfin, off);
  const int rank = max(min(kp, nfin), 1) - 1;
  u32 pick = 0;
#pragma unroll
  for (int r = 0; r < RG; ++r)
    if (lane * RG + r == rank) pick = v[r];
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) pick |= (u32)__shfl_xor((int)pick, off);
  if (lane == 0) {
    float t = unorder_f32(pick);
    if (nfin < kp) t += __builtin_fabsf(t) * 1e-3f;    // (the two sweeps round differently: keep the largest listed)
    tau[row] = fminf(t, 3.4028234e38f);
  }
}

// ---------------------------------------------------------------------------
// Exact re-rank: one wavefront per row of A.
// ---------------------------------------------------------------------------
template <int R, int METRIC>
__global__ __launch_bounds__(64) void rerank_kernel(
    const u64* __restrict__ shortlist, const int* __restrict__ cnt, const float* __restrict__ tau,
    int nsplit, int cap, int kp, const float* __restrict__ A,
    const float* __restrict__ B, int64_t nb, int d, int k, const float* __restrict__ Anorm,
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
  bool truncated = false;
  int64_t total = 0;                                            // columns with m <= tau
  // (eight splits at a time: their counts and the first 64 slots of their lists -- cap >= 64,
  // the slots exist whether filled or not -- are requested together, one round trip instead
  // of sixteen; a handful of rows against many splits is bound by exactly these)
  for (int sp0 = 0; sp0 < nsplit; sp0 += 8) {
    int listed[8];
    u64 first[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int sp = min(sp0 + u, nsplit - 1);
      listed[u] = sp0 + u < nsplit ? cnt[row * nsplit + sp] : 0;
      first[u] = shortlist[(row * nsplit + sp) * (int64_t)cap + lane];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (sp0 + u >= nsplit) break;
      const u64* __restrict__ src = shortlist + (row * nsplit + sp0 + u) * (int64_t)cap;
      truncated = truncated || listed[u] > cap;
      total += listed[u];
      const int n = min(listed[u], cap);
      if (n > 0) ws.push(lane < n && first[u] != KEY_EMPTY, first[u]);
      for (int j0 = VS_WAVE; j0 < n; j0 += VS_WAVE) {
        const int j = j0 + lane;
        const u64 key = j < n ? src[j] : KEY_EMPTY;
        ws.push(j < n && key != KEY_EMPTY, key);
      }
    }
  }
  ws.finish();
  const u64 tkey = ws.s[kp - 1];                                // kp-th best approximate key

  // canon value of every shortlisted row, then an exact sort
  // (one row per lane, R rows in flight per lane: staging 64 rows at a time through an LDS
  // tile, as the refinement kernel does, measured slower here)
  u64 v[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int e = lane * R + r;
    const u64 ak = e < kp ? ws.s[e] : KEY_EMPTY;
    if (ak == KEY_EMPTY) { v[r] = KEY_EMPTY; continue; }
    const u32 idx = key_index(ak);
    v[r] = make_key(canon_row<METRIC>(qs, B + (int64_t)idx * d, d, vec), idx, METRIC);
  }
  wave_sort_regs(v);
  wave_lds_sync();
#pragma unroll
  for (int r = 0; r < R; ++r) slots[lane * R + r] = v[r];
  wave_lds_sync();
  const lds_u64_ptr sorted = to_lds(slots);
  const u64 vk = sorted[k - 1];                                 // k-th best canon key

  // Is the shortlist provably sufficient?  Every column that is not listed has m > tau, i.e.
  // an approximate value beyond `ub`; every listed column that was not re-ranked is no better
  // than the kp-th best approximate key.
  bool ok = true;
  if (vk == KEY_EMPTY) {
    ok = total >= nb;                    // fewer than k candidates: right only if every column is listed
  } else {
    const float na2 = Anorm[row], nb2 = __uint_as_float(Binfo->max_norm_bits);
    // Integer data exactly representable in bf16: every number the sweeps and this kernel
    // form is a multiple of 1/2 below 2^23 in magnitude, hence exact, when N = max|q|^2 +
    // max|x|^2 satisfies 1.5 N < 2^23 (|<q,x>| <= N / 2, |tau| / 2 <= N), or N < 2^23 when
    // no value is negative (0 <= <q,x>, -|q|^2 <= tau <= |x|^2).
    const float nsum = __uint_as_float(Ainfo->max_norm_bits) + nb2;
    const bool nonneg = Ainfo->all_nonneg && Binfo->all_nonneg;
    const bool exact = Ainfo->all_int && Binfo->all_int && Ainfo->all_bf16 && Binfo->all_bf16 &&
                       (nonneg ? nsum < 8388608.f : nsum < 5592405.f);
    if (!exact) {   // (exact: approximate = canon bit for bit, so the k best listed keys are the answer)
      const bool inexact = !(Ainfo->all_bf16 && Binfo->all_bf16);
      // |approx - canon| <= eps: bf16 head/tail split drops terms below 2^-15 |q||x| per product;
      // fp32 accumulation and the canon chain each stay below d 2^-22 (|q|^2 + |x|^2); the
      // collect sweep's own rounding (a few ulps of |tau| / 2 + |<q,x>|) is the last term.
      // fp16 heads alone: qh_i = q_i + a_i with |a_i| <= u |q_i| + s, u = 2^-11 (rounding to 11
      // significant bits) and s = 2^-25 (half the spacing of fp16 subnormals), likewise x, so
      // |<q,x> - <qh,xh>| <= (2u + u^2) |q||x| + s (1 + u) sqrt(d) (|q| + |x|) + d s^2; with
      // |q||x| <= N / 2 and |q| + |x| <= sqrt(2 N), N = |q|^2 + |x|^2, twice that on the distance:
      // 9.78e-4 N + 6.0e-8 sqrt(2 d N) + 1.8e-15 d (inner product: the value is the product itself,
      // half of each).
      const bool f16 = precision_variant(Ainfo, Binfo, k == 1 ? 1 : 2, false) == 3;
      const float nn = na2 + nb2;
      constexpr float F16_S = METRIC == 0 ? 1.f : 0.5f;
      const float split_term = !inexact ? 0.f : (f16 ? F16_S * 9.78e-4f : 6.2e-5f);
      const float coef = split_term + (float)d * 4.8e-7f + 2e-6f;
      const float abs_term = f16 ? F16_S * (6.0e-8f * sqrtf(2.f * (float)d * nn) + 1.8e-15f * (float)d) : 0.f;
      const float eps = eps_scale * (coef * nn + abs_term);
      const float tau_v = tau[row];
      const float ub = METRIC == 0 ? na2 + tau_v : -tau_v;
      const float kv = key_value(vk, METRIC);
      float tv = ub;
      if (total > kp && tkey != KEY_EMPTY) {
        const float t2 = key_value(tkey, METRIC);
        tv = METRIC == 0 ? fminf(tv, t2) : fmaxf(tv, t2);
      }
      ok = METRIC == 0 ? (tv - eps > kv) : (tv + eps < kv);
    }
  }
  if (truncated) ok = false;                                    // a candidate list was truncated
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

// How the exact fallback cuts the columns of B into chunks.  The host plans chunks for the worst
// case (every row redone); with few redone rows those would leave most of the chip idle (5 rows x
// 2 chunks of 8192 columns x 768 dimensions: 0.8 ms on ten workgroups), so the kernels cut finer
// -- about three tasks per compute unit, at most 64 chunks of at least 256 columns -- as far as
// the buffer of partial results (cap_keys keys; 0: keep the host's plan) holds count * nchunk * k.
struct FallbackSplit { int64_t chunk_cols; int nchunk; };
__device__ __forceinline__ FallbackSplit fallback_split(int count, int64_t nb, int k, int64_t chunk_cols,
                                                        int nchunk, int64_t cap_keys) {
  FallbackSplit f;
  f.chunk_cols = chunk_cols; f.nchunk = nchunk;
  if (cap_keys > 0 && count > 0) {
    int64_t want = (768 + count - 1) / count;
    want = min(min(want, (int64_t)64), min((nb + 255) / 256, cap_keys / ((int64_t)count * k)));
    if (want > nchunk) {
      f.chunk_cols = ((nb + want - 1) / want + 255) / 256 * 256;
      f.nchunk = (int)((nb + f.chunk_cols - 1) / f.chunk_cols);
    }
  }
  return f;
}

// Canon over ALL columns for the rows listed in fb_rows.  Persistent workgroups walk over
// (listed row, column chunk) tasks, so that even a single listed row is spread over the
// chip; with more than one chunk the k best of each chunk go to `partial` as keys and
// canon_rows_merge_kernel picks the k best of a row's chunks.
template <int R, int METRIC>
__global__ __launch_bounds__(256) void canon_rows_kernel(const float* __restrict__ A,
                                                         const float* __restrict__ B, int64_t nb,
                                                         int d, int k, int tot, int64_t chunk_cols0,
                                                         int nchunk0, int64_t cap_keys,
                                                         u64* __restrict__ partial, SelectOut out,
                                                         const int* __restrict__ fb_count,
                                                         const int* __restrict__ fb_rows,
                                                         PrepInfo* __restrict__ adapt, int64_t na) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  u64* slots = reinterpret_cast<u64*>(smem);                    // 4 * tot
  float* qs = reinterpret_cast<float*>(slots + 4 * tot);        // d
  const int wave = threadIdx.x >> 6;
  const bool vec = (d & 3) == 0;
  const int count = *fb_count;
  if (blockIdx.x == 0 && threadIdx.x == 0 && count > 0) {
    atomicAdd(&g_fallback_total, (unsigned long long)count);
    // heads alone did not do for calls of this kind on this operand: so many rows had to be redone
    // here (more than one in 512) that it cost more than the two matrix products saved: a redone row
    // costs some hundred times its share of a sweep -- from the next call on the sweeps use all three
    const u32 bit = k == 1 ? 1u : 2u;
    if (adapt && (adapt->heads_only & bit) && count >= 8 && (int64_t)count * 512 > na) atomicAnd(&adapt->heads_only, ~bit);
  }
  const FallbackSplit fs = fallback_split(count, nb, k, chunk_cols0, nchunk0, cap_keys);
  const int64_t chunk_cols = fs.chunk_cols;
  const int nchunk = fs.nchunk;
  const int64_t tasks = (int64_t)count * nchunk;
  for (int64_t task = blockIdx.x; task < tasks; task += gridDim.x) {
    const int64_t f = task / nchunk;
    const int ch = (int)(task - f * nchunk);
    const int64_t row = fb_rows[f];
    const int64_t c_begin = ch * chunk_cols, c_end = min(nb, c_begin + chunk_cols);
    __syncthreads();
    for (int t = threadIdx.x; t < d; t += 256) qs[t] = A[row * d + t];
    WaveSelect<R> ws;
    ws.init(slots + wave * tot, tot, k);
    __syncthreads();
    for (int64_t c0 = c_begin; c0 < c_end; c0 += 256) {
      const int64_t c = c0 + threadIdx.x;
      const bool valid = c < c_end;
      const float val = valid ? canon_row<METRIC>(qs, B + c * d, d, vec) : 0.f;
      ws.push(valid, make_key(val, (u32)c, METRIC));
    }
    ws.finish();
    __syncthreads();
    KeySink sink;
    sink.idmap = nullptr; sink.metric = METRIC;
    if (nchunk == 1) {
      sink.keys = nullptr; sink.val = out.val; sink.id64 = out.id64; sink.idx32 = out.idx32;
      block_rank_merge(slots, tot, 4, k, sink, row * (int64_t)k);
    } else {
      sink.keys = partial; sink.val = nullptr; sink.id64 = nullptr; sink.idx32 = nullptr;
      block_rank_merge(slots, tot, 4, k, sink, task * (int64_t)k);
    }
  }
}

// The same fallback for d a multiple of 32 (every shape the matrix-core route serves), with the
// columns staged through LDS: one row of B per lane read straight from memory makes every load
// instruction touch 64 cache lines and the chain wait for each of them (6 us per redone row at
// 65536 x 96).  Here a tile of 256 rows of B x 32 dimensions is fetched with 8 lanes per row (128
// consecutive bytes per request), written to LDS with a row stride of 36 floats (16-byte aligned,
// conflict-free for the 16-byte reads that follow), and lane r continues the canon chain of row r
// over those 32 dimensions -- the same values in the same order as canon_row, hence the same bits.
// The next tile chunk is in flight (registers) while the current one is summed.
template <int R, int METRIC>
__global__ __launch_bounds__(256) void canon_rows_tiled_kernel(const float* __restrict__ A,
                                                               const float* __restrict__ B, int64_t nb,
                                                               int d, int k, int tot, int64_t chunk_cols0,
                                                               int nchunk0, int64_t cap_keys,
                                                               u64* __restrict__ partial, SelectOut out,
                                                               const int* __restrict__ fb_count,
                                                               const int* __restrict__ fb_rows,
                                                               PrepInfo* __restrict__ adapt, int64_t na) {
  constexpr int DC = 32, LD = 36, TR = 256;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  u64* slots = reinterpret_cast<u64*>(smem);                    // 4 * tot
  float* qs = reinterpret_cast<float*>(slots + 4 * tot);        // d
  float* tile = qs + d;                                         // 2 x TR x LD
  const int tid = threadIdx.x, wave = tid >> 6;
  const int r_ld = tid >> 3, c_ld = tid & 7;                    // fetch: 8 lanes per row, 32 rows per pass
  const int count = *fb_count;
  if (blockIdx.x == 0 && threadIdx.x == 0 && count > 0) {
    atomicAdd(&g_fallback_total, (unsigned long long)count);
    // heads alone did not do for calls of this kind on this operand: so many rows had to be redone
    // here (more than one in 512) that it cost more than the two matrix products saved -- from the
    // next call on the sweeps use all three
    const u32 bit = k == 1 ? 1u : 2u;
    if (adapt && (adapt->heads_only & bit) && count >= 8 && (int64_t)count * 512 > na) atomicAnd(&adapt->heads_only, ~bit);
  }
  const FallbackSplit fs = fallback_split(count, nb, k, chunk_cols0, nchunk0, cap_keys);
  const int64_t chunk_cols = fs.chunk_cols;
  const int nchunk = fs.nchunk;
  const int64_t tasks = (int64_t)count * nchunk;
  for (int64_t task = blockIdx.x; task < tasks; task += gridDim.x) {
    const int64_t f = task / nchunk;
    const int ch = (int)(task - f * nchunk);
    const int64_t row = fb_rows[f];
    const int64_t c_begin = ch * chunk_cols, c_end = min(nb, c_begin + chunk_cols);
    __syncthreads();                                            // the task before is done with qs, tile and slots
    for (int t = tid; t < d; t += 256) qs[t] = A[row * d + t];
    WaveSelect<R> ws;
    ws.init(slots + wave * tot, tot, k);
    u32x4 stg[8];
    auto fetch = [&](int64_t i0, int c0) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int64_t r = min(i0 + j * 32 + r_ld, c_end - 1);   // rows past the end: masked at the push
        stg[j] = *reinterpret_cast<const u32x4*>(B + r * d + c0 + c_ld * 4);
      }
    };
    auto stash = [&](int buf) {
#pragma unroll
      for (int j = 0; j < 8; ++j)
        *reinterpret_cast<u32x4*>(tile + (buf * TR + j * 32 + r_ld) * LD + c_ld * 4) = stg[j];
    };
    int64_t i0 = c_begin;
    int c0 = 0, buf = 0;
    bool ok = i0 < c_end;                                        // (uniform)
    if (ok) { fetch(i0, c0); stash(0); }
    __syncthreads();                                            // query and the first chunk
    float acc = 0.f;
    while (ok) {
      int64_t ni0 = i0;
      int nc0 = c0 + DC;
      if (nc0 >= d) { nc0 = 0; ni0 += TR; }
      const bool nok = ni0 < c_end;
      if (nok) fetch(ni0, nc0);                                 // in flight during the arithmetic
      const float* __restrict__ tr = tile + (buf * TR + tid) * LD;
      const float* __restrict__ qc = qs + c0;
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
      if (c0 + DC >= d) {                                       // the row is complete
        const int64_t i = i0 + tid;
        ws.push(i < c_end, make_key(acc, (u32)i, METRIC));
        acc = 0.f;
      }
      if (nok) stash(buf ^ 1);
      block_sync_lds();
      i0 = ni0; c0 = nc0; ok = nok; buf ^= 1;
    }
    ws.finish();
    __syncthreads();
    KeySink sink;
    sink.idmap = nullptr; sink.metric = METRIC;
    if (nchunk == 1) {
      sink.keys = nullptr; sink.val = out.val; sink.id64 = out.id64; sink.idx32 = out.idx32;
      block_rank_merge(slots, tot, 4, k, sink, row * (int64_t)k);
    } else {
      sink.keys = partial; sink.val = nullptr; sink.id64 = nullptr; sink.idx32 = nullptr;
      block_rank_merge(slots, tot, 4, k, sink, task * (int64_t)k);
    }
  }
}

// One wavefront per listed row: k best of its nchunk * k partial keys.
template <int R, int METRIC>
__global__ __launch_bounds__(64) void canon_rows_merge_kernel(const u64* __restrict__ partial, int64_t nb,
                                                              int64_t chunk_cols0, int nchunk0,
                                                              int64_t cap_keys, int k, int tot,
                                                              SelectOut out,
                                                              const int* __restrict__ fb_count,
                                                              const int* __restrict__ fb_rows) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  u64* slots = reinterpret_cast<u64*>(smem);                    // tot
  const int lane = lane_id();
  const int count = *fb_count;
  const int nchunk = fallback_split(count, nb, k, chunk_cols0, nchunk0, cap_keys).nchunk;
  if (nchunk == 1) return;                                      // the rows were written directly
  for (int f = blockIdx.x; f < count; f += gridDim.x) {
    const int64_t row = fb_rows[f];
    WaveSelect<R> ws;
    ws.init(slots, tot, k);
    const u64* __restrict__ src = partial + (int64_t)f * nchunk * k;
    const int n = nchunk * k;
    for (int j0 = 0; j0 < n; j0 += VS_WAVE) {
      const int j = j0 + lane;
      const u64 key = j < n ? src[j] : KEY_EMPTY;
      ws.push(j < n && key != KEY_EMPTY, key);
    }
    ws.finish();
    for (int j = lane; j < k; j += VS_WAVE) {
      const u64 key = ws.s[j];
      const bool empty = key == KEY_EMPTY;
      const int64_t at = row * (int64_t)k + j;
      if (out.val) out.val[at] = empty ? (METRIC ? -__builtin_inff() : __builtin_inff()) : key_value(key, METRIC);
      if (out.id64) out.id64[at] = empty ? -1 : (int64_t)key_index(key);
      if (out.idx32) out.idx32[at] = empty ? -1 : (int32_t)key_index(key);
    }
    wave_lds_sync();
  }
}


}  // namespace

// ------------------------------------------------------------------ launchers

int64_t mfma_padded_rows(int64_t n) { return (n + 63) / 64 * 64; }

bool mfma_knn_supported(int d, int k) {
  return d >= 32 && d % 32 == 0 && d <= 2048 && k <= 150;
}

int mfma_knn_kp(int k) {
  // (k = 1, the assignment of the add path and of k-means: 8 candidates are re-ranked instead
  // of 24 -- the re-rank's gathers are 7 % of an assignment -- and a row whose best is not
  // provably among them takes the exact fallback as always)
  int kp = k + (k == 1 ? 7 : std::max(16, k / 4));
  kp = (kp + 7) / 8 * 8;
  return std::min(kp, 192);
}

namespace {
// (the register-stationary kernel measured 1.3 - 1.45x faster than the tiled one at these d)
bool stationary_d(int d) { return d == 32 || d == 64 || d == 96 || d == 128; }
}  // namespace

void launch_prep(const float* x, int64_t n, int d, unsigned short* hi, unsigned short* lo,
                 float* norm, PrepInfo* info, hipStream_t st, bool try_heads_only) {
  hipLaunchKernelGGL(prep_info_init_kernel, dim3(1), dim3(1), 0, st, info, try_heads_only ? 1u : 0u);
  if (n <= 0) return;
  const int64_t n_pad = mfma_padded_rows(n);
  if (!stationary_d(d)) {                            // the tiled kernel reads panels
    hipLaunchKernelGGL(prep_panel_kernel, dim3((unsigned)std::min<int64_t>(n_pad / 32, 4096)), dim3(256), 0,
                       st, x, n, n_pad, d, hi, lo, norm, info);
    return;
  }
  const int rpb = 2048 / d;                          // d % 8 == 0
  const int64_t ngroups = (n_pad + rpb - 1) / rpb;
  hipLaunchKernelGGL(prep_kernel, dim3((unsigned)std::min<int64_t>(ngroups, 4096)), dim3(256), 0, st, x, n,
                     n_pad, d, rpb, hi, lo, norm, info);
}

namespace {
struct MfmaPlan {
  bool kc;                                   // general-d kernel (256 x 256 tiles) instead of the
                                             // register-stationary one (128 rows x 64 columns)
  int RB, nsplit, nphase, g_raw, rg, kp, kp_tau, stride, cap;
  int hbit;                                  // the bit of PrepInfo::heads_only that calls with this k go by
  int64_t cols_per_split, cols_per_phase, row_tiles;
  size_t o_minima, o_tau, o_cnt, bytes;      // offsets behind the shortlist [na][nsplit][cap]
};
size_t up256(size_t v) { return (v + 255) / 256 * 256; }
// Calls for the single nearest row (list assignment) and calls for the k > 1 nearest (probes, flat
// search) learn separately whether the heads alone do: their margins differ.
__host__ __device__ inline int heads_only_bit(int k) { return k == 1 ? 1 : 2; }

MfmaPlan make_plan(int64_t na, int64_t nb, int k, int d) {
  MfmaPlan p;
  p.kc = !stationary_d(d);
  const int bm = p.kc ? 256 : 128, bn = p.kc ? 256 : 64;      // tile of one workgroup step
  p.kp = mfma_knn_kp(k);
  p.hbit = heads_only_bit(k);
  p.cap = std::max(64, 3 * p.kp);
  // Row blocks of A per wavefront.  Operands split in head and tail: one 32-row block (two
  // workgroups per CU).  Operands exactly bf16: the fragments are half as many, and the
  // collect sweep takes two row blocks per wavefront (still two workgroups per CU; half
  // the tile traffic, LDS reads and barriers per product; measured 7-10 % faster than
  // three workgroups per CU with one block) unless A is so short that the second block
  // would be mostly padding.
  p.RB = na >= 1024 ? 2 : 1;
  p.row_tiles = (na + bm - 1) / bm;
  const int64_t col_steps = std::max<int64_t>(1, (nb + bn - 1) / bn);
  // Most splits of B a plan may use: 16 resp. 24, and more when A is so short that those
  // would leave most of the chip idle (a handful of queries against a long B) -- as long as
  // the per-(row, split) lists stay within 256 MB.
  const int64_t stride0 = p.kc ? 16 : std::max<int64_t>(1, std::min<int64_t>(16, col_steps / 192));
  const double r0 = stride0 == 1 ? 0.0 : std::ceil((double)k / stride0 + 4.0 * std::sqrt((double)k / stride0) + 2.0);
  const int64_t cap0 = stride0 == 1 ? p.cap
                                    : std::max<int64_t>(64, (int64_t)std::ceil(1.15 * stride0 * (r0 + 5.5 * std::sqrt(r0) + 8.0)) + 16);
  const int64_t slots = p.kc ? 256 : 512, ns_usual = p.kc ? 16 : 24;
  int64_t ns_cap = ns_usual;
  if (p.row_tiles * ns_usual < slots) {
    ns_cap = (slots + p.row_tiles - 1) / p.row_tiles;
    const int64_t by_memory = (int64_t)((256ull << 20) / ((size_t)na * cap0 * sizeof(u64)));
    ns_cap = std::max(ns_usual, std::min(ns_cap, by_memory));
  }
  // ... and at least 8 tiles of B per split, unless that leaves fewer than 128 workgroups
  int64_t by_length = std::max<int64_t>(1, col_steps / 8);
  if (p.row_tiles * by_length < 128) by_length = std::max(by_length, std::min<int64_t>(col_steps, 128 / p.row_tiles));
  int64_t ns;
  if (p.kc) {   // 256 resident workgroups
    ns = std::max<int64_t>(1, 256 / p.row_tiles);
    ns = std::min(ns, by_length);
    ns = std::min<int64_t>(ns, ns_cap);
  } else {
    // Splits of B so that the workgroups come in full rounds for both variants of the
    // collect sweep (which one runs is decided on the device): 128-row tiles on 512
    // resident workgroups, and 256-row tiles on 512 or 128-row tiles on 768.
    const int64_t tiles_b = p.RB == 2 ? (na + 255) / 256 : p.row_tiles;
    const double slots_b = p.RB == 2 ? 512.0 : 768.0;
    ns = 1;
    double best = -1.0;
    const int64_t ns_max = std::min<int64_t>(ns_cap, by_length);
    for (int64_t c = 1; c <= ns_max; ++c) {
      const double ga = (double)(p.row_tiles * c), gb = (double)(tiles_b * c);
      const double ea = ga / (std::ceil(ga / 512.0) * 512.0), eb = gb / (std::ceil(gb / slots_b) * slots_b);
      const double score = std::min(ea, eb);
      if (score > best + 0.02) { best = score; ns = c; }
      if (best >= 0.9) break;                                   // good enough: no more splits
    }
  }
  p.nsplit = (int)ns;
  const int64_t steps_per_split = (col_steps + ns - 1) / ns;
  p.cols_per_split = steps_per_split * bn;
  // The minima sweep computes every S-th row of B once a split of B is long enough: tau then
  // comes from 1/S of the columns.  With S = 1 the kp-th
  // smallest group minimum guarantees kp listed columns; with S > 1 the rank is chosen so that
  // about S * kp_tau columns are expected below tau, at least k of them except with small
  // probability (rows that end up with fewer, or with more than their lists hold, fail the
  // re-rank test and are recomputed).
  if (p.kc) {
    // (long rows make a sweep expensive: the tiled kernel samples as soon as 1024 columns
    // remain in the sample; measured on 16384 and 200000 columns: S = 16 beats 8, 4 and 2)
    p.stride = (int)std::max<int64_t>(1, std::min<int64_t>(16, nb / 1024));
  } else {
    // (independent of the number of splits; measured flat between half and twice this)
    p.stride = (int)std::max<int64_t>(1, std::min<int64_t>(16, col_steps / 192));
  }
  p.stride = (int)std::min<int64_t>(p.stride, steps_per_split);        // at least one tile per split
  if (p.stride == 1) {
    p.kp_tau = p.kp;
  } else {
    const double ks = (double)k / p.stride;
    p.kp_tau = std::min(p.kp, (int)std::ceil(ks + 4.0 * std::sqrt(ks) + 2.0));
    // Room for the listed columns -- in EVERY split: when B is stored in cluster order a
    // row's candidates all fall into one of them.  Their number is about S times a
    // gamma(kp_tau) variable (a little more, as two of the best sampled columns may share
    // a group); r + 5.5 sqrt(r) + 8 is beyond its 1 - 1e-6 quantile for every r.
    const double r = p.kp_tau;
    p.cap = std::max(64, (int)std::ceil(1.15 * p.stride * (r + 5.5 * std::sqrt(r) + 8.0)) + 16);
  }
  // groups: at least 8 per wanted rank, so that two of the best values rarely share a group
  const int want = (p.kp_tau + 7) / 8;
  p.rg = want <= 1 ? 1 : (want <= 2 ? 2 : (want <= 4 ? 4 : 8));
  if (p.stride == 1) p.rg = p.kp <= 32 ? 1 : (p.kp <= 64 ? 2 : (p.kp <= 128 ? 4 : 8));
  const int64_t visited = (steps_per_split + p.stride - 1) / p.stride;   // tiles per split
  int64_t nph = (p.rg + ns - 1) / ns;
  nph = std::max<int64_t>(1, std::min(nph, visited));
  p.nphase = (int)nph;
  p.cols_per_phase = (visited + nph - 1) / nph * bn * p.stride;
  p.g_raw = 64 * p.nsplit * p.nphase;
  size_t o = up256((size_t)na * p.nsplit * p.cap * sizeof(u64));
  p.o_minima = o; o += up256((size_t)na * p.g_raw * sizeof(float));
  p.o_tau = o; o += up256((size_t)na * sizeof(float));
  p.o_cnt = o; o += up256((size_t)na * p.nsplit * sizeof(int));
  p.bytes = o;
  return p;
}
}  // namespace

namespace {
struct FallbackPlan { int64_t chunk_cols; int nchunk; int64_t cap_keys; };
// Column chunks of the exact fallback for the case that every row is redone: at least 8192 columns
// each (a few hundred redone rows still make a few thousand tasks), at most 64 chunks.  From 8192
// columns on, the kernels cut finer when few rows are redone (fallback_split): cap_keys > 0 is the
// size of the buffer of partial results, which then also holds 64 rows x 64 chunks.
FallbackPlan fallback_plan(int64_t na, int64_t nb, int k) {
  FallbackPlan f;
  f.chunk_cols = std::max<int64_t>(8192, ((nb + 63) / 64 + 255) / 256 * 256);
  f.nchunk = (int)std::max<int64_t>(1, (nb + f.chunk_cols - 1) / f.chunk_cols);
  f.cap_keys = 0;
  if (nb >= 8192)
    f.cap_keys = std::max<int64_t>(f.nchunk == 1 ? 0 : na * f.nchunk * k, std::min<int64_t>(na, 64) * 64 * k);
  return f;
}
}  // namespace

size_t mfma_knn_fallback_bytes(int64_t na, int64_t nb, int k) {
  const FallbackPlan f = fallback_plan(na, nb, k);
  if (f.cap_keys > 0) return (size_t)f.cap_keys * sizeof(u64);
  return f.nchunk == 1 ? 0 : (size_t)na * f.nchunk * k * sizeof(u64);
}

size_t mfma_knn_shortlist_bytes(int64_t na, int64_t nb, int d, int k, int* nsplit_out) {
  const MfmaPlan p = make_plan(na, nb, k, d);
  *nsplit_out = p.nsplit;
  return p.bytes;
}

// which operand-precision variant is ruled out by what the host knows of the operands
static bool certainly_three(const MfmaOperand& A, const MfmaOperand& B) {
  return A.known_bf16 == 0 || B.known_bf16 == 0;
}
static bool certainly_one(const MfmaOperand& A, const MfmaOperand& B) {
  return A.known_bf16 == 1 && B.known_bf16 == 1;
}
// The two-pass variant is one more (possibly empty) launch: only for an A long enough that
// the sweeps, not the launches, are what a call costs.  The kernels get the same answer as
// a flag, so that exactly one variant takes the work.
static bool two_pass_allowed(const MfmaOperand& A) { return A.n >= 256; }
// ... and not next to the fp16 attempt (one more empty launch per sweep in nearly every call; when
// the attempt has been given up on such an operand, exactly-bf16 queries take the three-pass variant)
static bool two_pass_allowed(const MfmaOperand& A, const MfmaOperand& B) {
  return two_pass_allowed(A) && !B.try_heads_only;
}

template <int KSTEPS, int RB, int METRIC, int MODE, int PREC>
static void launch_sweep_t(const MfmaPlan& p, const MfmaOperand& A, const MfmaOperand& B, char* work,
                           hipStream_t st) {
  constexpr int D = KSTEPS * 16, NPL = PREC == 1 || PREC == 2 ? 2 : 1;
  const size_t shmem = (size_t)2 * NPL * 64 * (D + 8) * sizeof(unsigned short) + 2 * 64 * sizeof(float) +
                       (size_t)128 * RB * (sizeof(int) + sizeof(float)) +
                       4 * 128 * (sizeof(u64) + sizeof(int));
  auto kern = &mfma_sweep_kernel<KSTEPS, RB, METRIC, MODE, PREC>;
  if (shmem > 48 * 1024)
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
  const int64_t row_tiles = (A.n + 128 * RB - 1) / (128 * RB);   // (the lists are per row: any RB fits)
  const int64_t per_xcd = (row_tiles * p.nsplit + 7) / 8;         // the kernel deals the items out by XCD
  hipLaunchKernelGGL(kern, dim3((unsigned)(8 * per_xcd)), dim3(256), shmem, st,
                     PREC == 3 ? A.h16 : A.hi, A.lo, A.norm, A.info, A.n,
                     PREC == 3 ? B.h16 : B.hi, B.lo, B.norm, B.info, B.n, p.nsplit, p.cols_per_split,
                     MODE == 0 ? p.stride : 1, p.nphase, p.cols_per_phase,
                     reinterpret_cast<float*>(work + p.o_minima), p.g_raw,
                     reinterpret_cast<const float*>(work + p.o_tau), reinterpret_cast<int*>(work + p.o_cnt),
                     reinterpret_cast<u64*>(work), p.cap, (two_pass_allowed(A, B) ? 1 : 0) | (p.hbit << 1));
}

template <int KSTEPS, int METRIC, int MODE>
static void launch_sweep_k(const MfmaPlan& p, const MfmaOperand& A, const MfmaOperand& B, char* work,
                           hipStream_t st) {
  // both operand-precision variants are enqueued; the kernel that does not match the flags
  // written by operand preparation returns immediately (the flags live in device memory) --
  // unless the host already knows an operand's flag and with it which variant cannot run
  // (an operand that may be swept by its fp16 heads alone needs that variant enqueued too)
  if (B.try_heads_only && !certainly_one(A, B)) {
    if (MODE == 1 && p.RB == 2) launch_sweep_t<KSTEPS, MODE == 1 ? 2 : 1, METRIC, MODE, 3>(p, A, B, work, st);
    else launch_sweep_t<KSTEPS, 1, METRIC, MODE, 3>(p, A, B, work, st);
  }
  if (!certainly_three(A, B)) {
    if (MODE == 1 && p.RB == 2) launch_sweep_t<KSTEPS, MODE == 1 ? 2 : 1, METRIC, MODE, 0>(p, A, B, work, st);
    else launch_sweep_t<KSTEPS, 1, METRIC, MODE, 0>(p, A, B, work, st);
  }
  if (!certainly_one(A, B)) {
    // A exact and B not (integer vectors against trained centroids): two passes instead of three
    if (two_pass_allowed(A, B) && A.known_bf16 != 0 && B.known_bf16 != 1)
      launch_sweep_t<KSTEPS, 1, METRIC, MODE, 1>(p, A, B, work, st);
    launch_sweep_t<KSTEPS, 1, METRIC, MODE, 2>(p, A, B, work, st);
  }
}

template <int METRIC, int MODE, int PREC>
static void launch_sweep_kc_t(const MfmaPlan& p, const MfmaOperand& A, const MfmaOperand& B, int d,
                              char* work, hipStream_t st) {
  constexpr int NPL = PREC == 2 ? 2 : 1;
  const size_t shmem = (size_t)2 * NPL * 2 * 16 * 1024 + 2 * 256 * sizeof(float) +
                       (size_t)256 * (sizeof(int) + 2 * sizeof(float)) + 8 * 128 * (sizeof(u64) + sizeof(int));
  auto kern = &mfma_sweep_kc_kernel<METRIC, MODE, PREC>;
  (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
  const int64_t per_xcd = (p.row_tiles * p.nsplit + 7) / 8;       // the kernel deals the items out by XCD
  hipLaunchKernelGGL(kern, dim3((unsigned)(8 * per_xcd)), dim3(512), shmem, st,
                     PREC == 3 ? A.h16 : A.hi, A.lo, A.norm, A.info, A.n,
                     PREC == 3 ? B.h16 : B.hi, B.lo, B.norm, B.info, B.n, d, p.nsplit, p.cols_per_split,
                     MODE == 0 ? p.stride : 1, p.nphase, p.cols_per_phase,
                     reinterpret_cast<float*>(work + p.o_minima), p.g_raw,
                     reinterpret_cast<const float*>(work + p.o_tau), reinterpret_cast<int*>(work + p.o_cnt),
                     reinterpret_cast<u64*>(work), p.cap, p.hbit);
}

template <int MODE>
static void launch_sweep(const MfmaPlan& p, const MfmaOperand& A, const MfmaOperand& B, int d,
                         int metric, char* work, hipStream_t st) {
  if (p.kc) {   // both operand-precision variants, as below
    const bool one = !certainly_three(A, B), three = !certainly_one(A, B), f16 = B.try_heads_only && three;
    if (metric == 0) {
      if (f16) launch_sweep_kc_t<0, MODE, 3>(p, A, B, d, work, st);
      if (one) launch_sweep_kc_t<0, MODE, 0>(p, A, B, d, work, st);
      if (three) launch_sweep_kc_t<0, MODE, 2>(p, A, B, d, work, st);
    } else {
      if (f16) launch_sweep_kc_t<1, MODE, 3>(p, A, B, d, work, st);
      if (one) launch_sweep_kc_t<1, MODE, 0>(p, A, B, d, work, st);
      if (three) launch_sweep_kc_t<1, MODE, 2>(p, A, B, d, work, st);
    }
    return;
  }
#define GO(KS)                                                                      \
  do {                                                                              \
    if (metric == 0) launch_sweep_k<KS, 0, MODE>(p, A, B, work, st);                \
    else             launch_sweep_k<KS, 1, MODE>(p, A, B, work, st);                \
  } while (0)
  switch (d / 16) {
    case 2: GO(2); break;
    case 4: GO(4); break;
    case 6: GO(6); break;
    default: GO(8); break;
  }
#undef GO
}

void launch_mfma_shortlist(const MfmaOperand& A, const MfmaOperand& B, int d, int metric, int k,
                           int nsplit, u64* shortlist, int* fb_count, hipStream_t st) {
  (void)nsplit;
  const MfmaPlan p = make_plan(A.n, B.n, k, d);
  char* work = reinterpret_cast<char*>(shortlist);
  launch_sweep<0>(p, A, B, d, metric, work, st);
  const dim3 grid((unsigned)((A.n + 3) / 4)), block(256);
  float* tau = reinterpret_cast<float*>(work + p.o_tau);
  const float* minima = reinterpret_cast<const float*>(work + p.o_minima);
  switch (p.rg) {
    case 1: hipLaunchKernelGGL((tau_kernel<1>), grid, block, 0, st, minima, p.g_raw, A.n, p.kp_tau, tau, fb_count); break;
    case 2: hipLaunchKernelGGL((tau_kernel<2>), grid, block, 0, st, minima, p.g_raw, A.n, p.kp_tau, tau, fb_count); break;
    case 4: hipLaunchKernelGGL((tau_kernel<4>), grid, block, 0, st, minima, p.g_raw, A.n, p.kp_tau, tau, fb_count); break;
    default: hipLaunchKernelGGL((tau_kernel<8>), grid, block, 0, st, minima, p.g_raw, A.n, p.kp_tau, tau, fb_count); break;
  }
  launch_sweep<1>(p, A, B, d, metric, work, st);
}

void launch_rerank(const MfmaOperand& A, const MfmaOperand& B, int d, int metric, int k, int nsplit,
                   const u64* shortlist, float eps_scale, const SelectOut& out, int* fb_count,
                   int* fb_rows, u64* fb_partial, hipStream_t st) {
  (void)nsplit;
  const MfmaPlan p = make_plan(A.n, B.n, k, d);
  const int kp = p.kp;
  const int* cnt = reinterpret_cast<const int*>(reinterpret_cast<const char*>(shortlist) + p.o_cnt);
  const float* tau = reinterpret_cast<const float*>(reinterpret_cast<const char*>(shortlist) + p.o_tau);
  const int R = kp <= 64 ? 2 : 4;   // (fb_count was cleared by launch_mfma_shortlist's threshold kernel)
  const size_t sh = (size_t)64 * R * sizeof(u64) + (size_t)d * sizeof(float);
#define RR(RV, MET)                                                                               \
  hipLaunchKernelGGL((rerank_kernel<RV, MET>), dim3((unsigned)A.n), dim3(64), sh, st, shortlist,  \
                     cnt, tau, p.nsplit, p.cap, kp, A.x, B.x, B.n, d, k, A.norm, A.info, B.info,   \
                     eps_scale, out, fb_count, fb_rows)
  if (R == 2) { if (metric == 0) RR(2, 0); else RR(2, 1); }
  else        { if (metric == 0) RR(4, 0); else RR(4, 1); }
#undef RR
  // rows whose shortlist could not be proven sufficient: canon over all columns
  const int tot = select_slots_for_k(k);
  const bool tiled = d % 32 == 0;
  const size_t sh2 = (size_t)4 * tot * sizeof(u64) + (size_t)d * sizeof(float) +
                     (tiled ? (size_t)2 * 256 * 36 * sizeof(float) : 0);
  const FallbackPlan fp = fallback_plan(A.n, B.n, k);
  const int grid = (int)std::min<int64_t>(A.n * (fp.cap_keys > 0 ? 64 : fp.nchunk), 2048);   // (idle workgroups leave at once)
#define CR(RV, MET)                                                                              \
  do {                                                                                           \
    auto kern = tiled ? &canon_rows_tiled_kernel<RV, MET> : &canon_rows_kernel<RV, MET>;         \
    if (sh2 > 48 * 1024)                                                                         \
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                             \
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)sh2);           \
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), sh2, st, A.x, B.x, B.n, d,                   \
                       k, tot, fp.chunk_cols, fp.nchunk, fp.cap_keys, fb_partial, out, fb_count, fb_rows, \
                       eps_scale < 0.f ? nullptr : const_cast<PrepInfo*>(B.info), A.n);          \
    if (fp.nchunk > 1 || fp.cap_keys > 0)                                                        \
      hipLaunchKernelGGL((canon_rows_merge_kernel<RV, MET>), dim3((unsigned)std::min<int64_t>(A.n, 1024)), \
                         dim3(64), (size_t)tot * sizeof(u64), st, fb_partial, B.n, fp.chunk_cols, \
                         fp.nchunk, fp.cap_keys, k, tot, out, fb_count, fb_rows);                \
  } while (0)
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
