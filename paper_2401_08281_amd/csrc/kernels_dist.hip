// Canon distance tiles for gfx950.
//
// "Canon" is the arithmetic every bit-exact decision of the library is taken
// in (list assignment, probe order): for a pair (a, b) of fp32 vectors one
// sequential chain over the dimensions t = 0..d-1,
//     L2: diff = a[t] - b[t] (rounded to fp32); acc = fma(diff, diff, acc)
//     IP: acc = fma(a[t], b[t], acc)
// starting from acc = +0.  Each accumulator below is such a chain; tiling is
// across pairs only, never across t, so the result is independent of the
// tiling.  Padding dimensions contribute fma(0, 0, acc) = acc exactly.
//
// Work decomposition: a workgroup of 256 lanes (4 wavefronts) owns a 64 x 64
// tile of pairs; each lane owns a 4 x 4 register block.  Both operand tiles
// go through LDS, transposed to [t][row], so that the inner loop issues two
// 128-bit LDS reads (one broadcast, one conflict-free) per 32 FMAs + 16 SUBs.
#include "common.hpp"
#include "internal.hpp"

namespace {

constexpr int TM = 64;       // A rows per tile
constexpr int TN = 64;       // B rows per tile
constexpr int KT = 32;       // dimensions per LDS stage
constexpr int TS = TM + 4;   // padded row stride of the transposed tile (keeps 16-B alignment)

// Loads rows [row0, row0 + 64) x dims [t0, t0 + KT) of P into dst[t][row], zero-padded.
template <bool VEC>
__device__ __forceinline__ void load_tile(const float* __restrict__ P, int64_t nrows, int d,
                                          int64_t row0, int t0, float (*dst)[TS]) {
  const int tid = threadIdx.x;
  if (VEC) {
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
      const int r = (tid >> 3) + 32 * pass;
      const int t = (tid & 7) * 4;
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (row0 + r < nrows && t0 + t < d)   // d % 4 == 0: the whole float4 is in range
        v = *reinterpret_cast<const float4*>(P + (row0 + r) * (int64_t)d + t0 + t);
      dst[t + 0][r] = v.x; dst[t + 1][r] = v.y; dst[t + 2][r] = v.z; dst[t + 3][r] = v.w;
    }
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int idx = tid + 256 * e;
      const int r = idx >> 5, t = idx & 31;
      float v = 0.f;
      if (row0 + r < nrows && t0 + t < d) v = P[(row0 + r) * (int64_t)d + t0 + t];
      dst[t][r] = v;
    }
  }
}

// acc[i][j] += canon contribution of dims [t0, t0+KT) for rows (ty*4+i, tx*4+j)
template <int METRIC>
__device__ __forceinline__ void tile_fma(const float (*As)[TS], const float (*Bs)[TS], int ty,
                                         int tx, float acc[4][4]) {
#pragma unroll 8
  for (int t = 0; t < KT; ++t) {
    const float4 a4 = *reinterpret_cast<const float4*>(&As[t][ty * 4]);
    const float4 b4 = *reinterpret_cast<const float4*>(&Bs[t][tx * 4]);
    const float a[4] = {a4.x, a4.y, a4.z, a4.w};
    const float b[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (METRIC == 0) {
          const float diff = a[i] - b[j];
          acc[i][j] = __builtin_fmaf(diff, diff, acc[i][j]);
        } else {
          acc[i][j] = __builtin_fmaf(a[i], b[j], acc[i][j]);
        }
      }
  }
}

template <int METRIC, bool VEC>
__global__ __launch_bounds__(256) void canon_matrix_kernel(const float* __restrict__ A, int64_t na,
                                                           const float* __restrict__ B, int64_t nb,
                                                           int d, float* __restrict__ out,
                                                           int64_t ldo, int64_t tiles_b) {
  __shared__ __attribute__((aligned(16))) float As[KT][TS];
  __shared__ __attribute__((aligned(16))) float Bs[KT][TS];
  const int64_t ta = blockIdx.x / tiles_b, tb = blockIdx.x % tiles_b;
  const int64_t a0 = ta * TM, b0 = tb * TN;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  float acc[4][4] = {};
  for (int t0 = 0; t0 < d; t0 += KT) {
    load_tile<VEC>(A, na, d, a0, t0, As);
    load_tile<VEC>(B, nb, d, b0, t0, Bs);
    __syncthreads();
    tile_fma<METRIC>(As, Bs, ty, tx, acc);
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t a = a0 + ty * 4 + i;
    if (a >= na) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int64_t b = b0 + tx * 4 + j;
      if (b < nb) out[a * ldo + b] = acc[i][j];
    }
  }
}

// One workgroup per (A tile, B split): walks the B tiles of its split and keeps,
// per A row, the best key seen; one 64-bit atomicMin per row at the end.
template <int METRIC, bool VEC>
__global__ __launch_bounds__(256) void canon_argbest_kernel(const float* __restrict__ A, int64_t na,
                                                            const float* __restrict__ B, int64_t nb,
                                                            int d, u64* __restrict__ best,
                                                            int nsplit) {
  __shared__ __attribute__((aligned(16))) float As[KT][TS];
  __shared__ __attribute__((aligned(16))) float Bs[KT][TS];
  const int64_t ta = blockIdx.x / nsplit;
  const int split = blockIdx.x % nsplit;
  const int64_t a0 = ta * TM;
  const int64_t tiles_b = (nb + TN - 1) / TN;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  u64 bk[4] = {KEY_EMPTY, KEY_EMPTY, KEY_EMPTY, KEY_EMPTY};
  for (int64_t tb = split; tb < tiles_b; tb += nsplit) {
    const int64_t b0 = tb * TN;
    float acc[4][4] = {};
    for (int t0 = 0; t0 < d; t0 += KT) {
      load_tile<VEC>(A, na, d, a0, t0, As);
      load_tile<VEC>(B, nb, d, b0, t0, Bs);
      __syncthreads();
      tile_fma<METRIC>(As, Bs, ty, tx, acc);
      __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int64_t b = b0 + tx * 4 + j;
        if (b < nb) {
          const u64 key = make_key(acc[i][j], (u32)b, METRIC);
          bk[i] = key < bk[i] ? key : bk[i];
        }
      }
  }
  // the 16 lanes sharing ty are consecutive lanes of one wavefront
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    u64 v = bk[i];
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) {
      const u64 o = __shfl_xor(v, off);
      v = o < v ? o : v;
    }
    const int64_t a = a0 + ty * 4 + i;
    if (tx == 0 && a < na && v != KEY_EMPTY) atomicMin(&best[a], v);
  }
}

inline bool vec_ok(const float* A, const float* B, int d) {
  return d % 4 == 0 && (reinterpret_cast<uintptr_t>(A) & 15) == 0 &&
         (reinterpret_cast<uintptr_t>(B) & 15) == 0;
}

}  // namespace

void launch_canon_matrix(const float* A, int64_t na, const float* B, int64_t nb, int d, int metric,
                         float* out, int64_t ldo, hipStream_t st) {
  if (na <= 0 || nb <= 0) return;
  const int64_t tiles_a = (na + TM - 1) / TM, tiles_b = (nb + TN - 1) / TN;
  const dim3 grid((unsigned)(tiles_a * tiles_b)), block(256);
  const bool vec = vec_ok(A, B, d);
#define LAUNCH(MET, VEC) \
  hipLaunchKernelGGL((canon_matrix_kernel<MET, VEC>), grid, block, 0, st, A, na, B, nb, d, out, ldo, tiles_b)
  if (metric == 0) { if (vec) LAUNCH(0, true); else LAUNCH(0, false); }
  else             { if (vec) LAUNCH(1, true); else LAUNCH(1, false); }
#undef LAUNCH
}

void launch_canon_argbest(const float* A, int64_t na, const float* B, int64_t nb, int d,
                          int metric, u64* best, hipStream_t st) {
  if (na <= 0 || nb <= 0) return;
  const int64_t tiles_a = (na + TM - 1) / TM, tiles_b = (nb + TN - 1) / TN;
  // enough workgroups to fill 256 CUs several times over, but no more splits than B tiles
  int64_t nsplit = (4096 + tiles_a - 1) / tiles_a;
  if (nsplit > tiles_b) nsplit = tiles_b;
  if (nsplit < 1) nsplit = 1;
  const dim3 grid((unsigned)(tiles_a * nsplit)), block(256);
  const bool vec = vec_ok(A, B, d);
#define LAUNCH(MET, VEC) \
  hipLaunchKernelGGL((canon_argbest_kernel<MET, VEC>), grid, block, 0, st, A, na, B, nb, d, best, (int)nsplit)
  if (metric == 0) { if (vec) LAUNCH(0, true); else LAUNCH(0, false); }
  else             { if (vec) LAUNCH(1, true); else LAUNCH(1, false); }
#undef LAUNCH
}
