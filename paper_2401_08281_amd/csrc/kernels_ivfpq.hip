// IVF-PQ kernels for gfx950: residual PQ encoding, list re-layout, the fused
// look-up-table build + ADC scan + wavefront k-selection, and the merge across
// probe splits.
#include <algorithm>

#include "common.hpp"
#include "internal.hpp"

namespace {

// ---------------------------------------------------------------------------
// PQ encoding (Sec. 4.1 product quantizer; Sec. 5.1 residual encoding).
// One lane per (vector, sub-quantizer m); a workgroup covers 256 vectors of
// one m and keeps that sub-codebook in LDS, read as broadcasts.  The residual
// is one fp32 subtraction per component; the nearest codeword is taken on the
// canon chain (diff, fma) over the dsub components; a strict '<' while walking
// j upward keeps the smaller code on ties.
// ---------------------------------------------------------------------------
template <int DSUB>
__global__ __launch_bounds__(256) void pq_encode_kernel(const float* __restrict__ x, int64_t n,
                                                        int d, int dsub_rt, int K,
                                                        const int32_t* __restrict__ list_of,
                                                        const float* __restrict__ centroids,
                                                        const float* __restrict__ codebooks, int M,
                                                        uint8_t* __restrict__ tmp_codes) {
  extern __shared__ __attribute__((aligned(16))) float T[];  // [K][dsub]
  const int m = blockIdx.y;
  const int dsub = DSUB > 0 ? DSUB : dsub_rt;
  const float* __restrict__ Tm = codebooks + (int64_t)m * K * dsub;
  for (int e = threadIdx.x; e < K * dsub; e += 256) T[e] = Tm[e];
  __syncthreads();
  const int64_t i = blockIdx.x * 256ll + threadIdx.x;
  if (i >= n) return;
  const float* __restrict__ xi = x + i * d + m * dsub;
  const float* __restrict__ c = centroids + (int64_t)list_of[i] * d + m * dsub;
  int best = 0;
  float bd = __builtin_inff();
  if (DSUB > 0) {
    float r[DSUB > 0 ? DSUB : 1];
#pragma unroll
    for (int u = 0; u < DSUB; ++u) r[u] = xi[u] - c[u];
    for (int j = 0; j < K; ++j) {
      float acc = 0.f;
#pragma unroll
      for (int u = 0; u < DSUB; ++u) {
        const float diff = r[u] - T[j * DSUB + u];
        acc = __builtin_fmaf(diff, diff, acc);
      }
      if (acc < bd) { bd = acc; best = j; }
    }
  } else {
    for (int j = 0; j < K; ++j) {
      float acc = 0.f;
      for (int u = 0; u < dsub; ++u) {
        const float r = xi[u] - c[u];
        const float diff = r - T[j * dsub + u];
        acc = __builtin_fmaf(diff, diff, acc);
      }
      if (acc < bd) { bd = acc; best = j; }
    }
  }
  tmp_codes[i * M + m] = (uint8_t)best;
}

// same, sub-codebook read from global memory (sub-codebooks too large for LDS)
__global__ __launch_bounds__(256) void pq_encode_global_kernel(
    const float* __restrict__ x, int64_t n, int d, int dsub, int K,
    const int32_t* __restrict__ list_of, const float* __restrict__ centroids,
    const float* __restrict__ codebooks, int M, uint8_t* __restrict__ tmp_codes) {
  const int m = blockIdx.y;
  const float* __restrict__ T = codebooks + (int64_t)m * K * dsub;
  const int64_t i = blockIdx.x * 256ll + threadIdx.x;
  if (i >= n) return;
  const float* __restrict__ xi = x + i * d + m * dsub;
  const float* __restrict__ c = centroids + (int64_t)list_of[i] * d + m * dsub;
  int best = 0;
  float bd = __builtin_inff();
  for (int j = 0; j < K; ++j) {
    float acc = 0.f;
    for (int u = 0; u < dsub; ++u) {
      const float r = xi[u] - c[u];
      const float diff = r - T[j * dsub + u];
      acc = __builtin_fmaf(diff, diff, acc);
    }
    if (acc < bd) { bd = acc; best = j; }
  }
  tmp_codes[i * M + m] = (uint8_t)best;
}

// ---------------------------------------------------------------------------
// list storage
// ---------------------------------------------------------------------------
// Squared norm of the decoded vector x' = c_list + concat_m T_m[c_m] of every new entry
// (Sec. 4.3: the norm stored next to the code for the decomposition |q|^2 + |x'|^2 - 2<q,x'>):
// one fp32 addition per component, squares accumulated by one fma chain in dimension order.
// One lane per vector; tmp_codes holds one byte per (vector, m).
__global__ void pq_norms_kernel(const uint8_t* __restrict__ tmp_codes, int64_t n, int d, int dsub,
                                int K, int M, const int32_t* __restrict__ list_of,
                                const float* __restrict__ centroids,
                                const float* __restrict__ codebooks, float* __restrict__ tmp_norms) {
  const int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i >= n) return;
  const float* __restrict__ c = centroids + (int64_t)list_of[i] * d;
  float acc = 0.f;
  for (int m = 0; m < M; ++m) {
    const float* __restrict__ T = codebooks + ((int64_t)m * K + tmp_codes[i * M + m]) * dsub;
    for (int u = 0; u < dsub; ++u) {
      const float xt = c[m * dsub + u] + T[u];
      acc = __builtin_fmaf(xt, xt, acc);
    }
  }
  tmp_norms[i] = acc;
}

// norms[i] = |row i|^2 as one fma chain in dimension order.  One lane per row.
__global__ void row_norms_kernel(const float* __restrict__ x, int64_t n, int d,
                                 float* __restrict__ norms) {
  const int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i >= n) return;
  float acc = 0.f;
  for (int t = 0; t < d; ++t) acc = __builtin_fmaf(x[i * d + t], x[i * d + t], acc);
  norms[i] = acc;
}

__global__ void move_old_kernel(const uint8_t* __restrict__ old_codes,
                                const int64_t* __restrict__ old_ids,
                                const float* __restrict__ old_norms, int64_t old_total,
                                const int64_t* __restrict__ old_off,
                                const int64_t* __restrict__ new_off, int nlist, int cs,
                                uint8_t* __restrict__ codes, int64_t* __restrict__ ids,
                                float* __restrict__ norms) {
  const int64_t p = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (p >= old_total) return;
  const int l = list_of_position(old_off, nlist, p);
  const int64_t np = new_off[l] + (p - old_off[l]);
  ids[np] = old_ids[p];
  if (norms) norms[np] = old_norms[p];
  for (int b = 0; b < cs; ++b) codes[np * cs + b] = old_codes[p * cs + b];
}

__global__ void scatter_new_kernel(const uint8_t* __restrict__ tmp_codes,
                                   const int64_t* __restrict__ new_ids, int64_t id_base,
                                   const float* __restrict__ tmp_norms,
                                   const int64_t* __restrict__ dest, int64_t n, int M, int nbits,
                                   int cs, uint8_t* __restrict__ codes, int64_t* __restrict__ ids,
                                   float* __restrict__ norms) {
  const int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int64_t p = dest[i];
  ids[p] = new_ids ? new_ids[i] : id_base + i;
  if (norms) norms[p] = tmp_norms[i];
  const uint8_t* __restrict__ t = tmp_codes + i * M;
  if (nbits == 8) {
    for (int b = 0; b < cs; ++b) codes[p * cs + b] = t[b];
  } else {  // two 4-bit codes per byte, even m in the low nibble
    for (int b = 0; b < cs; ++b) codes[p * cs + b] = (uint8_t)(t[2 * b] | (t[2 * b + 1] << 4));
  }
}

__global__ void list_of_storage_kernel(const int64_t* __restrict__ off, int nlist, int64_t total,
                                       int32_t* __restrict__ list_of) {
  const int64_t p = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (p < total) list_of[p] = list_of_position(off, nlist, p);
}

__global__ void list_sizes_kernel(const int64_t* __restrict__ off, int nlist,
                                  int64_t* __restrict__ sizes) {
  const int l = blockIdx.x * blockDim.x + threadIdx.x;
  if (l < nlist) sizes[l] = off[l + 1] - off[l];
}

// ---------------------------------------------------------------------------
// Fused LUT build + ADC scan + k-selection (Sec. 4 Eq. 10 (ADC) and Eq. 14 (look-up
// tables); Sec. 5.1; App. A.3 "GPU Faiss": tables staged in on-chip memory, lists
// streamed from HBM).
//
// One workgroup (4 wavefronts) serves one query and a contiguous range of its
// probes.  Per probed list l:
//   L2: r = q - c_l (fp32), LUT[m][j] = canon_l2(r_m, T_m[j]) into LDS;
//   IP: LUT[m][j] = canon_ip(q_m, T_m[j]) once per workgroup, bias = <q, c_l>
//       (the coarse score of the probe);
// then every lane takes one code of the list per step (codes of a list are
// contiguous, so a wavefront reads 64 * code_size consecutive bytes), sums
// its M table entries in m order and offers (distance, storage position) to
// its wavefront's WaveSelect.  At the end wavefront 0 absorbs the other
// three and writes the k best keys of this (query, split).
// ---------------------------------------------------------------------------
template <int NBITS>
__device__ __forceinline__ float adc_bytes(const float* __restrict__ lut, u32 word, int m_base,
                                           float dist) {
  // consumes 4 code bytes = 4 (NBITS=8) or 8 (NBITS=4) sub-quantizers starting at m_base
  constexpr int K = 1 << NBITS;
#pragma unroll
  for (int b = 0; b < 4; ++b) {
    const u32 byte = (word >> (8 * b)) & 0xFFu;
    if (NBITS == 8) {
      dist += lut[(m_base + b) * K + byte];
    } else {
      dist += lut[(m_base + 2 * b) * K + (byte & 15u)];
      dist += lut[(m_base + 2 * b + 1) * K + (byte >> 4)];
    }
  }
  return dist;
}

// Look-ups of one 32-bit word of 4-bit codes (8 sub-quantizers from m_base on) in tables that
// start at the beginning of the workgroup's LDS.  The byte offset of an entry, nibble * 4, is
// one instruction per nibble: with lo = word << 2 and hi = word >> 2 the scaled low / high
// nibble of code byte b sits in bits 2..5 of byte b of lo / hi, and a byte-selecting AND with
// 0x3C (v_and_b32_sdwa) isolates it; the table's own offset is the load's immediate.  The
// scan of 4-bit codes is bound by its vector instructions: this form has 2.25 per look-up
// (with the addition) where shift-and-mask extraction and address arithmetic have 3.
template <int B>
__device__ __forceinline__ u32 byte_and(u32 x, u32 mask) {
  u32 r;
  if constexpr (B == 0) asm("v_and_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_0 src1_sel:DWORD" : "=v"(r) : "v"(x), "v"(mask));
  if constexpr (B == 1) asm("v_and_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_1 src1_sel:DWORD" : "=v"(r) : "v"(x), "v"(mask));
  if constexpr (B == 2) asm("v_and_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_2 src1_sel:DWORD" : "=v"(r) : "v"(x), "v"(mask));
  if constexpr (B == 3) asm("v_and_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_3 src1_sel:DWORD" : "=v"(r) : "v"(x), "v"(mask));
  return r;
}
// (the tables are addressed as LDS address 0 + offset: the caller has checked that they start there)
typedef __attribute__((address_space(3))) const float* lds_cfloat_ptr;
template <int B>
__device__ __forceinline__ float adc_nibble_pair(u32 lo, u32 hi, u32 mask, int m_base, float dist) {
  const u32 o0 = byte_and<B>(lo, mask), o1 = byte_and<B>(hi, mask);
  dist += *reinterpret_cast<lds_cfloat_ptr>((uintptr_t)(o0 + (u32)((m_base + 2 * B) * 64)));
  dist += *reinterpret_cast<lds_cfloat_ptr>((uintptr_t)(o1 + (u32)((m_base + 2 * B + 1) * 64)));
  return dist;
}
__device__ __forceinline__ float adc_word4(u32 word, int m_base, float dist) {
  const u32 lo = word << 2, hi = word >> 2, mask = 0x3Cu;
  dist = adc_nibble_pair<0>(lo, hi, mask, m_base, dist);
  dist = adc_nibble_pair<1>(lo, hi, mask, m_base, dist);
  dist = adc_nibble_pair<2>(lo, hi, mask, m_base, dist);
  dist = adc_nibble_pair<3>(lo, hi, mask, m_base, dist);
  return dist;
}

template <int NBITS, int R>
__global__ __launch_bounds__(256) void ivfpq_scan_kernel(
    const float* __restrict__ q, int d, int mode, int M, int dsub,
    const float* __restrict__ centroids, const float* __restrict__ codebooks,
    const int32_t* __restrict__ probes, const float* __restrict__ cdist, int nprobe, int ppb,
    int nsplit, const int64_t* __restrict__ list_off, const uint8_t* __restrict__ codes,
    const float* __restrict__ norms, const float* __restrict__ cnorm, int cs, int k, int tot,
    KeySink sink) {
  // mode 0: L2, one table of squared residual distances per (query, list); mode 1: inner
  // product, one table per query, cdist = <q, c_l>; mode 2: L2 through stored norms (Sec. 4.3):
  // one table -2 <q_m, T_m[j]> per query; per list |q|^2 - 2 <q, c_l> = |q - c_l|^2 - |c_l|^2,
  // the coarse distance minus the centroid's norm; norms = |x'|^2 per code
  constexpr int K = 1 << NBITS;
  const int metric = mode == 1 ? 1 : 0;                         // ordering of the keys
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  // (the tables come first, see adc_word4)
  float* lut = reinterpret_cast<float*>(smem);                  // M * K
  float* rs = lut + M * K;                                      // d
  u64* slots = reinterpret_cast<u64*>(rs + ((d + 1) & ~1));     // 4 * tot
  const bool lut_at_zero =
      (u32)(uintptr_t)((__attribute__((address_space(3))) unsigned char*)smem) == 0u &&
      M * K * (int)sizeof(float) <= 65536;

  const int64_t qi = blockIdx.x / nsplit;
  const int split = blockIdx.x % nsplit;
  const int wave = threadIdx.x >> 6, lane = lane_id();
  const float* __restrict__ qv = q + qi * d;
  const int p_begin = split * ppb;
  const int p_end = min(nprobe, p_begin + ppb);

  WaveSelect<R> ws;
  ws.init(slots + wave * tot, tot, k);

  if (mode != 0) {  // per-query tables
    for (int e = threadIdx.x; e < M * K; e += 256) {
      const int m = e >> NBITS;
      const float* __restrict__ T = codebooks + (int64_t)e * dsub;
      float acc = 0.f;
      for (int u = 0; u < dsub; ++u) acc = __builtin_fmaf(qv[m * dsub + u], T[u], acc);
      lut[e] = mode == 2 ? -2.f * acc : acc;
    }
    __syncthreads();
  }

  for (int p = p_begin; p < p_end; ++p) {
    const int l = probes[qi * nprobe + p];
    if (l < 0) continue;
    const int64_t begin = list_off[l], end = list_off[l + 1];
    if (begin == end) continue;  // uniform over the workgroup
    float bias = 0.f;
    if (mode == 0) {
      const float* __restrict__ c = centroids + (int64_t)l * d;
      __syncthreads();  // previous list's scan is done with lut
      for (int t = threadIdx.x; t < d; t += 256) rs[t] = qv[t] - c[t];
      __syncthreads();
      for (int e = threadIdx.x; e < M * K; e += 256) {
        const int m = e >> NBITS;
        const float* __restrict__ T = codebooks + (int64_t)e * dsub;
        const float* r = rs + m * dsub;
        float acc = 0.f;
        for (int u = 0; u < dsub; ++u) {
          const float diff = r[u] - T[u];
          acc = __builtin_fmaf(diff, diff, acc);
        }
        lut[e] = acc;
      }
      __syncthreads();
    } else {
      bias = cdist[qi * nprobe + p];
      if (mode == 2) bias -= cnorm[l];
    }
    for (int64_t i0 = begin + wave * VS_WAVE; i0 < end; i0 += 4 * VS_WAVE) {
      const int64_t i = i0 + lane;
      const bool valid = i < end;
      float dist = bias;
      if (valid) {
        if (mode == 2) dist += norms[i];
        const uint8_t* __restrict__ cp = codes + i * cs;
        if ((cs & 15) == 0) {
          for (int w = 0; w < (cs >> 4); ++w) {
            const uint4 v = reinterpret_cast<const uint4*>(cp)[w];
            const int mb = w * (NBITS == 8 ? 16 : 32);
            if (NBITS == 4 && lut_at_zero) {
              dist = adc_word4(v.x, mb, dist);
              dist = adc_word4(v.y, mb + 8, dist);
              dist = adc_word4(v.z, mb + 16, dist);
              dist = adc_word4(v.w, mb + 24, dist);
            } else {
              dist = adc_bytes<NBITS>(lut, v.x, mb, dist);
              dist = adc_bytes<NBITS>(lut, v.y, mb + (NBITS == 8 ? 4 : 8), dist);
              dist = adc_bytes<NBITS>(lut, v.z, mb + (NBITS == 8 ? 8 : 16), dist);
              dist = adc_bytes<NBITS>(lut, v.w, mb + (NBITS == 8 ? 12 : 24), dist);
            }
          }
        } else if ((cs & 3) == 0) {
          for (int w = 0; w < (cs >> 2); ++w) {
            if (NBITS == 4 && lut_at_zero) dist = adc_word4(reinterpret_cast<const u32*>(cp)[w], w * 8, dist);
            else dist = adc_bytes<NBITS>(lut, reinterpret_cast<const u32*>(cp)[w], w * (NBITS == 8 ? 4 : 8), dist);
          }
        } else {
          for (int b = 0; b < cs; ++b) {
            const u32 byte = cp[b];
            if (NBITS == 8) dist += lut[b * K + byte];
            else { dist += lut[(2 * b) * K + (byte & 15u)]; dist += lut[(2 * b + 1) * K + (byte >> 4)]; }
          }
        }
      }
      if (mode == 2) dist = fmaxf(dist, 0.f);   // the expanded square can round below zero
      ws.push(valid, make_key(dist, (u32)i, metric));
    }
  }
  ws.finish();
  __syncthreads();
  block_rank_merge(slots, tot, 4, k, sink, ((int64_t)qi * nsplit + split) * k);
}

// ---------------------------------------------------------------------------
// The same scan for codes of 16, 32 or 64 bytes (W16 = code size / 16), software
// pipelined: the workgroup walks over the chunks of 256 codes of all its lists as one
// sequence, and the codes of the next chunk -- of the same list or of the next
// non-empty one -- are requested before the current chunk is summed, so a short list
// costs no exposed memory latency beyond the first one of the item.  Requests are
// clamped into the code array; lanes past the end of a list are masked when consumed.
// ---------------------------------------------------------------------------
template <int NBITS, int R, int W16>
__global__ __launch_bounds__(256) void ivfpq_scan_pipe_kernel(
    const float* __restrict__ q, int d, int mode, int M, int dsub,
    const float* __restrict__ centroids, const float* __restrict__ codebooks,
    const int32_t* __restrict__ probes, const float* __restrict__ cdist, int nprobe, int ppb,
    int nsplit, const int64_t* __restrict__ list_off, const uint8_t* __restrict__ codes,
    const float* __restrict__ norms, const float* __restrict__ cnorm, int64_t ntotal, int k, int tot,
    KeySink sink) {
  constexpr int K = 1 << NBITS;
  constexpr int MPW = NBITS == 8 ? 16 : 32;                      // sub-quantizers per 16 code bytes
  const int metric = mode == 1 ? 1 : 0;                         // ordering of the keys
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  // (the tables come first: with no static LDS in this kernel they start at LDS address 0, and
  // the 4-bit look-ups then carry a table's offset as an immediate; checked, not assumed)
  float* lut = reinterpret_cast<float*>(smem);                  // M * K
  const bool lut_at_zero =
      (u32)(uintptr_t)((__attribute__((address_space(3))) unsigned char*)smem) == 0u &&
      M * K * (int)sizeof(float) <= 65536;
  float* rs = lut + M * K;                                      // d (+ 1 to keep what follows aligned)
  int64_t* s_begin = reinterpret_cast<int64_t*>(rs + ((d + 1) & ~1));   // ppb
  int64_t* s_end = s_begin + ppb;                               // ppb
  int32_t* s_list = reinterpret_cast<int32_t*>(s_end + ppb);    // ppb
  u64* slots = reinterpret_cast<u64*>(                          // 4 * tot
      (reinterpret_cast<uintptr_t>(s_list + ppb) + 7) & ~(uintptr_t)7);

  const int64_t qi = blockIdx.x / nsplit;
  const int split = blockIdx.x % nsplit;
  const int tid = threadIdx.x, wave = tid >> 6;
  const float* __restrict__ qv = q + qi * d;
  const int p_begin = split * ppb;
  const int np = ntotal > 0 ? max(0, min(nprobe, p_begin + ppb) - p_begin) : 0;
  const int64_t last = ntotal > 0 ? ntotal - 1 : 0;
  const int cs = 16 * W16;

  WaveSelect<R> ws;
  ws.init(slots + wave * tot, tot, k);
  for (int p = tid; p < np; p += 256) {
    const int l = probes[qi * nprobe + p_begin + p];
    s_list[p] = l >= 0 ? l : 0;
    s_begin[p] = l >= 0 ? list_off[l] : 0;
    s_end[p] = l >= 0 ? list_off[l + 1] : 0;
  }
  if (mode != 0) {  // per-query tables
    for (int e = tid; e < M * K; e += 256) {
      const int m = e >> NBITS;
      const float* __restrict__ T = codebooks + (int64_t)e * dsub;
      float acc = 0.f;
      for (int u = 0; u < dsub; ++u) acc = __builtin_fmaf(qv[m * dsub + u], T[u], acc);
      lut[e] = mode == 2 ? -2.f * acc : acc;
    }
  }
  __syncthreads();

  int p = 0;
  while (p < np && s_begin[p] == s_end[p]) ++p;                 // first non-empty list (uniform)
  int64_t base = p < np ? s_begin[p] : 0;                       // first code of the current chunk
  u32x4 cw[W16], cwn[W16];
  float nrm = 0.f, nrmn = 0.f;
  if (p < np) {
    const int64_t i = min(base + tid, last);
#pragma unroll
    for (int w = 0; w < W16; ++w) cw[w] = reinterpret_cast<const u32x4*>(codes + i * cs)[w];
    if (mode == 2) nrm = norms[i];
  }
  bool first = true;                                            // first chunk of its list
  float bias = 0.f;
  while (p < np) {
    const int64_t end = s_end[p];
    int pn = p;
    int64_t base_n = base + 256;
    if (base_n >= end) {
      pn = p + 1;
      while (pn < np && s_begin[pn] == s_end[pn]) ++pn;
      base_n = pn < np ? s_begin[pn] : 0;
    }
    if (pn < np) {
      const int64_t i = min(base_n + tid, last);
#pragma unroll
      for (int w = 0; w < W16; ++w) cwn[w] = reinterpret_cast<const u32x4*>(codes + i * cs)[w];
      if (mode == 2) nrmn = norms[i];
    }
    if (first) {
      const int l = s_list[p];
      if (mode == 0) {
        const float* __restrict__ c = centroids + (int64_t)l * d;
        __syncthreads();  // the previous list's scan is done with lut
        for (int t = tid; t < d; t += 256) rs[t] = qv[t] - c[t];
        __syncthreads();
        for (int e = tid; e < M * K; e += 256) {
          const int m = e >> NBITS;
          const float* __restrict__ T = codebooks + (int64_t)e * dsub;
          const float* r = rs + m * dsub;
          float acc = 0.f;
          for (int u = 0; u < dsub; ++u) {
            const float diff = r[u] - T[u];
            acc = __builtin_fmaf(diff, diff, acc);
          }
          lut[e] = acc;
        }
        __syncthreads();
        bias = 0.f;
      } else {
        bias = cdist[qi * nprobe + p_begin + p];
        if (mode == 2) bias -= cnorm[l];
      }
    }
    const int64_t i = base + tid;
    const bool valid = i < end;
    float dist = mode == 2 ? bias + nrm : bias;
    if (valid) {
#pragma unroll
      for (int w = 0; w < W16; ++w) {
        if (NBITS == 4 && lut_at_zero) {
          dist = adc_word4(cw[w].x, w * MPW, dist);
          dist = adc_word4(cw[w].y, w * MPW + MPW / 4, dist);
          dist = adc_word4(cw[w].z, w * MPW + MPW / 2, dist);
          dist = adc_word4(cw[w].w, w * MPW + 3 * (MPW / 4), dist);
        } else {
          dist = adc_bytes<NBITS>(lut, cw[w].x, w * MPW, dist);
          dist = adc_bytes<NBITS>(lut, cw[w].y, w * MPW + MPW / 4, dist);
          dist = adc_bytes<NBITS>(lut, cw[w].z, w * MPW + MPW / 2, dist);
          dist = adc_bytes<NBITS>(lut, cw[w].w, w * MPW + 3 * (MPW / 4), dist);
        }
      }
    }
    if (mode == 2) dist = fmaxf(dist, 0.f);     // the expanded square can round below zero
    ws.push(valid, make_key(dist, (u32)i, metric));
    first = pn != p;
    p = pn;
    base = base_n;
#pragma unroll
    for (int w = 0; w < W16; ++w) cw[w] = cwn[w];
    nrm = nrmn;
  }
  ws.finish();
  __syncthreads();
  block_rank_merge(slots, tot, 4, k, sink, ((int64_t)qi * nsplit + split) * k);
}

// ---------------------------------------------------------------------------
// Register-resident-codebook variant for 8-bit codes (K = 256) and shapes known
// at compile time.  Lane j of the workgroup owns codeword j of EVERY
// sub-quantizer: M * DSUB floats in registers, loaded once per workgroup.  The
// workgroups are persistent: each walks over (query, probe split) items, so
// the codebook is read from memory once per workgroup, not once per list.
// Building a table then costs, per lane, M * DSUB (sub, fma) pairs against the
// residual, which every lane reads from LDS as broadcasts, and M conflict-free
// LDS stores.  The first 256 codes of a list are requested from memory before
// the table is built, so their latency hides under the arithmetic.
// ---------------------------------------------------------------------------
template <int M>
struct CodeWords {           // one PQ code of M bytes held in registers
  static constexpr int W = M / 4;
  u32 w[W];
  __device__ __forceinline__ void load(const uint8_t* __restrict__ p) {
    if constexpr (M % 16 == 0) {
#pragma unroll
      for (int i = 0; i < M / 16; ++i) {
        const uint4 v = reinterpret_cast<const uint4*>(p)[i];
        w[4 * i] = v.x; w[4 * i + 1] = v.y; w[4 * i + 2] = v.z; w[4 * i + 3] = v.w;
      }
    } else if constexpr (M % 8 == 0) {
#pragma unroll
      for (int i = 0; i < M / 8; ++i) {
        const uint2 v = reinterpret_cast<const uint2*>(p)[i];
        w[2 * i] = v.x; w[2 * i + 1] = v.y;
      }
    } else {
#pragma unroll
      for (int i = 0; i < W; ++i) w[i] = reinterpret_cast<const u32*>(p)[i];
    }
  }
  __device__ __forceinline__ float adc(const float* __restrict__ lut, float dist) const {
#pragma unroll
    for (int i = 0; i < W; ++i) dist = adc_bytes<8>(lut, w[i], 4 * i, dist);
    return dist;
  }
  // the same for tables whose rows are KP floats apart
  template <int KP>
  __device__ __forceinline__ float adc_rows(const float* __restrict__ lut, float dist) const {
#pragma unroll
    for (int i = 0; i < W; ++i)
#pragma unroll
      for (int b = 0; b < 4; ++b) dist += lut[(4 * i + b) * KP + ((w[i] >> (8 * b)) & 0xFFu)];
    return dist;
  }
};

#ifdef VS_SCAN_TIMING
// debug builds only: cycles spent per phase, summed over wavefront 0 of every workgroup
__device__ unsigned long long g_scan_cycles[8];
#define TICK(slot)                                                        \
  do {                                                                    \
    if (tid == 0) {                                                       \
      const unsigned long long now_ = clock64();                     \
      tacc[slot] += now_ - tprev;                                         \
      tprev = now_;                                                       \
    }                                                                     \
  } while (0)
#else
#define TICK(slot) do {} while (0)
#endif

template <int M, int DSUB, int METRIC, int R, int NBUF>
__global__ __launch_bounds__(256) void ivfpq_scan_reg_kernel(
    const float* __restrict__ q, const float* __restrict__ centroids,
    const float* __restrict__ codebooks, const int32_t* __restrict__ probes,
    const float* __restrict__ cdist, int nprobe, int ppb, int nsplit, int64_t nitems,
    const int64_t* __restrict__ list_off, const uint8_t* __restrict__ codes,
    const float* __restrict__ norms, const float* __restrict__ cnorm, int64_t ntotal, int k, int tot,
    KeySink sink, unsigned long long* __restrict__ next_item) {
  // METRIC 0: L2 with a table per (query, list); 1: inner product; 2: L2 through stored norms
  // (one table -2 <q_m, T_m[j]> per query; per list cdist - |c_l|^2 = |q|^2 - 2 <q, c_l>;
  // + |x'|^2 per code)
  constexpr int K = 256, D = M * DSUB;
  constexpr int KEY_METRIC = METRIC == 1 ? 1 : 0;
  constexpr int TPM = 256 / M;    // lanes that share one sub-quantizer
  // Rows of a table are K + TPM floats apart: the lanes of a wavefront store entries of 64 / TPM
  // consecutive sub-quantizers at the same column, and with rows a multiple of 256 bytes apart
  // those stores would all fall into the same TPM banks.
  constexpr int KP = K + TPM;
  static_assert(256 % M == 0 && M % 4 == 0, "M must divide 256 and codes are read as 32-bit words");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  u64* slots = reinterpret_cast<u64*>(smem);                    // 4 * tot
  u64* bound = slots + 4 * tot;                                 // workgroup bound (+ pad)
  float* lut0 = reinterpret_cast<float*>(bound + 2);            // NBUF x M * KP
  int64_t* s_begin = reinterpret_cast<int64_t*>(lut0 + NBUF * M * KP);  // ppb
  int64_t* s_end = s_begin + ppb;                               // ppb
  int32_t* s_list = reinterpret_cast<int32_t*>(s_end + ppb);    // ppb
  unsigned long long* s_item = reinterpret_cast<unsigned long long*>(bound + 1);   // the item in hand

  const int tid = threadIdx.x, wave = tid >> 6;
  const int m_own = tid / TPM, jj = tid % TPM;
  const int64_t last = ntotal > 0 ? ntotal - 1 : 0;             // clamp for speculative code loads
#ifdef VS_SCAN_TIMING
  unsigned long long tacc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  unsigned long long tprev = clock64();
#endif

  // Lane (m_own, jj) owns codewords jj, jj + TPM, ... of sub-quantizer m_own: M codewords
  // of DSUB floats = D registers, loaded once per workgroup.
  float T[M * DSUB];
#pragma unroll
  for (int i = 0; i < M; ++i)
#pragma unroll
    for (int u = 0; u < DSUB; ++u)
      T[i * DSUB + u] = codebooks[((int64_t)m_own * K + jj + TPM * i) * DSUB + u];
  wait_all_global_loads();   // the codebook is in registers from here on
  // L2 tables are built as |r|^2 + |t|^2 - 2 <r, t> (Sec. 4.3's decomposition applied to one
  // sub-vector): per entry DSUB fused multiply-adds on -2 t and one addition, against DSUB
  // subtractions and DSUB fused multiply-adds for sum (r - t)^2 -- the table build is vector
  // arithmetic only, and a third to 45 % of it goes away.  Exact for integer data; otherwise the
  // entry differs from the subtraction form by rounding of the order 1e-7 (|r|^2 + |t|^2).
  float TN[METRIC == 0 ? M : 1];
  if (METRIC == 0) {
#pragma unroll
    for (int i = 0; i < M; ++i) {
      float tn = 0.f;
#pragma unroll
      for (int u = 0; u < DSUB; ++u) {
        tn = __builtin_fmaf(T[i * DSUB + u], T[i * DSUB + u], tn);
        T[i * DSUB + u] *= -2.f;
      }
      TN[i] = tn;
    }
  }

  // Items are handed out through a counter in memory (*next_item starts at 0), one at a time: the
  // items of a batch differ in length (the sum of their lists), and with a fixed share per
  // workgroup the launch would end with the unluckiest share.
  for (;;) {
    if (tid == 0) *s_item = atomicAdd(next_item, 1ull);
    block_sync_lds();
    const int64_t item = (int64_t)*s_item;
    if (item >= nitems) break;
    const int64_t qi = item / nsplit;
    const int split = (int)(item % nsplit);
    const int p_begin = split * ppb;
    const int np = ntotal > 0 ? min(nprobe, p_begin + ppb) - p_begin : 0;
    float qm[DSUB];                                             // this lane's slice of the query
#pragma unroll
    for (int u = 0; u < DSUB; ++u) qm[u] = q[qi * D + m_own * DSUB + u];

    WaveSelect<R> ws;
    ws.init(slots + wave * tot, tot, k, bound);
    if (tid == 0) *bound = KEY_EMPTY;
    // the item's probes and list extents, fetched in one parallel round
    for (int p = tid; p < np; p += 256) {
      const int l = probes[qi * nprobe + p_begin + p];
      s_list[p] = l >= 0 ? l : 0;
      s_begin[p] = l >= 0 ? list_off[l] : 0;
      s_end[p] = l >= 0 ? list_off[l + 1] : 0;
    }
    if (METRIC != 0) {  // one table per query
#pragma unroll
      for (int i = 0; i < M; ++i) {
        float acc = 0.f;
#pragma unroll
        for (int u = 0; u < DSUB; ++u) acc = __builtin_fmaf(qm[u], T[i * DSUB + u], acc);
        lut0[m_own * KP + jj + TPM * i] = METRIC == 2 ? -2.f * acc : acc;
      }
    }
    block_sync_lds();   // probes, bound and the IP table are visible
    TICK(0);

    // Software pipeline over the item's lists (L2 metric): iteration p builds table p into
    // lut[p & 1] from registers only (query slice, centroid slice, codewords), then -- after
    // ONE barrier -- scans list p.  The first 256 codes and the centroid slice of list p + 1
    // are requested at the top of iteration p, a full iteration ahead.  These requests are
    // unconditional (indices clamped into range; lanes past a list's end are masked when
    // they are consumed), so the number of loads in flight is the same on every path.
    CodeWords<M> cw, cw_n;
    float nrm = 0.f, nrm_n = 0.f;                               // METRIC 2: the code's stored norm
    int64_t i_cur = 0;
    bool v_cur = false;
    float cm[DSUB], cm_n[DSUB];
#pragma unroll
    for (int u = 0; u < DSUB; ++u) cm[u] = cm_n[u] = 0.f;
    if (np > 0) {
      i_cur = s_begin[0] + tid;
      v_cur = i_cur < s_end[0];
      cw.load(codes + min(i_cur, last) * M);
      if (METRIC == 2) nrm = norms[min(i_cur, last)];
      if (METRIC == 0) {
        const int l0 = s_list[0];
#pragma unroll
        for (int u = 0; u < DSUB; ++u) cm[u] = centroids[(int64_t)l0 * D + m_own * DSUB + u];
      }
    }
    TICK(1);
    for (int p = 0; p < np; ++p) {
      float* __restrict__ lut = (METRIC == 0 && NBUF == 2) ? lut0 + (p & 1) * (M * KP) : lut0;
      const int64_t end = s_end[p];
      // requests for the next iteration (the last iteration re-requests its own list)
      const int pn = min(p + 1, np - 1);
      const int64_t i_n = s_begin[pn] + tid;
      const bool v_n = (p + 1 < np) && (i_n < s_end[pn]);
      cw_n.load(codes + min(i_n, last) * M);
      if (METRIC == 2) nrm_n = norms[min(i_n, last)];
      float bias = 0.f;
      if (METRIC == 0) {
        const int l1 = s_list[pn];
#pragma unroll
        for (int u = 0; u < DSUB; ++u) cm_n[u] = centroids[(int64_t)l1 * D + m_own * DSUB + u];
        float r[DSUB];
#pragma unroll
        for (int u = 0; u < DSUB; ++u) r[u] = qm[u] - cm[u];
        if (NBUF == 1 && p > 0) block_sync_lds();   // single table: scan p - 1 finished everywhere
        float rn = 0.f;
#pragma unroll
        for (int u = 0; u < DSUB; ++u) rn = __builtin_fmaf(r[u], r[u], rn);
#pragma unroll
        for (int i = 0; i < M; ++i) {
          float acc = rn + TN[i];
#pragma unroll
          for (int u = 0; u < DSUB; ++u) acc = __builtin_fmaf(r[u], T[i * DSUB + u], acc);
          lut[m_own * KP + jj + TPM * i] = acc;
        }
        TICK(2);
        block_sync_lds();   // table p visible; scan p - 1 (on the other buffer) finished everywhere
        TICK(3);
      } else {
        bias = cdist[qi * nprobe + p_begin + p];
        if (METRIC == 2) bias -= cnorm[s_list[p]];
      }
      // scan list p; the next chunk of a long list is requested before the current one is summed
      CodeWords<M> cw2;
      float nrm2 = 0.f;
      for (;;) {
        const int64_t i2 = i_cur + 256;
        const bool more = i2 - tid < end;      // uniform: i2 - tid is the next chunk's base
        const bool v2 = i2 < end;
        if (more) {
          cw2.load(codes + min(i2, last) * M);
          if (METRIC == 2) nrm2 = norms[min(i2, last)];
        }
        float dist = v_cur ? cw.template adc_rows<KP>(lut, METRIC == 2 ? bias + nrm : bias) : 0.f;
        if (METRIC != 1) dist = fmaxf(dist, 0.f);   // a squared distance: the expanded square can round below zero
        ws.push(v_cur, make_key(dist, (u32)i_cur, KEY_METRIC), true);
        if (!more) break;
        cw = cw2; nrm = nrm2; i_cur = i2; v_cur = v2;
      }
      cw = cw_n; nrm = nrm_n; i_cur = i_n; v_cur = v_n;
#pragma unroll
      for (int u = 0; u < DSUB; ++u) cm[u] = cm_n[u];
      TICK(4);
    }
    ws.finish();
    block_sync_lds();
    TICK(5);
    block_rank_merge(slots, tot, 4, k, sink, item * k);
    block_sync_lds();   // the slots have been read; the next item may reset them
    TICK(6);
#ifdef VS_SCAN_TIMING
    if (tid == 0) { tacc[7] += ws.trim_cycles; }
#endif
  }
#ifdef VS_SCAN_TIMING
  if (tid == 0)
    for (int t = 0; t < 8; ++t) atomicAdd(&g_scan_cycles[t], tacc[t]);
#endif
}

// One wavefront per query: k best of the nsplit partial lists, then
// (value, stored id).  Storage position -> id goes through the ids array
// (Sec. 6.1: IVF indexes store the 64-bit id next to each code).
template <int R>
__global__ __launch_bounds__(64) void ivfpq_merge_kernel(const u64* __restrict__ partial,
                                                         int nsplit, int k, int tot, int metric,
                                                         const int64_t* __restrict__ ids,
                                                         float* __restrict__ out_dist,
                                                         int64_t* __restrict__ out_ids) {
  extern __shared__ u64 mslots[];
  const int64_t qi = blockIdx.x;
  const int lane = lane_id();
  WaveSelect<R> ws;
  ws.init(mslots, tot, k);
  const u64* __restrict__ src = partial + qi * (int64_t)nsplit * k;
  const int n = nsplit * k;
  for (int j0 = 0; j0 < n; j0 += VS_WAVE) {
    const int j = j0 + lane;
    const u64 key = j < n ? src[j] : KEY_EMPTY;
    ws.push(j < n && key != KEY_EMPTY, key);
  }
  ws.finish();
  for (int j = lane; j < k; j += VS_WAVE) {
    const u64 key = ws.s[j];
    float v; int64_t id;
    if (key == KEY_EMPTY) { v = metric ? -__builtin_inff() : __builtin_inff(); id = -1; }
    else { v = key_value(key, metric); id = ids[key_index(key)]; }
    out_dist[qi * k + j] = v;
    out_ids[qi * k + j] = id;
  }
}

}  // namespace

// ------------------------------------------------------------------ launchers

void launch_pq_encode(const IvfpqDims& g, const float* x, int64_t n, const int32_t* list_of,
                      const float* centroids, const float* codebooks, uint8_t* tmp_codes,
                      hipStream_t st) {
  if (n <= 0) return;
  const dim3 grid((unsigned)((n + 255) / 256), (unsigned)g.M), block(256);
  const size_t shmem = (size_t)g.K * g.dsub * sizeof(float);
  if (shmem > 48 * 1024) {
    hipLaunchKernelGGL(pq_encode_global_kernel, grid, block, 0, st, x, n, g.d, g.dsub, g.K, list_of,
                       centroids, codebooks, g.M, tmp_codes);
    return;
  }
#define LAUNCH(DS) \
  hipLaunchKernelGGL((pq_encode_kernel<DS>), grid, block, shmem, st, x, n, g.d, g.dsub, g.K, list_of, \
                     centroids, codebooks, g.M, tmp_codes)
  switch (g.dsub) {
    case 2: LAUNCH(2); break;
    case 3: LAUNCH(3); break;
    case 4: LAUNCH(4); break;
    case 8: LAUNCH(8); break;
    case 12: LAUNCH(12); break;
    case 16: LAUNCH(16); break;
    default: LAUNCH(0); break;
  }
#undef LAUNCH
}

void launch_relayout(const IvfpqDims& g, const uint8_t* old_codes, const int64_t* old_ids,
                     const float* old_norms, int64_t old_total, const int64_t* old_off,
                     const int64_t* new_off, const uint8_t* tmp_codes,
                     const int64_t* new_ids_or_null, int64_t id_base, const float* tmp_norms,
                     const int64_t* dest, int64_t n_new, uint8_t* codes, int64_t* ids, float* norms,
                     hipStream_t st) {
  if (old_total > 0)
    hipLaunchKernelGGL(move_old_kernel, dim3((unsigned)((old_total + 255) / 256)), dim3(256), 0, st,
                       old_codes, old_ids, old_norms, old_total, old_off, new_off, g.nlist,
                       g.code_size, codes, ids, norms);
  if (n_new > 0)
    hipLaunchKernelGGL(scatter_new_kernel, dim3((unsigned)((n_new + 255) / 256)), dim3(256), 0, st,
                       tmp_codes, new_ids_or_null, id_base, tmp_norms, dest, n_new, g.M, g.nbits,
                       g.code_size, codes, ids, norms);
}

void launch_pq_norms(const IvfpqDims& g, const uint8_t* tmp_codes, int64_t n, const int32_t* list_of,
                     const float* centroids, const float* codebooks, float* tmp_norms,
                     hipStream_t st) {
  if (n <= 0) return;
  hipLaunchKernelGGL(pq_norms_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, tmp_codes,
                     n, g.d, g.dsub, g.K, g.M, list_of, centroids, codebooks, tmp_norms);
}

void launch_row_norms(const float* x, int64_t n, int d, float* norms, hipStream_t st) {
  if (n <= 0) return;
  hipLaunchKernelGGL(row_norms_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, x, n, d, norms);
}

void launch_list_of_storage(const int64_t* off, int nlist, int64_t total, int32_t* list_of,
                            hipStream_t st) {
  if (total <= 0) return;
  hipLaunchKernelGGL(list_of_storage_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                     off, nlist, total, list_of);
}

void launch_list_sizes(const int64_t* off, int nlist, int64_t* sizes, hipStream_t st) {
  hipLaunchKernelGGL(list_sizes_kernel, dim3((unsigned)((nlist + 255) / 256)), dim3(256), 0, st, off,
                     nlist, sizes);
}

template <int M, int DSUB, int METRIC, int R, int NBUF>
static void launch_scan_reg(const IvfpqDims& g, const float* q, int64_t nq, const float* centroids,
                            const float* codebooks, const int32_t* probes, const float* cdist,
                            int nprobe, int ppb, int nsplit, const int64_t* list_off,
                            const uint8_t* codes, const float* norms, const float* cnorm,
                            int64_t ntotal, int k, int tot, KeySink sink, u64* counter, hipStream_t st) {
  const size_t shmem = (size_t)(4 * tot + 2) * sizeof(u64) + (size_t)NBUF * M * (256 + 256 / M) * sizeof(float) +
                       (size_t)ppb * 20 + 16;
  auto kern = &ivfpq_scan_reg_kernel<M, DSUB, METRIC, R, NBUF>;
  if (shmem > 48 * 1024)
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
  const int64_t nitems = nq * nsplit;
  // persistent workgroups: as many as are resident at once on the 256 CUs, each walks over items
  int per_cu = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, 256, shmem) != hipSuccess || per_cu < 1)
    per_cu = 1;
  const int64_t grid = std::min<int64_t>(nitems, 256ll * per_cu);
  launch_fill_u64(counter, 1, 0ull, st);
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), shmem, st, q, centroids, codebooks,
                     probes, cdist, nprobe, ppb, nsplit, nitems, list_off, codes, norms, cnorm, ntotal,
                     k, tot, sink, reinterpret_cast<unsigned long long*>(counter));
}

template <int M, int DSUB>
static void launch_scan_reg_any(const IvfpqDims& g, const float* q, int64_t nq,
                                const float* centroids, const float* codebooks,
                                const int32_t* probes, const float* cdist, int nprobe, int ppb,
                                int nsplit, const int64_t* list_off, const uint8_t* codes,
                                const float* norms, const float* cnorm, int mode, int64_t ntotal,
                                int k, int tot, KeySink sink, u64* counter, hipStream_t st) {
#define GO(MET, RR, NB)                                                                           \
  launch_scan_reg<M, DSUB, MET, RR, NB>(g, q, nq, centroids, codebooks, probes, cdist, nprobe, ppb, \
                                        nsplit, list_off, codes, norms, cnorm, ntotal, k, tot, sink, counter, st)
  const int r = select_regs_for_slots(tot);
  // L2 tables alternate between two buffers (one barrier per list); the single inner-product
  // table needs one.  A single L2 table with a third resident workgroup per CU measured
  // slower at 1500-code lists: the 168-register budget it needs spills the codebook.
  if (mode == 1)      { if (r == 2) GO(1, 2, 1); else if (r == 4) GO(1, 4, 1); else GO(1, 0, 1); }
  else if (mode == 2) { if (r == 2) GO(2, 2, 1); else if (r == 4) GO(2, 4, 1); else GO(2, 0, 1); }
  else                { if (r == 2) GO(0, 2, 2); else if (r == 4) GO(0, 4, 2); else GO(0, 0, 2); }
#undef GO
}

template <int NBITS, int R, int W16>
static void launch_scan_pipe(const IvfpqDims& g, const float* q, int64_t nq,
                             const float* centroids, const float* codebooks,
                             const int32_t* probes, const float* cdist, int nprobe, int ppb,
                             int nsplit, const int64_t* list_off, const uint8_t* codes,
                             const float* norms, const float* cnorm, int mode, int64_t ntotal, int k,
                             int tot, size_t shmem, KeySink sink, hipStream_t st) {
  auto kern = &ivfpq_scan_pipe_kernel<NBITS, R, W16>;
  if (shmem > 48 * 1024)
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
  hipLaunchKernelGGL(kern, dim3((unsigned)(nq * nsplit)), dim3(256), shmem, st, q, g.d, mode,
                     g.M, g.dsub, centroids, codebooks, probes, cdist, nprobe, ppb, nsplit, list_off,
                     codes, norms, cnorm, ntotal, k, tot, sink);
}

template <int NBITS, int R>
static void launch_scan_generic(const IvfpqDims& g, const float* q, int64_t nq,
                                const float* centroids, const float* codebooks,
                                const int32_t* probes, const float* cdist, int nprobe, int ppb,
                                int nsplit, const int64_t* list_off, const uint8_t* codes,
                                const float* norms, const float* cnorm, int mode, int k, int tot,
                                size_t shmem, KeySink sink, hipStream_t st) {
  auto kern = &ivfpq_scan_kernel<NBITS, R>;
  if (shmem > 48 * 1024)
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
  hipLaunchKernelGGL(kern, dim3((unsigned)(nq * nsplit)), dim3(256), shmem, st, q, g.d, mode,
                     g.M, g.dsub, centroids, codebooks, probes, cdist, nprobe, ppb, nsplit, list_off,
                     codes, norms, cnorm, g.code_size, k, tot, sink);
}

int launch_ivfpq_scan(const IvfpqDims& g, const float* q, int64_t nq, const float* centroids,
                      const float* codebooks, const int32_t* probes, const float* cdist,
                      int nprobe, int nsplit, const int64_t* list_off, const uint8_t* codes,
                      const float* norms, const float* cnorm, int64_t ntotal, int k, u64* partial,
                      u64* counter, const int64_t* ids, float* out_dist, int64_t* out_ids, hipStream_t st) {
  if (nq <= 0) return 0;
  // table form: 1 inner product; 2 L2 through the stored norms (norms non-null; cnorm = the
  // centroids' squared norms); 0 L2 with one table of squared residual distances per (query, list)
  const int mode = g.metric == 1 ? 1 : (norms ? 2 : 0);
  KeySink sink;
  sink.metric = g.metric;
  sink.idx32 = nullptr;
  if (nsplit == 1) { sink.keys = nullptr; sink.val = out_dist; sink.id64 = out_ids; sink.idmap = ids; }
  else             { sink.keys = partial; sink.val = nullptr; sink.id64 = nullptr; sink.idmap = nullptr; }
  const int ppb = (nprobe + nsplit - 1) / nsplit;
  const int tot = select_slots_for_k(k);
  const size_t shmem = (size_t)4 * tot * sizeof(u64) + (size_t)g.M * g.K * sizeof(float) +
                       (size_t)(g.d + 2) * sizeof(float);
  if (shmem + 64 > 160 * 1024) return -1;
  const size_t reg_shmem = shmem + (size_t)g.M * g.K * sizeof(float) + 2 * 256 * sizeof(float) +
                           (size_t)ppb * 20 + 32;   // two tables, their rows padded
#define REG(MM, DS)                                                                              \
  if (g.nbits == 8 && g.M == MM && g.dsub == DS && reg_shmem <= 160 * 1024) {                    \
    launch_scan_reg_any<MM, DS>(g, q, nq, centroids, codebooks, probes, cdist, nprobe, ppb,      \
                                nsplit, list_off, codes, norms, cnorm, mode, ntotal, k, tot, sink, counter, st); \
    return 0;                                                                                    \
  }
  REG(16, 8)   // PQ16x8 on d = 128
  REG(32, 3)   // PQ32x8 on d = 96
  REG(8, 4)    // PQ8x8 on d = 32
#undef REG
  const int r = select_regs_for_slots(tot);
  // codes of 16, 32 or 64 bytes: the software-pipelined kernel
  const size_t pipe_shmem = shmem + sizeof(float) + (size_t)ppb * 20 + 24;
  if ((g.code_size == 16 || g.code_size == 32 || g.code_size == 64) && pipe_shmem + 64 <= 160 * 1024) {
#define PIPE3(NB, RR, WW)                                                                        \
  launch_scan_pipe<NB, RR, WW>(g, q, nq, centroids, codebooks, probes, cdist, nprobe, ppb, nsplit, \
                               list_off, codes, norms, cnorm, mode, ntotal, k, tot, pipe_shmem, sink, st)
#define PIPE2(NB, RR)                                                                            \
  do {                                                                                           \
    if (g.code_size == 16) PIPE3(NB, RR, 1);                                                     \
    else if (g.code_size == 32) PIPE3(NB, RR, 2);                                                \
    else PIPE3(NB, RR, 4);                                                                       \
  } while (0)
    if (g.nbits == 8) { if (r == 2) PIPE2(8, 2); else if (r == 4) PIPE2(8, 4); else PIPE2(8, 0); }
    else              { if (r == 2) PIPE2(4, 2); else if (r == 4) PIPE2(4, 4); else PIPE2(4, 0); }
#undef PIPE2
#undef PIPE3
    return 0;
  }
#define GEN(NB, RR)                                                                              \
  launch_scan_generic<NB, RR>(g, q, nq, centroids, codebooks, probes, cdist, nprobe, ppb, nsplit, \
                              list_off, codes, norms, cnorm, mode, k, tot, shmem, sink, st)
  if (g.nbits == 8) { if (r == 2) GEN(8, 2); else if (r == 4) GEN(8, 4); else GEN(8, 0); }
  else              { if (r == 2) GEN(4, 2); else if (r == 4) GEN(4, 4); else GEN(4, 0); }
#undef GEN
  return 0;
}

#ifdef VS_SCAN_TIMING
extern "C" __attribute__((visibility("default"))) int vs_debug_scan_cycles(unsigned long long* out8) {
  unsigned long long zero[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (hipMemcpyFromSymbol(out8, HIP_SYMBOL(g_scan_cycles), sizeof(zero)) != hipSuccess) return -1;
  if (hipMemcpyToSymbol(HIP_SYMBOL(g_scan_cycles), zero, sizeof(zero)) != hipSuccess) return -1;
  return 0;
}
#endif

void launch_ivfpq_merge(const u64* partial, int64_t nq, int nsplit, int k, int metric,
                        const int64_t* ids, float* out_dist, int64_t* out_ids, hipStream_t st) {
  if (nq <= 0) return;
  const int tot = select_slots_for_k(k);
  const size_t shmem = (size_t)tot * sizeof(u64);
  const dim3 grid((unsigned)nq), block(64);
  switch (select_regs_for_slots(tot)) {
    case 2: hipLaunchKernelGGL((ivfpq_merge_kernel<2>), grid, block, shmem, st, partial, nsplit, k, tot, metric, ids, out_dist, out_ids); break;
    case 4: hipLaunchKernelGGL((ivfpq_merge_kernel<4>), grid, block, shmem, st, partial, nsplit, k, tot, metric, ids, out_dist, out_ids); break;
    default: hipLaunchKernelGGL((ivfpq_merge_kernel<0>), grid, block, shmem, st, partial, nsplit, k, tot, metric, ids, out_dist, out_ids); break;
  }
}
