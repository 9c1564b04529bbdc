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
// One lane per vector; tmp_codes holds one byte per (vector, m), or -- packed4 -- the stored form of
// 4-bit codes, two per byte (byte i = c_{2i} | c_{2i+1} << 4).
__global__ void pq_norms_kernel(const uint8_t* __restrict__ tmp_codes, int64_t n, int d, int dsub,
                                int K, int M, bool packed4, const int32_t* __restrict__ list_of,
                                const float* __restrict__ centroids,
                                const float* __restrict__ codebooks, float* __restrict__ tmp_norms) {
  const int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i >= n) return;
  const float* __restrict__ c = centroids + (int64_t)list_of[i] * d;
  float acc = 0.f;
  for (int m = 0; m < M; ++m) {
    const int cm = packed4 ? (tmp_codes[i * (M / 2) + (m >> 1)] >> (4 * (m & 1))) & 15 : tmp_codes[i * M + m];
    const float* __restrict__ T = codebooks + ((int64_t)m * K + cm) * dsub;
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

// rot > 0 (= M, 8-bit codes): the code at position p of its list is stored rotated by p bytes,
// stored byte b = c_{(b + p) mod M} (the layout ivfpq_scan_bank_kernel reads); rot == 0: as is.
__global__ void scatter_new_kernel(const uint8_t* __restrict__ tmp_codes,
                                   const int64_t* __restrict__ new_ids, int64_t id_base,
                                   const float* __restrict__ tmp_norms,
                                   const int64_t* __restrict__ dest, int64_t n, int M, int nbits,
                                   int cs, int rot, const int32_t* __restrict__ list_of,
                                   const int64_t* __restrict__ new_off, uint8_t* __restrict__ codes,
                                   int64_t* __restrict__ ids, float* __restrict__ norms) {
  const int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int64_t p = dest[i];
  ids[p] = new_ids ? new_ids[i] : id_base + i;
  if (norms) norms[p] = tmp_norms[i];
  const uint8_t* __restrict__ t = tmp_codes + i * M;
  if (rot > 0) {
    const int shift = (int)((p - new_off[list_of[i]]) & (int64_t)(rot - 1));   // rot is a power of two
    for (int b = 0; b < cs; ++b) codes[p * cs + b] = t[(b + shift) & (rot - 1)];
  } else if (nbits == 8) {
    for (int b = 0; b < cs; ++b) codes[p * cs + b] = t[b];
  } else {  // two 4-bit codes per byte, even m in the low nibble
    for (int b = 0; b < cs; ++b) codes[p * cs + b] = (uint8_t)(t[2 * b] | (t[2 * b + 1] << 4));
  }
}

// The stored codes as the header defines them (byte m = c_m): undoes the rotation above.
__global__ void unrotate_codes_kernel(const uint8_t* __restrict__ stored, const int64_t* __restrict__ off,
                                      int nlist, int64_t total, int M, uint8_t* __restrict__ out) {
  const int64_t s = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (s >= total) return;
  const int l = list_of_position(off, nlist, s);
  const int shift = (int)((s - off[l]) & (int64_t)(M - 1));
  for (int b = 0; b < M; ++b) out[s * M + ((b + shift) & (M - 1))] = stored[s * M + b];
}

// Per-list term of the split look-up tables (Sec. 4.3 "Compressed-domain search"):
// B[l][j][m] = |T_m[j]|^2 + 2 <c_{l,m}, T_m[j]>, inner products as fma chains in dimension order.
// One lane per entry; layout [nlist][K][M] (the M entries of a codeword number are adjacent, as
// the scan kernel's table rows are).
__global__ void pq_list_tables_kernel(const float* __restrict__ centroids, const float* __restrict__ codebooks,
                                      int nlist, int d, int M, int K, int dsub, float* __restrict__ out) {
  const int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (e >= (int64_t)nlist * K * M) return;
  const int m = (int)(e % M), j = (int)((e / M) % K);
  const int64_t l = e / ((int64_t)M * K);
  const float* __restrict__ T = codebooks + ((int64_t)m * K + j) * dsub;
  const float* __restrict__ c = centroids + l * d + m * dsub;
  float ct = 0.f, tt = 0.f;
  for (int u = 0; u < dsub; ++u) { ct = __builtin_fmaf(c[u], T[u], ct); tt = __builtin_fmaf(T[u], T[u], tt); }
  out[e] = __builtin_fmaf(2.f, ct, tt);
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
// costs no exposed memory latency beyond the first one of the item.  Lanes past the end of
// a list request nothing (with 610-code lists the tail of every list's last chunk was a
// fifth of the kernel's memory traffic) and are masked when consumed.
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
#pragma unroll
  for (int w = 0; w < W16; ++w) cw[w] = cwn[w] = u32x4{0u, 0u, 0u, 0u};
  if (p < np && base + tid < s_end[p]) {
    const int64_t i = base + tid;
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
    if (pn < np && base_n + tid < s_end[pn]) {
      const int64_t i = base_n + tid;
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
// Register-resident codebook + bank-private look-up tables, for 8-bit codes (K = 256) of
// M = 8, 16 or 32 sub-quantizers and shapes known at compile time.
//
// Look-ups.  A wavefront's LDS read of one dword per lane is served 32 lanes at a time by 64
// banks; 32 random addresses collide in some bank almost always (measured: 5.9 - 7.9 clk per
// wavefront read against 3.0 - 3.7 when the 32 lanes hit 32 different banks).  So the tables
// are laid out [j][column] with rows of 64 floats = one pass over all banks: entry j of
// sub-quantizer m sits at float j * 64 + column, its bank is its column, and at every step the
// 32 lanes of a pass read 32 DIFFERENT columns: lane l looks up sub-quantizer (t + l) mod M at
// step t, in copy (l / M) mod (32 / M) of that table (every table exists 32 / M times).  Columns
// 0 .. 31 hold one set of tables, columns 32 .. 63 the other one of the double buffer (L2: the
// next list's tables are built while this one is scanned, in banks the scan never touches).
// For the lanes to find byte t of their code to be c_{(t + l) mod M}, the index stores the code
// at position p of its list rotated by p bytes (see rotate_code): a chunk starts at a multiple
// of 256 codes from the list's start, so l = p mod 64.
// The address of an entry is then ONE instruction: v_perm_b32 puts the code byte into byte 1
// (j * 256) and the lane's column byte (4 * column, a per-lane constant of the step) into byte 0;
// the tables start at LDS address 0 (checked at run time, with a plain fallback).
//
// Tables.  Lane (m, jg) of the workgroup owns codewords jg * M .. jg * M + M - 1 of sub-quantizer
// m = lane mod M: M * DSUB floats in registers, loaded once per (persistent) workgroup.  The 32
// lanes of a pass then store one row segment of 32 consecutive columns: conflict-free as well.
// ---------------------------------------------------------------------------
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x3 __attribute__((ext_vector_type(3)));

// One PQ code of M bytes (8, 16 or 32) per lane, fetched by hand-issued loads.  The compiler
// tracks the loads it issues itself register by register, but at the joins of a loop it merges
// that knowledge conservatively and then waits for EVERY load in flight (vmcnt(0)) where one old
// load is needed -- which ends a prefetch of more than one chunk.  So the scan issues its code
// loads in asm and waits for them by count: vector memory loads return in order, and
// wait_newer<N>() returns once at most N younger load INSTRUCTIONS are outstanding, i.e. once
// this code (and everything older) has arrived.  The registers are operands of the wait, so no
// use can be scheduled ahead of it.
template <int M>
struct CodeWords {
  static constexpr int W = M / 4;
  static constexpr int NLOAD = M == 32 ? 2 : 1;       // load instructions per code
  u32x4 a = {0u, 0u, 0u, 0u}, b = {0u, 0u, 0u, 0u};    // M == 32: a, b; M == 16: a; M == 8: a.xy as a2
  u32x2 a2 = {0u, 0u};
  __device__ __forceinline__ u32 word(int i) const {
    if constexpr (M == 8) return a2[i & 1];
    else return i < 4 ? a[i & 3] : b[i & 3];
  }
  // (the destination registers are asm outputs and nothing else touches them before the wait:
  // a copy issued in between would read them before the data has arrived)
  __device__ __forceinline__ void load_async(const uint8_t* p) {
    if constexpr (M == 32)
      asm volatile("global_load_dwordx4 %0, %2, off\n\tglobal_load_dwordx4 %1, %2, off offset:16"
                   : "=&v"(a), "=&v"(b) : "v"(p) : "memory");
    else if constexpr (M == 16)
      asm volatile("global_load_dwordx4 %0, %1, off" : "=&v"(a) : "v"(p) : "memory");
    else
      asm volatile("global_load_dwordx2 %0, %1, off" : "=&v"(a2) : "v"(p) : "memory");
  }
  template <int N>
  __device__ __forceinline__ void wait_newer() {
    if constexpr (M == 32) asm volatile("s_waitcnt vmcnt(%2)" : "+v"(a), "+v"(b) : "n"(N) : "memory");
    else if constexpr (M == 16) asm volatile("s_waitcnt vmcnt(%1)" : "+v"(a) : "n"(N) : "memory");
    else asm volatile("s_waitcnt vmcnt(%1)" : "+v"(a2) : "n"(N) : "memory");
  }
  // all loads issued so far have landed in this set's registers
  __device__ __forceinline__ void drain() {
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(a), "+v"(b), "+v"(a2) : : "memory");
  }
  // sum of the M table entries; col[w] holds the lane's four column bytes of steps 4w .. 4w + 3.
  // Look-ups go in groups of at most 16: the addresses of a group, its reads back to back (LDS
  // returns in order, so each addition then waits for its own value only), its additions.  Left to
  // itself the scheduler issues five reads and drains them all before the next five.
  template <bool AT_ZERO>
  __device__ __forceinline__ float adc_banked(const unsigned char* __restrict__ lut, const u32 (&col)[W],
                                              float dist) const {
    constexpr int G = M < 16 ? M : 16;          // look-ups per group
#pragma unroll
    for (int g0 = 0; g0 < M; g0 += G) {
      u32 a[G];
#pragma unroll
      for (int i = 0; i < G / 4; ++i) {
        const u32 cwd = word(g0 / 4 + i), cl = col[g0 / 4 + i];
        // byte 0 <- column byte b of cl, byte 1 <- code byte b of cwd, bytes 2 and 3 <- 0
        a[4 * i] = __builtin_amdgcn_perm(cwd, cl, 0x0c0c0400u);
        a[4 * i + 1] = __builtin_amdgcn_perm(cwd, cl, 0x0c0c0501u);
        a[4 * i + 2] = __builtin_amdgcn_perm(cwd, cl, 0x0c0c0602u);
        a[4 * i + 3] = __builtin_amdgcn_perm(cwd, cl, 0x0c0c0703u);
      }
      float v[G];
#pragma unroll
      for (int t = 0; t < G; ++t) {
        if constexpr (AT_ZERO) v[t] = *reinterpret_cast<lds_cfloat_ptr>((uintptr_t)a[t]);
        else v[t] = *reinterpret_cast<const float*>(lut + a[t]);
      }
#pragma unroll
      for (int t = 0; t < G; ++t) dist += v[t];
      if constexpr (AT_ZERO) {
        __builtin_amdgcn_sched_group_barrier(0x002, G, 0);     // the group's address instructions
        __builtin_amdgcn_sched_group_barrier(0x100, G, 0);     // its reads, back to back
        __builtin_amdgcn_sched_group_barrier(0x002, G, 0);     // its additions
      }
    }
    return dist;
  }
  // The same sums for TWO tables at once, one in each column set (32 floats = 128 bytes apart):
  // one address instruction and one LDS instruction (a two-address read) per pair of look-ups.
  // Each sum adds its entries in the order of adc_banked: the same bits.
  __device__ __forceinline__ void adc_banked2(const u32 (&col)[W], float& da, float& db) const {
    constexpr int G = M < 16 ? M : 16;
#pragma unroll
    for (int g0 = 0; g0 < M; g0 += G) {
      u32 a[G];
#pragma unroll
      for (int i = 0; i < G / 4; ++i) {
        const u32 cwd = word(g0 / 4 + i), cl = col[g0 / 4 + i];
        a[4 * i] = __builtin_amdgcn_perm(cwd, cl, 0x0c0c0400u);
        a[4 * i + 1] = __builtin_amdgcn_perm(cwd, cl, 0x0c0c0501u);
        a[4 * i + 2] = __builtin_amdgcn_perm(cwd, cl, 0x0c0c0602u);
        a[4 * i + 3] = __builtin_amdgcn_perm(cwd, cl, 0x0c0c0703u);
      }
      float va[G], vb[G];
#pragma unroll
      for (int t = 0; t < G; ++t) {
        const lds_cfloat_ptr e = reinterpret_cast<lds_cfloat_ptr>((uintptr_t)a[t]);
        va[t] = e[0];
        vb[t] = e[32];
      }
#pragma unroll
      for (int t = 0; t < G; ++t) { da += va[t]; db += vb[t]; }
      __builtin_amdgcn_sched_group_barrier(0x002, G, 0);       // the group's address instructions
      __builtin_amdgcn_sched_group_barrier(0x100, 2 * G, 0);   // its reads, back to back
      __builtin_amdgcn_sched_group_barrier(0x002, 2 * G, 0);   // its additions
    }
  }
};

constexpr int kBankTableBytes = 256 * 64 * (int)sizeof(float);   // 256 rows of 64 floats

template <int M, int DSUB, int METRIC, int R, int NT>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(NT / 128, NT / 128)))
void ivfpq_scan_bank_kernel(
    const float* __restrict__ q, const float* __restrict__ centroids,
    const float* __restrict__ codebooks, const int32_t* __restrict__ probes,
    const float* __restrict__ cdist, int nprobe, int ppb, int nsplit, int64_t nitems,
    const int64_t* __restrict__ list_off, const uint8_t* __restrict__ codes,
    const float* __restrict__ norms, const float* __restrict__ cnorm,
    const float* __restrict__ list_tables, int64_t ntotal, int k, int tot,
    KeySink sink, unsigned long long* __restrict__ next_item, const u32* __restrict__ item_list,
    const u32* __restrict__ item_count) {
  // item_list / item_count: null, or (nsplit = 1 only) the queries to scan and how many they are,
  // both in device memory: the second launch after a list-major scan, for the queries whose
  // candidate buffer overflowed (usually none: every workgroup then leaves at its first look)
  // METRIC 0: L2 with a table per (query, list); 1: inner product; 2: L2 through stored norms
  // (one table -2 <q_m, T_m[j]> per query; per list cdist - |c_l|^2 = |q|^2 - 2 <q, c_l>;
  // + |x'|^2 per code); 3: L2 with the table of a (query, list) pair formed as a per-query term
  // A_m[j] = -2 <q_m, T_m[j]>, kept in registers, plus a per-list term B_l[j][m] = |T_m[j]|^2 +
  // 2 <c_{l,m}, T_m[j]> read from list_tables [nlist][256][M] (Sec. 4.3): one addition per entry
  // instead of DSUB multiply-adds, for indexes whose lists are too short to amortise a table
  constexpr int K = 256, D = M * DSUB;
  constexpr int KEY_METRIC = METRIC == 1 ? 1 : 0;
  constexpr bool PER_LIST = METRIC == 0 || METRIC == 3;   // a table per (query, list), double buffered
  constexpr int REP = 32 / M;     // copies of every table
  constexpr int NW = NT / 64;     // wavefronts of the workgroup (two workgroups share a CU)
  constexpr int EPL = K * M / NT; // table entries a lane builds = codewords it keeps
  // EXPAND: an L2 table entry holds |t|^2 - 2 <r_m, t> (|t|^2 in registers, DSUB instructions per
  // entry) rather than sum (r_m - t)^2 (2 DSUB instructions); the missing sum_m |r_m|^2 = |q - c_l|^2
  // is the coarse distance of the probe, which starts every code's sum
  constexpr bool EXPAND = METRIC == 0;
  static_assert(NT == 256 || NT == 512, "two workgroups per CU");
  static_assert(M == 8 || M == 16 || M == 32, "tables of M sub-quantizers fill 32 banks in 32 / M copies");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  // (the tables come first: with no static LDS in this kernel they start at LDS address 0)
  float* lut0 = reinterpret_cast<float*>(smem);                 // [256][64]
  u64* slots = reinterpret_cast<u64*>(smem + kBankTableBytes);  // NW * tot
  u64* bound = slots + NW * tot;                                 // workgroup bound (+ the item in hand)
  // the item's NON-EMPTY probed lists, compacted: first and one-past-last storage position
  // (positions fit 32 bits: an index holds fewer than 2^32 vectors), list number, per-list term
  u32* s_begin = reinterpret_cast<u32*>(bound + 3);             // ppb
  u32* s_end = s_begin + ppb;                                   // ppb
  int32_t* s_list = reinterpret_cast<int32_t*>(s_end + ppb);    // ppb
  float* s_bias = reinterpret_cast<float*>(s_list + ppb);       // ppb (inner product / stored norms)
  int* s_nl = reinterpret_cast<int*>(bound + 2);                // how many of them
  unsigned long long* s_item = reinterpret_cast<unsigned long long*>(bound + 1);
  // (the kernel has no static LDS, so its dynamic LDS -- the tables first -- starts at LDS address
  // 0 and a table offset is an LDS address: the launcher checks this)
  const int tid = threadIdx.x, wave = tid >> 6;
  const int m_own = tid & (M - 1), jg = tid / M;                // table build: codewords jg * EPL + i of m_own
  const int rep0 = jg & (REP - 1);                              // this lane's copy (build: the first it stores)

  float T[EPL * DSUB];
#pragma unroll
  for (int i = 0; i < EPL; ++i)
#pragma unroll
    for (int u = 0; u < DSUB; ++u)
      T[i * DSUB + u] = codebooks[((int64_t)m_own * K + jg * EPL + i) * DSUB + u];
  wait_all_global_loads();   // the codebook is in registers from here on
  // EXPAND: |r - t|^2 = |r|^2 + |t|^2 - 2 <r, t> (Sec. 4.3's expansion applied to one sub-vector):
  // per entry DSUB fused multiply-adds on -2 t starting from |t|^2.  Exact for integer data;
  // otherwise a distance differs from the subtraction form by rounding of at most
  // (DSUB + 2) 2^-23 (|r|^2 + |t|^2).
  float TN[EXPAND ? EPL : 1];
  if (EXPAND) {
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
      float tn = 0.f;
#pragma unroll
      for (int u = 0; u < DSUB; ++u) {
        tn = __builtin_fmaf(T[i * DSUB + u], T[i * DSUB + u], tn);
        T[i * DSUB + u] *= -2.f;
      }
      TN[i] = tn;
    }
  }
  // scan role: column byte (4 * column) of every step, four steps per register
  u32 col[M / 4];
#pragma unroll
  for (int w = 0; w < M / 4; ++w) {
    u32 v = 0;
#pragma unroll
    for (int b = 0; b < 4; ++b)
      v |= (u32)(4 * (((4 * w + b + tid) & (M - 1)) + M * rep0)) << (8 * b);
    col[w] = v;
  }

  // Items are handed out through a counter in memory (*next_item starts at 0), one at a time: the
  // items of a batch differ in length (the sum of their lists), and with a fixed share per
  // workgroup the launch would end with the unluckiest share.
  for (;;) {
    if (tid == 0) *s_item = atomicAdd(next_item, 1ull);
    block_sync_lds();
    const int64_t item = (int64_t)*s_item;
    if (item >= (item_count != nullptr ? (int64_t)*item_count : nitems)) break;
    const int64_t qi = item_list != nullptr ? (int64_t)item_list[item] : item / nsplit;
    const int split = (int)(item % nsplit);
    const int p_begin = split * ppb;
    const int np = ntotal > 0 ? min(nprobe, p_begin + ppb) - p_begin : 0;
    float qm[DSUB];                                             // this lane's slice of the query
#pragma unroll
    for (int u = 0; u < DSUB; ++u) qm[u] = q[qi * D + m_own * DSUB + u];

    WaveSelect<R> ws;
    ws.init(slots + wave * tot, tot, k, bound);
    ws.set_metric(KEY_METRIC);
    if (tid == 0) *bound = KEY_EMPTY;
    // the item's probes and list extents: wavefront 0 fetches them 64 at a time and keeps the
    // non-empty lists, in probe order
    if (wave == 0) {
      int cnt = 0;
      for (int p0 = 0; p0 < np; p0 += VS_WAVE) {
        const int p = p0 + tid;
        const int l = p < np ? probes[qi * nprobe + p_begin + p] : -1;
        const int64_t b = l >= 0 ? list_off[l] : 0, e = l >= 0 ? list_off[l + 1] : 0;
        const bool keep = e > b;
        const u64 mask = __ballot(keep);
        const int pos = cnt + __popcll(mask & ((1ull << tid) - 1ull));
        if (keep) {
          s_list[pos] = l;
          s_begin[pos] = (u32)b;
          s_end[pos] = (u32)e;
          float bs = cdist[qi * nprobe + p_begin + p];   // L2 tables: |q - c_l|^2 = sum_m |r_m|^2, see EXPAND
          if (METRIC == 2) bs -= cnorm[l];
          s_bias[pos] = bs;
        }
        cnt += __popcll(mask);
      }
      if (tid == 0) *s_nl = cnt;
    }
    // (the query slice is in registers before the scan's hand-counted loads start: a use here makes
    // the compiler wait for it now rather than, for everything in flight, inside the scan)
#pragma unroll
    for (int u = 0; u < DSUB; ++u) asm volatile("" : "+v"(qm[u]));
    float tq[METRIC == 3 ? EPL : 1];                            // METRIC 3: the per-query term of this lane's entries
    if (METRIC == 3) {
#pragma unroll
      for (int i = 0; i < EPL; ++i) {
        float acc = 0.f;
#pragma unroll
        for (int u = 0; u < DSUB; ++u) acc = __builtin_fmaf(qm[u], T[i * DSUB + u], acc);
        tq[i] = -2.f * acc;
      }
    }
    if (METRIC == 1 || METRIC == 2) {  // one table per query, in the first set of columns
#pragma unroll
      for (int i = 0; i < EPL; ++i) {
        float acc = 0.f;
#pragma unroll
        for (int u = 0; u < DSUB; ++u) acc = __builtin_fmaf(qm[u], T[i * DSUB + u], acc);
        const float e = METRIC == 2 ? -2.f * acc : acc;
#pragma unroll
        for (int c = 0; c < REP; ++c)
          lut0[(jg * EPL + i) * 64 + m_own + M * ((rep0 + c) & (REP - 1))] = e;
      }
    }
    block_sync_lds();   // probes, bound and the per-query table are visible

    // The chunks of NT codes of the item's non-empty lists form ONE sequence, and the scan is a
    // stream from HBM whose rate is bounded by what is in flight (bytes in flight = rate x
    // latency; one chunk ahead per wavefront is 16 KB per CU, about 4 TB/s chip-wide at the
    // latency measured under load).  So the codes of chunk c + 2 are requested before chunk c is
    // summed, across list boundaries, into one of three register sets that take turns -- the loop
    // is unrolled three times so that no set is ever copied (a copy would wait for the load just
    // issued).  Requests are clamped into the code array; lanes past a list's end are masked when
    // consumed.  At the first chunk of a list (L2 metric) its table is built into column set
    // `parity` from registers only (query slice, centroid slice requested one list ahead,
    // codewords), then ONE barrier, then the list is scanned while the other set's table may
    // still be in use by a slower wavefront.
    // Control state is wave-uniform and kept in scalar registers (readfirstlane of the LDS
    // arrays, touched once per list, not once per chunk): consumer / producer list, the extents
    // of that list, the first code of the current chunk.
    const int nl = __builtin_amdgcn_readfirstlane(*s_nl);
    // (the first 64 lists' entries also sit one per lane in registers: a cross-lane read costs a
    // few cycles where an LDS read costs a round trip, and short lists switch every chunk)
    const int lane = tid & (VS_WAVE - 1);
    const u32 xb = lane < nl ? s_begin[lane] : 0u, xe = lane < nl ? s_end[lane] : 0u;
    const int xl = lane < nl ? s_list[lane] : 0;
    auto list_begin = [&](int pl) -> u32 {
      return pl < VS_WAVE ? (u32)__builtin_amdgcn_readlane((int)xb, pl) : (u32)__builtin_amdgcn_readfirstlane(s_begin[pl]);
    };
    auto list_end = [&](int pl) -> u32 {
      return pl < VS_WAVE ? (u32)__builtin_amdgcn_readlane((int)xe, pl) : (u32)__builtin_amdgcn_readfirstlane(s_end[pl]);
    };
    auto list_number = [&](int pl) -> int {
      return pl < VS_WAVE ? __builtin_amdgcn_readlane(xl, pl) : __builtin_amdgcn_readfirstlane(s_list[pl]);
    };
    int pc = 0, pp = 0;
    u32 cb = 0, ce = 0, pe = 0;
    if (nl > 0) {
      cb = list_begin(0);
      ce = pe = list_end(0);
    }
    u32 base_c = cb, base_p = cb;
    // load instructions per request: the code, and its stored norm (METRIC 2)
    constexpr int NLT = CodeWords<M>::NLOAD + (METRIC == 2 ? 1 : 0);
    // Always issues exactly NLT loads (past the item's last chunk: of code 0, unused),
    // so that "2 * NLT younger loads" below means the same on every path.
    auto request = [&](CodeWords<M>& dst, float& nrm_dst) {
      // lanes past the list's end fetch the chunk's first code again (one cache line the wavefront
      // reads anyway) instead of the next list's codes: a list's last chunk is half empty on average
      const u32 iv = base_p + (u32)tid;
      const u32 i = iv < pe ? iv : base_p;
      dst.load_async(codes + (u64)i * M);
      if (METRIC == 2) asm volatile("global_load_dword %0, %1, off" : "=&v"(nrm_dst) : "v"(norms + i) : "memory");
      if (pp < nl) {
        base_p += NT;
        if (base_p >= pe) {
          ++pp;
          base_p = pp < nl ? list_begin(pp) : 0u;
          pe = pp < nl ? list_end(pp) : 0u;
        }
      }
    };
    // centroid slice of the next list to build (L2 tables), hand-issued like the codes: one dword
    // load per component into a register of its own, so that the wait and the first use (the
    // residual q - c) are ONE asm statement and nothing can read a component before it has arrived
    float cn[DSUB];
#pragma unroll
    for (int u = 0; u < DSUB; ++u) cn[u] = 0.f;
    auto request_centroid = [&](int pl) {
      if (METRIC == 0 && pl < nl) {
        const float* src = centroids + (int64_t)list_number(pl) * D + m_own * DSUB;
#pragma unroll
        for (int u = 0; u < DSUB; ++u)
          asm volatile("global_load_dword %0, %1, off" : "=&v"(cn[u]) : "v"(src + u) : "memory");
      }
    };
    // METRIC 3: the per-list term of this lane's entries of the next list to build, likewise
    float tl[METRIC == 3 ? EPL : 1];
#pragma unroll
    for (int i = 0; i < (METRIC == 3 ? EPL : 1); ++i) tl[i] = 0.f;
    auto request_list_table = [&](int pl) {
      if (METRIC == 3 && pl < nl) {
        const float* src = list_tables + ((int64_t)list_number(pl) * K + jg * EPL) * M + m_own;
#pragma unroll
        for (int i = 0; i < EPL; ++i)
          asm volatile("global_load_dword %0, %1, off" : "=&v"(tl[i]) : "v"(src + i * M) : "memory");
      }
    };
    CodeWords<M> S0, S1, S2;
    float n0 = 0.f, n1 = 0.f, n2 = 0.f;                         // METRIC 2: the codes' stored norms
    int parity = 0;
    float bias = 0.f;
    auto consume = [&](CodeWords<M>& cw, float& nrm) {
      // this chunk's code was requested two requests ago: everything but the 2 * NLT youngest
      // loads has arrived once this returns
      cw.template wait_newer<2 * NLT>();
      if (METRIC == 2) asm volatile("s_waitcnt vmcnt(%1)" : "+v"(nrm) : "n"(2 * NLT) : "memory");
      if (base_c == cb) {                                       // (uniform) first chunk of list pc
        if ((pc & 3) == 0) ws.refresh_shared();
        if (PER_LIST) {
#pragma unroll
          for (int w = 0; w < M / 4; ++w)   // this list's column set: + 32 floats = bit 7 of every column byte
            col[w] = (col[w] & 0x7f7f7f7fu) | (parity ? 0x80808080u : 0u);
          float* __restrict__ lutp = lut0 + 32 * parity;
          if (METRIC == 0) {
            // the slice was requested at the first chunk of the list before (or in the prologue):
            // only this step's request is younger.  r = q - c, one fp32 subtraction per component.
            float r[DSUB];
            asm volatile("s_waitcnt vmcnt(%0)" : : "n"(NLT) : "memory");
#pragma unroll
            for (int u = 0; u < DSUB; ++u)
              asm volatile("s_waitcnt vmcnt(%3)\n\tv_sub_f32 %0, %1, %2" : "=v"(r[u]) : "v"(qm[u]), "v"(cn[u]), "n"(NLT) : "memory");
            request_centroid(pc + 1);                             // one list ahead
#pragma unroll
            for (int i = 0; i < EPL; ++i) {
              float acc;
              if (EXPAND) {
                acc = TN[i];
#pragma unroll
                for (int u = 0; u < DSUB; ++u) acc = __builtin_fmaf(r[u], T[i * DSUB + u], acc);
              } else {
                acc = 0.f;
#pragma unroll
                for (int u = 0; u < DSUB; ++u) {
                  const float diff = r[u] - T[i * DSUB + u];
                  acc = __builtin_fmaf(diff, diff, acc);
                }
              }
#pragma unroll
              for (int c = 0; c < REP; ++c)
                lutp[(jg * EPL + i) * 64 + m_own + M * ((rep0 + c) & (REP - 1))] = acc;
            }
          } else {
            // entry = per-query term + per-list term; the wait and the addition are one statement
            float e[EPL];
#pragma unroll
            for (int i = 0; i < EPL; ++i)
              asm volatile("s_waitcnt vmcnt(%3)\n\tv_add_f32 %0, %1, %2" : "=v"(e[i]) : "v"(tq[i]), "v"(tl[i]), "n"(NLT) : "memory");
            request_list_table(pc + 1);                           // one list ahead
#pragma unroll
            for (int i = 0; i < EPL; ++i)
#pragma unroll
              for (int c = 0; c < REP; ++c)
                lutp[(jg * EPL + i) * 64 + m_own + M * ((rep0 + c) & (REP - 1))] = e[i];
          }
          parity ^= 1;
          block_sync_lds();   // this table is visible; the scan on the other column set has finished everywhere
        }
        bias = s_bias[pc];
      }
      const u32 i = base_c + (u32)tid;
      const bool valid = i < ce;
      float dist = 0.f;
      if (valid) {
        const float d0 = METRIC == 2 ? bias + nrm : bias;
        dist = cw.template adc_banked<true>(smem, col, d0);
      }
      if (METRIC != 1) dist = fmaxf(dist, 0.f);   // a squared distance: the expanded square can round below zero
      ws.push_value(valid, dist, i);
      base_c += NT;
      if (base_c >= ce) {
        ++pc;
        if (pc < nl) {
          cb = base_c = list_begin(pc);
          ce = list_end(pc);
        }
      }
    };
    if (nl > 0) {   // (uniform; ntotal > 0 here)
      request_centroid(pc);
      request_list_table(pc);
      request(S0, n0);
      request(S1, n1);
      for (;;) {
        request(S2, n2); consume(S0, n0);
        if (pc >= nl) break;
        request(S0, n0); consume(S1, n1);
        if (pc >= nl) break;
        request(S1, n1); consume(S2, n2);
        if (pc >= nl) break;
      }
      // The last two requests are still in flight.  They must land while their registers still
      // belong to them: once the sets are dead the compiler hands the registers to other values
      // (addresses of the result stores below), and a load arriving then would overwrite those.
      S0.drain(); S1.drain(); S2.drain();
      asm volatile("s_waitcnt vmcnt(0)" : "+v"(n0), "+v"(n1), "+v"(n2) : : "memory");
#pragma unroll
      for (int u = 0; u < DSUB; ++u) asm volatile("s_waitcnt vmcnt(0)" : "+v"(cn[u]) : : "memory");
#pragma unroll
      for (int i = 0; i < (METRIC == 3 ? EPL : 1); ++i) asm volatile("s_waitcnt vmcnt(0)" : "+v"(tl[i]) : : "memory");
    }
    ws.finish();
    block_sync_lds();
    block_rank_merge(slots, tot, NW, k, sink, (item_list != nullptr ? qi : item) * k);
    block_sync_lds();   // the slots have been read; the next item may reset them
  }
}

// ---------------------------------------------------------------------------
// List-major scan (Sec. 4.3 "Compressed-domain search", L2 with residual tables; the shapes of
// the bank-private kernel).  In a large batch every list is probed by several queries -- ten at
// 10,000 queries x 64 probes over 65,536 lists -- and a query-major scan reads it from memory
// every time: the queries that share a list do not run together.  Here the work item is a LIST:
// the workgroup takes the (query, list) pairs of its list two at a time, builds each pair's
// table exactly as the query-major kernel does (same registers, same arithmetic, and the
// entries of a code are added in the same order: the distances are the same bits), one table in
// each column set of the bank-private layout, and scans the list's codes again -- which the
// first pairs brought into the caches -- looking every code up in both tables with one address
// and one two-address read per sub-quantizer.  There is no selection state per pair: a code is kept
// only if its distance is not worse than the bound of ITS query, the k-th best distance the
// query-major kernel found in that query's first few lists, and kept codes are appended to the
// query's candidate buffer (one atomic per wavefront and chunk that has any).  A buffer that
// overflows flags its query, which a second launch of the query-major kernel then scans in
// full.  lm_merge_kernel selects the k best of a query's first-stage results and candidates.
// The pairs of a list come from pair_off / pairs (built by the lm_* kernels below); their
// order inside a list does not matter for the results.
// ---------------------------------------------------------------------------
constexpr int kLmGroup = 64;   // pairs of a list staged in LDS at a time

template <int M, int DSUB, int NT>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(NT / 128, NT / 128)))
void ivfpq_scan_listmajor_kernel(
    const float* __restrict__ q, const float* __restrict__ centroids,
    const float* __restrict__ codebooks, const float* __restrict__ cdist, int nprobe,
    const u32* __restrict__ pair_off, const u32* __restrict__ pairs, int nlist,
    const int64_t* __restrict__ list_off, const uint8_t* __restrict__ codes,
    const float* __restrict__ qbound, u32* __restrict__ cand_count, u64* __restrict__ cand, int cap,
    u32* __restrict__ overflow, unsigned long long* __restrict__ next_item) {
  constexpr int K = 256, D = M * DSUB;
  constexpr int REP = 32 / M;     // copies of every table
  constexpr int EPL = K * M / NT; // table entries a lane builds = codewords it keeps
  static_assert(NT == 256, "two workgroups per CU");
  static_assert(M == 8 || M == 16 || M == 32, "tables of M sub-quantizers fill 32 banks in 32 / M copies");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float* lut0 = reinterpret_cast<float*>(smem);                 // [256][64], at LDS address 0
  unsigned long long* s_item = reinterpret_cast<unsigned long long*>(smem + kBankTableBytes);
  int32_t* s_q = reinterpret_cast<int32_t*>(s_item + 1);        // kLmGroup: query of the pair
  float* s_bias = reinterpret_cast<float*>(s_q + kLmGroup);     // kLmGroup: |q - c_l|^2
  float* s_bnd = s_bias + kLmGroup;                             // kLmGroup: the query's bound
  const int tid = threadIdx.x;
  const int m_own = tid & (M - 1), jg = tid / M;
  const int rep0 = jg & (REP - 1);

  // codewords in registers as (|t|^2, -2 t), as in the query-major kernel
  float T[EPL * DSUB];
#pragma unroll
  for (int i = 0; i < EPL; ++i)
#pragma unroll
    for (int u = 0; u < DSUB; ++u)
      T[i * DSUB + u] = codebooks[((int64_t)m_own * K + jg * EPL + i) * DSUB + u];
  wait_all_global_loads();
  float TN[EPL];
#pragma unroll
  for (int i = 0; i < EPL; ++i) {
    float tn = 0.f;
#pragma unroll
    for (int u = 0; u < DSUB; ++u) {
      tn = __builtin_fmaf(T[i * DSUB + u], T[i * DSUB + u], tn);
      T[i * DSUB + u] *= -2.f;
    }
    TN[i] = tn;
  }
  u32 col[M / 4];
#pragma unroll
  for (int w = 0; w < M / 4; ++w) {
    u32 v = 0;
#pragma unroll
    for (int b = 0; b < 4; ++b)
      v |= (u32)(4 * (((4 * w + b + tid) & (M - 1)) + M * rep0)) << (8 * b);
    col[w] = v;
  }

  for (;;) {
    if (tid == 0) *s_item = atomicAdd(next_item, 1ull);
    block_sync_lds();
    const int64_t l = (int64_t)*s_item;
    block_sync_lds();                                           // everyone has read the item number
    if (l >= nlist) break;
    const u32 p0 = pair_off[l], p1 = pair_off[l + 1];
    const u32 cb = (u32)list_off[l], ce = (u32)list_off[l + 1];
    if (p0 == p1 || cb == ce) continue;                         // (uniform)
    float cl[DSUB];                                             // this lane's slice of the list's centroid
#pragma unroll
    for (int u = 0; u < DSUB; ++u) cl[u] = centroids[l * D + m_own * DSUB + u];
#pragma unroll
    for (int u = 0; u < DSUB; ++u) asm volatile("" : "+v"(cl[u]));   // in registers before the counted loads start

    for (u32 g0 = p0; g0 < p1; g0 += kLmGroup) {
      const int nl = (int)min((u32)kLmGroup, p1 - g0);
      if (tid < nl) {
        const u32 pr = pairs[g0 + tid];                         // query * nprobe + probe rank
        const int qi = (int)(pr / (u32)nprobe);
        s_q[tid] = qi;
        s_bias[tid] = cdist[pr];
        s_bnd[tid] = qbound[qi];
      }
      block_sync_lds();

      // Pairs are taken TWO at a time (a unit): the table of the first in column set 0, of the
      // second in column set 1, and every code of the list is looked up in both with the same
      // addresses -- per code and pair half an address instruction and half an LDS instruction
      // fewer than one table at a time.  (A last pair without a partner runs with itself and a
      // bound that nothing passes.)  The (unit, chunk) steps of the group form one sequence;
      // codes are requested two steps ahead into three register sets, the query slices of the
      // next unit one unit ahead, all by hand-issued loads with counted waits (see CodeWords).
      constexpr int NLT = CodeWords<M>::NLOAD;
      const int nu = (nl + 1) / 2;
      int pc = 0, pp = 0;
      u32 base_c = cb, base_p = cb;
      auto request = [&](CodeWords<M>& dst) {
        const u32 iv = base_p + (u32)tid;
        const u32 i = iv < ce ? iv : base_p;
        dst.load_async(codes + (u64)i * M);
        if (pp < nu) {
          base_p += NT;
          if (base_p >= ce) { ++pp; base_p = cb; }
        }
      };
      float qa[DSUB], qb[DSUB];
#pragma unroll
      for (int u = 0; u < DSUB; ++u) qa[u] = qb[u] = 0.f;
      auto request_queries = [&](int ul) {
        if (ul < nu) {
          const int ia = __builtin_amdgcn_readfirstlane(s_q[2 * ul]);
          const int ib = __builtin_amdgcn_readfirstlane(s_q[min(2 * ul + 1, nl - 1)]);
          const float* sa = q + (int64_t)ia * D + m_own * DSUB;
          const float* sb = q + (int64_t)ib * D + m_own * DSUB;
#pragma unroll
          for (int u = 0; u < DSUB; ++u)
            asm volatile("global_load_dword %0, %1, off" : "=&v"(qa[u]) : "v"(sa + u) : "memory");
#pragma unroll
          for (int u = 0; u < DSUB; ++u)
            asm volatile("global_load_dword %0, %1, off" : "=&v"(qb[u]) : "v"(sb + u) : "memory");
        }
      };
      CodeWords<M> S0, S1, S2;
      float bias_a = 0.f, bias_b = 0.f, bnd_a = 0.f, bnd_b = 0.f;
      int q_a = 0, q_b = 0;
      const int lane = tid & (VS_WAVE - 1);
      // codes that pass their query's bound go to that query's candidate buffer: one atomic per
      // wavefront and chunk that has any
      auto append = [&](bool pass, float dist, int qcur, u32 i) {
        const u64 mask = __ballot(pass);
        if (mask == 0) return;
        const int n = __popcll(mask);
        const int leader = (int)__builtin_ctzll(mask);
        u32 at = 0;
        if (lane == leader) at = atomicAdd(&cand_count[qcur], (u32)n);
        at = (u32)__builtin_amdgcn_readlane((int)at, leader);
        if (pass) {
          const u32 pos = at + (u32)__popcll(mask & ((1ull << lane) - 1ull));
          if (pos < (u32)cap) cand[(u64)qcur * (u64)cap + pos] = make_key(dist, i, 0);
          else overflow[qcur] = 1u;
        }
      };
      auto consume = [&](CodeWords<M>& cw) {
        cw.template wait_newer<2 * NLT>();
        if (base_c == cb) {                                     // (uniform) first chunk of unit pc
          // the slices were requested at the first chunk of the unit before (or ahead of the loop):
          // only this step's request is younger.  r = q - c, one fp32 subtraction per component.
          float ra[DSUB], rb[DSUB];
#pragma unroll
          for (int u = 0; u < DSUB; ++u)
            asm volatile("s_waitcnt vmcnt(%3)\n\tv_sub_f32 %0, %1, %2" : "=v"(ra[u]) : "v"(qa[u]), "v"(cl[u]), "n"(NLT) : "memory");
#pragma unroll
          for (int u = 0; u < DSUB; ++u)
            asm volatile("s_waitcnt vmcnt(%3)\n\tv_sub_f32 %0, %1, %2" : "=v"(rb[u]) : "v"(qb[u]), "v"(cl[u]), "n"(NLT) : "memory");
          request_queries(pc + 1);
          const bool single = 2 * pc + 1 >= nl;
          bias_a = s_bias[2 * pc];
          bnd_a = s_bnd[2 * pc];
          q_a = __builtin_amdgcn_readfirstlane(s_q[2 * pc]);
          bias_b = single ? bias_a : s_bias[2 * pc + 1];
          bnd_b = single ? -__builtin_inff() : s_bnd[2 * pc + 1];
          q_b = single ? q_a : __builtin_amdgcn_readfirstlane(s_q[2 * pc + 1]);
          block_sync_lds();   // the scan of the unit before has finished everywhere: its tables may go
#pragma unroll
          for (int i = 0; i < EPL; ++i) {
            float acc_a = TN[i], acc_b = TN[i];
#pragma unroll
            for (int u = 0; u < DSUB; ++u) {
              acc_a = __builtin_fmaf(ra[u], T[i * DSUB + u], acc_a);
              acc_b = __builtin_fmaf(rb[u], T[i * DSUB + u], acc_b);
            }
#pragma unroll
            for (int c = 0; c < REP; ++c) {
              float* e = lut0 + (jg * EPL + i) * 64 + m_own + M * ((rep0 + c) & (REP - 1));
              e[0] = acc_a;
              e[32] = acc_b;
            }
          }
          block_sync_lds();   // both tables are visible
        }
        const u32 i = base_c + (u32)tid;
        const bool valid = i < ce;
        float da = bias_a, db = bias_b;
        if (valid) cw.adc_banked2(col, da, db);
        da = fmaxf(da, 0.f);                                    // as the query-major kernel
        db = fmaxf(db, 0.f);
        // not worse in VALUE than the bound: a code that ties with the k-th best may still win on its id
        append(valid && !(da > bnd_a), da, q_a, i);
        append(valid && !(db > bnd_b), db, q_b, i);
        base_c += NT;
        if (base_c >= ce) { ++pc; base_c = cb; }
      };
      request_queries(0);
      request(S0);
      request(S1);
      for (;;) {
        request(S2); consume(S0);
        if (pc >= nu) break;
        request(S0); consume(S1);
        if (pc >= nu) break;
        request(S1); consume(S2);
        if (pc >= nu) break;
      }
      // the last requests land while their registers still belong to them (see the query-major kernel)
      S0.drain(); S1.drain(); S2.drain();
#pragma unroll
      for (int u = 0; u < DSUB; ++u) asm volatile("s_waitcnt vmcnt(0)" : "+v"(qa[u]), "+v"(qb[u]) : : "memory");
      block_sync_lds();   // everyone is done with the group's entries in LDS
    }
  }
}

// Bounds, counters and flags of a batch, and the number of pairs per list: one lane per (query,
// probe).  first[q][k] holds the k best keys of the query's first p_first probes, best first; the
// bound is the value of the k-th (+inf while there are fewer than k).  list_count must be zero.
__global__ __launch_bounds__(256) void lm_prepare_kernel(const int32_t* __restrict__ probes, int64_t nq,
                                                         int nprobe, int p_first,
                                                         const int64_t* __restrict__ list_off,
                                                         const u64* __restrict__ first, int k,
                                                         float* __restrict__ qbound, u32* __restrict__ cand_count,
                                                         u32* __restrict__ overflow, u32* __restrict__ list_count,
                                                         u32* __restrict__ rescan_count) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= nq * nprobe) return;
  if (i == 0) *rescan_count = 0u;
  const int64_t qi = i / nprobe;
  const int p = (int)(i - qi * nprobe);
  if (p == 0) {
    const u64 kth = first[qi * k + (k - 1)];
    qbound[qi] = kth == KEY_EMPTY ? __builtin_inff() : key_value(kth, 0);
    cand_count[qi] = 0u;
    overflow[qi] = 0u;
  }
  if (p < p_first) return;
  const int l = probes[i];
  if (l >= 0 && list_off[l + 1] > list_off[l]) atomicAdd(&list_count[l], 1u);
}

// pair_off = exclusive prefix sums of list_count (nlist + 1 entries), in two launches: sums of
// blocks of 1024 lists, then every block scans its lists starting from the sum of the blocks
// before it (at most a few hundred block sums, added up by every block for itself).  list_count
// itself is set back to zero to serve as the lists' fill cursors.
__global__ __launch_bounds__(1024) void lm_block_sums_kernel(const u32* __restrict__ list_count, int nlist,
                                                             u32* __restrict__ block_sum) {
  __shared__ u32 part[16];
  const int l = blockIdx.x * 1024 + threadIdx.x;
  u32 v = l < nlist ? list_count[l] : 0u;
  for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = v;
  __syncthreads();
  if (threadIdx.x == 0) {
    u32 t = 0;
    for (int w = 0; w < 16; ++w) t += part[w];
    block_sum[blockIdx.x] = t;
  }
}
__global__ __launch_bounds__(1024) void lm_offsets_kernel(u32* __restrict__ list_count, int nlist,
                                                          const u32* __restrict__ block_sum,
                                                          u32* __restrict__ pair_off) {
  __shared__ u32 part[1024];
  __shared__ u32 before;
  const int tid = threadIdx.x;
  const int l = blockIdx.x * 1024 + tid;
  if (tid == 0) {
    u32 t = 0;
    for (int b = 0; b < (int)blockIdx.x; ++b) t += block_sum[b];
    before = t;
  }
  const u32 own = l < nlist ? list_count[l] : 0u;
  part[tid] = own;
  __syncthreads();
  for (int off = 1; off < 1024; off <<= 1) {
    const u32 v = tid >= off ? part[tid - off] : 0u;
    __syncthreads();
    part[tid] += v;
    __syncthreads();
  }
  if (l < nlist) {
    pair_off[l] = before + part[tid] - own;                     // exclusive
    list_count[l] = 0u;
    if (l == nlist - 1) pair_off[nlist] = before + part[tid];
  }
}

__global__ __launch_bounds__(256) void lm_scatter_kernel(const int32_t* __restrict__ probes, int64_t nq,
                                                         int nprobe, int p_first,
                                                         const int64_t* __restrict__ list_off,
                                                         const u32* __restrict__ pair_off,
                                                         u32* __restrict__ cursor, u32* __restrict__ pairs) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= nq * nprobe) return;
  const int p = (int)(i % nprobe);
  if (p < p_first) return;
  const int l = probes[i];
  if (l >= 0 && list_off[l + 1] > list_off[l]) pairs[pair_off[l] + atomicAdd(&cursor[l], 1u)] = (u32)i;
}

// One wavefront per query: the k best of its first-stage keys and its candidates, best first.
// A query whose candidate buffer overflowed is put on the list of queries to scan again.
template <int R>
__global__ __launch_bounds__(64) void lm_merge_kernel(const u64* __restrict__ first,
                                                      const u32* __restrict__ cand_count,
                                                      const u64* __restrict__ cand, int cap, int k, int tot,
                                                      const int64_t* __restrict__ ids,
                                                      float* __restrict__ out_dist,
                                                      int64_t* __restrict__ out_ids,
                                                      const u32* __restrict__ overflow,
                                                      u32* __restrict__ rescan_list,
                                                      u32* __restrict__ rescan_count) {
  extern __shared__ u64 mslots[];
  const int64_t qi = blockIdx.x;
  const int lane = lane_id();
  if (lane == 0 && overflow[qi] != 0u) rescan_list[atomicAdd(rescan_count, 1u)] = (u32)qi;
  WaveSelect<R> ws;
  ws.init(mslots, tot, k);
  for (int j0 = 0; j0 < k; j0 += VS_WAVE) {
    const int j = j0 + lane;
    const u64 key = j < k ? first[qi * k + j] : KEY_EMPTY;
    ws.push(j < k && key != KEY_EMPTY, key);
  }
  const int n = (int)min(cand_count[qi], (u32)cap);
  const u64* __restrict__ src = cand + (u64)qi * (u64)cap;
  for (int j0 = 0; j0 < n; j0 += VS_WAVE) {
    const int j = j0 + lane;
    const u64 key = j < n ? src[j] : KEY_EMPTY;
    ws.push(j < n, key);
  }
  ws.finish();
  for (int j = lane; j < k; j += VS_WAVE) {
    const u64 key = ws.s[j];
    float v; int64_t id;
    if (key == KEY_EMPTY) { v = __builtin_inff(); id = -1; }
    else { v = key_value(key, 0); id = ids[key_index(key)]; }
    out_dist[qi * k + j] = v;
    out_ids[qi * k + j] = id;
  }
}

// ---------------------------------------------------------------------------
// Wavefront-private scan (Sec. 4.3 "Compressed-domain search") for 8-bit codes of M = 8 or 16
// sub-quantizers and the table forms whose per-(query, list) work is small: ONE WAVEFRONT per
// (query, probe split), nothing shared between wavefronts, so a CU runs nine independent streams
// and the latencies of one (its probes, the first codes of a list) are covered by the others --
// which is what lists of a few hundred codes need: there a (query, list) pair is one or two rounds
// of look-ups, and a workgroup that works through them together spends its time at barriers and on
// per-query set-up.
// MODE 1 (inner product) and MODE 2 (L2 through the stored norms): one table per query,
// A_q[j][m] = s <q_m, T_m[j]> with s = 1 or -2 (query_tables, written by pq_query_tables_kernel
// before this launch), copied to LDS once per work item; a list contributes one number (<q, c_l>,
// or |q - c_l|^2 - |c_l|^2) and, for MODE 2, every code its stored |x'|^2.
// MODE 3 (precomputed tables): the table of a pair is A_q + B_l with
// B_l[j][m] = |T_m[j]|^2 + 2 <c_{l,m}, T_m[j]> (list_tables, computed once per index); this lane's
// 4 * NI entries of A_q stay in registers for the whole item, and a list costs NI 16-byte loads,
// four additions and one 16-byte LDS store per lane each.  The distance of a code is the probe's
// coarse distance |q - c_l|^2 plus its M table entries.
// All of these are laid out [j][m], and so is the wavefront's table in LDS: rows of M floats.  The
// codes are stored rotated by their position in the list (rotate_code), so lane l finds
// sub-quantizer (t + l) mod M in byte t of its code.
// ---------------------------------------------------------------------------
typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr int kWaveScanShare = 2;   // wavefronts that share a per-query table (inner product, stored norms)

// One workgroup: the tables of kQtQueries queries.  A thread keeps one codebook entry T_m[j] in
// registers and takes the queries' sub-vectors from LDS.
constexpr int kQtQueries = 8;
template <int DSUB>
__global__ __launch_bounds__(256) void pq_query_tables_kernel(const float* __restrict__ q, int64_t nq,
                                                              const float* __restrict__ codebooks_by_entry, int d, int M,
                                                              int K, float scale, float* __restrict__ out) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float* qs = reinterpret_cast<float*>(smem);          // [kQtQueries][d]
  const int64_t q0 = (int64_t)blockIdx.x * kQtQueries;
  const int nqb = (int)min((int64_t)kQtQueries, nq - q0);
  for (int i = threadIdx.x; i < nqb * d; i += blockDim.x) qs[i] = q[q0 * d + i];
  __syncthreads();
  // a thread takes four consecutive entries e = j * M + m (one j, four m; M is a multiple of 4):
  // 4 * DSUB consecutive floats of codebooks_by_entry [K][M][DSUB], one 16-byte store per query
  for (int e4 = threadIdx.x; e4 < K * M / 4; e4 += blockDim.x) {
    const int m0 = (e4 * 4) % M;
    float T[4][DSUB];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int u = 0; u < DSUB; ++u) T[i][u] = codebooks_by_entry[((int64_t)e4 * 4 + i) * DSUB + u];
    for (int a = 0; a < nqb; ++a) {
      f32x4 r;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float acc = 0.f;
        if constexpr (DSUB % 4 == 0) {   // the query's sub-vector in 16-byte LDS reads
#pragma unroll
          for (int u4 = 0; u4 < DSUB / 4; ++u4) {
            const f32x4 qv = *reinterpret_cast<const f32x4*>(qs + a * d + (m0 + i) * DSUB + 4 * u4);
#pragma unroll
            for (int u = 0; u < 4; ++u) acc = __builtin_fmaf(qv[u], T[i][4 * u4 + u], acc);
          }
        } else {
#pragma unroll
          for (int u = 0; u < DSUB; ++u) acc = __builtin_fmaf(qs[a * d + (m0 + i) * DSUB + u], T[i][u], acc);
        }
        r[i] = scale * acc;
      }
      *reinterpret_cast<f32x4*>(out + (q0 + a) * K * M + (int64_t)e4 * 4) = r;
    }
  }
}

template <int M, int MODE, int R>
__global__ __launch_bounds__(MODE == 3 ? 64 : 64 * kWaveScanShare) void ivfpq_scan_wave_kernel(
    const float* __restrict__ query_tables, const float* __restrict__ list_tables,
    const int32_t* __restrict__ probes, const float* __restrict__ cdist, int nprobe, int ppb, int nsplit,
    const int64_t* __restrict__ list_off, const uint8_t* __restrict__ codes, const float* __restrict__ norms,
    const float* __restrict__ cnorm, int64_t ntotal, int k, int tot, KeySink sink) {
  constexpr int K = 256;
  constexpr int KEY_METRIC = MODE == 1 ? 1 : 0;
  constexpr int QPR = M / 4;          // 16-byte pieces per table row
  constexpr int RPI = 64 / QPR;       // rows one load instruction of the wavefront covers
  constexpr int NI = K / RPI;         // load instructions per table = 16-byte pieces per lane
  static_assert(M == 8 || M == 16, "rows of 8 or 16 floats");
  static_assert(MODE >= 1 && MODE <= 3, "table form");
  // MODE 1, 2: the table depends on the query alone, so NW wavefronts of one work item share it
  // (each scans every NW-th list of the item and selects on its own; the results are merged by
  // rank at the end): the LDS per wavefront shrinks and more wavefronts fit a CU, which is what
  // hides the latency of the per-list chain (extent -> first codes -> look-ups).
  constexpr int NW = MODE == 3 ? 1 : kWaveScanShare;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float* lut = reinterpret_cast<float*>(smem);                              // [256][M]
  const int lane = lane_id(), wave = threadIdx.x >> 6;
  u64* slots0 = reinterpret_cast<u64*>(smem + K * M * sizeof(float));       // NW x tot
  u64* slots = slots0 + wave * tot;
  u32* s_begin = reinterpret_cast<u32*>(slots0 + NW * tot) + wave * 4 * ppb; // ppb: this wavefront's non-empty lists
  u32* s_end = s_begin + ppb;
  int32_t* s_list = reinterpret_cast<int32_t*>(s_end + ppb);
  float* s_bias = reinterpret_cast<float*>(s_list + ppb);

  // (no static LDS: the table starts at LDS address 0 and a table offset is an LDS address; the
  // launcher checks this)
  const int64_t item = blockIdx.x;
  const int64_t qi = item / nsplit;
  const int split = (int)(item % nsplit);
  const int p_begin = split * ppb;
  const int np = ntotal > 0 ? min(nprobe, p_begin + ppb) - p_begin : 0;

  // this lane's pieces of the per-query term: piece i covers row (lane / QPR) + RPI * i, floats
  // 4 * (lane % QPR) .. + 3
  const int row0 = lane / QPR, quad = lane % QPR;
  f32x4 tq[MODE == 3 ? NI : 1];
  {
    const f32x4* __restrict__ src = reinterpret_cast<const f32x4*>(query_tables + qi * K * M) + lane;
    if constexpr (MODE == 3) {
#pragma unroll
      for (int i = 0; i < NI; ++i) tq[i] = src[i * 64];
    } else {   // wavefront w copies pieces w, w + NW, ...
#pragma unroll
      for (int i = 0; i < NI / NW; ++i) {
        const int ii = i * NW + wave;
        *reinterpret_cast<f32x4*>(lut + (row0 + RPI * ii) * M + 4 * quad) = src[ii * 64];
      }
    }
  }
  WaveSelect<R> ws;
  ws.init(slots, tot, k);
  ws.set_metric(KEY_METRIC);
  int nl = 0;
  for (int p0 = 0; p0 < np; p0 += VS_WAVE * NW) {   // this wavefront's non-empty lists, in probe order
    const int p = p0 + lane * NW + wave;            // (dealt out in turn: the probes come sorted by distance)
    const int l = p < np ? probes[qi * nprobe + p_begin + p] : -1;
    const int64_t b = l >= 0 ? list_off[l] : 0, e = l >= 0 ? list_off[l + 1] : 0;
    const bool keep = e > b;
    const u64 mask = __ballot(keep);
    const int pos = nl + __popcll(mask & ((1ull << lane) - 1ull));
    if (keep) {
      s_list[pos] = l;
      s_begin[pos] = (u32)b;
      s_end[pos] = (u32)e;
      float bs = cdist[qi * nprobe + p_begin + p];
      if (MODE == 2) bs -= cnorm[l];
      s_bias[pos] = bs;
    }
    nl += __popcll(mask);
  }
  if constexpr (NW == 1) wave_lds_sync();
  else block_sync_lds();                            // the shared table is complete
  // byte offset of this lane's column in a row for every step, four steps per register, in units
  // that leave room for it in one byte: v_perm_b32 puts the code byte j into byte 1 and this into
  // byte 0, and one shift turns (j << 8 | unit * column) into the byte offset j * 4 M + 4 * column
  constexpr int kShift = M == 16 ? 2 : 3;
  u32 col[M / 4];
#pragma unroll
  for (int w = 0; w < M / 4; ++w) {
    u32 v = 0;
#pragma unroll
    for (int b = 0; b < 4; ++b) v |= (u32)(((4 * w + b + lane) & (M - 1)) << (2 + kShift)) << (8 * b);
    col[w] = v;
  }
  auto load_codes = [&](CodeWords<M>& w, u32 i) {
    const uint8_t* cp = codes + (u64)i * M;
    if constexpr (M == 16) w.a = *reinterpret_cast<const u32x4*>(cp);
    else w.a2 = *reinterpret_cast<const u32x2*>(cp);
  };
  // The chunks of 64 codes of all the item's lists form one sequence; the codes of the chunk after
  // the current one -- the next of this list or the first of the next list -- are requested before
  // the current chunk's look-ups (lanes past a list's end read the chunk's first code).
  auto list_at = [&](int pl, u32& begin, u32& end) {
    begin = __builtin_amdgcn_readfirstlane(s_begin[pl]);
    end = __builtin_amdgcn_readfirstlane(s_end[pl]);
  };
  int pl = 0;
  u32 base = 0, end = 0;
  bool first = true;     // the current chunk is the first of its list (uniform)
  CodeWords<M> cw;
  float nrm = 0.f, bias = 0.f;
  if (nl > 0) {
    list_at(0, base, end);
    const u32 i = base + (u32)lane;
    const u32 at = i < end ? i : base;
    load_codes(cw, at);
    if (MODE == 2) nrm = norms[at];
  }
  while (pl < nl) {
    int npl = pl;
    u32 nbase = base + VS_WAVE, nend = end;
    if (nbase >= end) {
      ++npl;
      if (npl < nl) list_at(npl, nbase, nend);
    }
    CodeWords<M> nx;
    float nrm_nx = 0.f;
    if (npl < nl) {
      const u32 i2 = nbase + (u32)lane;
      const u32 at = i2 < nend ? i2 : nbase;
      load_codes(nx, at);
      if (MODE == 2) nrm_nx = norms[at];
    }
    if (first) {
      bias = s_bias[pl];
      if constexpr (MODE == 3) {
        const int l = __builtin_amdgcn_readfirstlane(s_list[pl]);
        const f32x4* __restrict__ tls = reinterpret_cast<const f32x4*>(list_tables + (int64_t)l * K * M) + lane;
        f32x4 tl[NI];
#pragma unroll
        for (int i = 0; i < NI; ++i) tl[i] = tls[i * 64];
        wave_lds_sync();     // the look-ups of the list before are done with the table
#pragma unroll
        for (int i = 0; i < NI; ++i)
          *reinterpret_cast<f32x4*>(lut + (row0 + RPI * i) * M + 4 * quad) = tq[i] + tl[i];
        wave_lds_sync();
      }
    }
    const u32 i = base + (u32)lane;
    const bool valid = i < end;
    float dist = MODE == 2 ? bias + nrm : bias;
#pragma unroll
    for (int t = 0; t < M; ++t) {
      constexpr u32 sel0 = 0x0c0c0400u;   // byte 1 = byte (t & 3) of the code word, byte 0 = of col
      const u32 a = __builtin_amdgcn_perm(cw.word(t >> 2), col[t >> 2], sel0 + 0x101u * (t & 3)) >> kShift;
      dist += *reinterpret_cast<lds_cfloat_ptr>((uintptr_t)a);
    }
    if (MODE != 1) dist = fmaxf(dist, 0.f);   // a squared distance: the expanded square can round below zero
    ws.push_value(valid, dist, i);
    first = npl != pl;
    pl = npl; base = nbase; end = nend;
    if (pl < nl) { cw = nx; nrm = nrm_nx; }
  }
  ws.finish();
  if constexpr (NW == 1) {
    for (int j = lane; j < k; j += VS_WAVE) sink.put(item * k + j, ws.s[j]);
  } else {
    block_sync_lds();
    block_rank_merge(slots0, tot, NW, k, sink, item * k);
  }
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

__global__ void pq_codebooks_by_entry_kernel(const float* __restrict__ codebooks, int M, int K, int dsub,
                                             float* __restrict__ out) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;      // index into out: (j, m, u)
  if (i >= M * K * dsub) return;
  const int u = i % dsub, m = (i / dsub) % M, j = i / (dsub * M);
  out[i] = codebooks[((int64_t)m * K + j) * dsub + u];
}

// One lane per (query, probe): the inner product of the query with the probed centroid, canon chain.
__global__ __launch_bounds__(256) void probe_inner_products_kernel(const float* __restrict__ q, int64_t nq, int d,
                                                                   const float* __restrict__ centroids,
                                                                   const int32_t* __restrict__ probes, int nprobe,
                                                                   float* __restrict__ cdist) {
  const int64_t e = blockIdx.x * 256ll + threadIdx.x;
  if (e >= nq * nprobe) return;
  const int l = probes[e];
  if (l < 0) return;
  const float* __restrict__ qa = q + (e / nprobe) * d;
  const float* __restrict__ c = centroids + (int64_t)l * d;
  float acc = 0.f;
  for (int t = 0; t < d; ++t) acc = __builtin_fmaf(qa[t], c[t], acc);
  cdist[e] = acc;
}

// What one search scanned: list sizes summed over its (query, probe) pairs.  stats was zeroed in
// stream order before this launch.
__global__ __launch_bounds__(256) void search_stats_kernel(const int32_t* __restrict__ probes, int64_t n,
                                                           const int64_t* __restrict__ list_off,
                                                           const int* __restrict__ fallback_count,
                                                           int64_t mfma_rows, int nprobe, int p_first,
                                                           unsigned long long* __restrict__ stats) {
  unsigned long long codes = 0, lists = 0, first = 0;
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
    const int l = probes[i];
    if (l < 0) continue;
    const unsigned long long sz = (unsigned long long)(list_off[l + 1] - list_off[l]);
    codes += sz;
    lists += sz > 0 ? 1ull : 0ull;
    if ((int)(i % nprobe) < p_first) first += sz;
  }
  for (int o = 32; o > 0; o >>= 1) {
    codes += __shfl_down(codes, o, 64);
    lists += __shfl_down(lists, o, 64);
    first += __shfl_down(first, o, 64);
  }
  // one pair of atomics per workgroup (thousands of wavefronts adding to the same two words
  // serialise: 63 us for 160k pairs)
  __shared__ unsigned long long part[3][4];
  if ((threadIdx.x & 63) == 0) {
    part[0][threadIdx.x >> 6] = codes; part[1][threadIdx.x >> 6] = lists; part[2][threadIdx.x >> 6] = first;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    codes = part[0][0] + part[0][1] + part[0][2] + part[0][3];
    lists = part[1][0] + part[1][1] + part[1][2] + part[1][3];
    first = part[2][0] + part[2][1] + part[2][2] + part[2][3];
    if (codes) atomicAdd(&stats[0], codes);
    if (lists) atomicAdd(&stats[1], lists);
    if (first) atomicAdd(&stats[5], first);
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    stats[2] = (unsigned long long)mfma_rows;
    stats[3] = fallback_count ? (unsigned long long)*fallback_count : 0ull;
    stats[4] = (unsigned long long)p_first;
  }
}
__global__ void search_stats_rescan_kernel(const unsigned* __restrict__ rescan_count,
                                           unsigned long long* __restrict__ stats) {
  stats[6] = (unsigned long long)*rescan_count;
}

// ------------------------------------------------------------------ launchers

// Shapes served by ivfpq_scan_bank_kernel; an index of such a shape stores its codes rotated.
bool ivfpq_codes_rotated(const IvfpqDims& g) {
  return g.nbits == 8 && ((g.M == 16 && g.dsub == 8) || (g.M == 32 && g.dsub == 3) || (g.M == 8 && g.dsub == 4));
}
// The wavefront-private kernel (one wavefront per (query, probe split), rows of M floats) serves the
// rotated shapes with M = 8 or 16 while the lists are short: with long lists the workgroup-wide
// kernel streams better.
bool ivfpq_wave_scan_applies(const IvfpqDims& g, int64_t ntotal) {
  return ivfpq_codes_rotated(g) && (g.M == 8 || g.M == 16) && ntotal <= (int64_t)g.nlist * kWaveScanMaxMeanList;
}
constexpr int kBankThreads = 256;   // 4 wavefronts per workgroup, two workgroups per CU
static size_t bank_scan_lds_bytes(int tot, int ppb) {
  return (size_t)kBankTableBytes + (size_t)((kBankThreads / 64) * tot + 2) * sizeof(u64) + (size_t)ppb * 16 + 24;
}
// Selection slots per wavefront for the bank kernel: as for the other kernels (a power of two >=
// k + 64) unless a multiple of 32 between k + 64 and that lets two workgroups share a CU's LDS.
static int bank_slots_for_k(int k, int ppb) {
  const int tot = select_slots_for_k(k);
  if (tot > 256) return tot;                               // sorted through LDS: powers of two only
  if (2 * bank_scan_lds_bytes(tot, ppb) <= 160 * 1024) return tot;
  for (int t = tot - 32; t >= k + 64; t -= 32)
    if (2 * bank_scan_lds_bytes(t, ppb) <= 160 * 1024) return t;
  return tot;
}

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
                     const int64_t* dest, const int32_t* new_list_of, int64_t n_new, uint8_t* codes,
                     int64_t* ids, float* norms, hipStream_t st) {
  // (old entries keep their position inside their list, hence their rotation)
  if (old_total > 0)
    hipLaunchKernelGGL(move_old_kernel, dim3((unsigned)((old_total + 255) / 256)), dim3(256), 0, st,
                       old_codes, old_ids, old_norms, old_total, old_off, new_off, g.nlist,
                       g.code_size, codes, ids, norms);
  if (n_new > 0)
    hipLaunchKernelGGL(scatter_new_kernel, dim3((unsigned)((n_new + 255) / 256)), dim3(256), 0, st,
                       tmp_codes, new_ids_or_null, id_base, tmp_norms, dest, n_new, g.M, g.nbits,
                       g.code_size, ivfpq_codes_rotated(g) ? g.M : 0, new_list_of, new_off, codes, ids,
                       norms);
}

void launch_codes_canonical(const IvfpqDims& g, const uint8_t* stored, const int64_t* off,
                            int64_t total, uint8_t* out, hipStream_t st) {
  if (total <= 0) return;
  hipLaunchKernelGGL(unrotate_codes_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                     stored, off, g.nlist, total, g.M, out);
}

void launch_pq_norms(const IvfpqDims& g, const uint8_t* tmp_codes, int64_t n, const int32_t* list_of,
                     const float* centroids, const float* codebooks, float* tmp_norms,
                     hipStream_t st, bool stored_form) {
  if (n <= 0) return;
  hipLaunchKernelGGL(pq_norms_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, tmp_codes,
                     n, g.d, g.dsub, g.K, g.M, stored_form && g.nbits == 4, list_of, centroids, codebooks,
                     tmp_norms);
}

void launch_row_norms(const float* x, int64_t n, int d, float* norms, hipStream_t st) {
  if (n <= 0) return;
  hipLaunchKernelGGL(row_norms_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, x, n, d, norms);
}

void launch_probe_inner_products(const float* q, int64_t nq, int d, const float* centroids,
                                 const int32_t* probes, int nprobe, float* cdist, hipStream_t st) {
  const int64_t n = nq * nprobe;
  if (n <= 0) return;
  hipLaunchKernelGGL(probe_inner_products_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, q, nq, d,
                     centroids, probes, nprobe, cdist);
}

void launch_search_stats(const int32_t* probes, int64_t n, const int64_t* list_off, const int* fallback_count,
                         int64_t mfma_rows, int nprobe, int p_first, long long* stats, hipStream_t st) {
  launch_fill_u64(reinterpret_cast<u64*>(stats), 7, 0ull, st);
  const int64_t blocks = std::max<int64_t>(1, std::min<int64_t>(256, (n + 255) / 256));
  hipLaunchKernelGGL(search_stats_kernel, dim3((unsigned)blocks), dim3(256), 0, st, probes, n, list_off,
                     fallback_count, mfma_rows, nprobe, p_first, reinterpret_cast<unsigned long long*>(stats));
}
void launch_search_stats_rescan(const unsigned* rescan_count, long long* stats, hipStream_t st) {
  hipLaunchKernelGGL(search_stats_rescan_kernel, dim3(1), dim3(1), 0, st, rescan_count,
                     reinterpret_cast<unsigned long long*>(stats));
}

void launch_pq_codebooks_by_entry(const IvfpqDims& g, const float* codebooks, float* out, hipStream_t st) {
  const int n = g.M * g.K * g.dsub;
  hipLaunchKernelGGL(pq_codebooks_by_entry_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, codebooks,
                     g.M, g.K, g.dsub, out);
}

void launch_pq_list_tables(const IvfpqDims& g, const float* centroids, const float* codebooks, float* out,
                           hipStream_t st) {
  const int64_t n = (int64_t)g.nlist * g.K * g.M;
  hipLaunchKernelGGL(pq_list_tables_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, centroids,
                     codebooks, g.nlist, g.d, g.M, g.K, g.dsub, out);
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

// A kernel without static LDS has its dynamic LDS at LDS address 0, which the bank-private and the
// wavefront-private scans rely on (a table offset is used as an LDS address).
static bool dynamic_lds_starts_at_zero(const void* kernel) {
  hipFuncAttributes attr;
  return hipFuncGetAttributes(&attr, kernel) == hipSuccess && attr.sharedSizeBytes == 0;
}

template <int M, int DSUB, int METRIC, int R>
static int launch_scan_bank(const IvfpqDims& g, const float* q, int64_t nq, const float* centroids,
                             const float* codebooks, const int32_t* probes, const float* cdist,
                             int nprobe, int ppb, int nsplit, const int64_t* list_off,
                             const uint8_t* codes, const float* norms, const float* cnorm,
                             const float* list_tables, int64_t ntotal, int k, int tot, KeySink sink,
                             u64* counter, hipStream_t st, const u32* item_list = nullptr,
                             const u32* item_count = nullptr) {
  const size_t shmem = bank_scan_lds_bytes(tot, ppb);
  constexpr int NT = kBankThreads;
  auto kern = &ivfpq_scan_bank_kernel<M, DSUB, METRIC, R, NT>;
  static const bool at_zero = dynamic_lds_starts_at_zero(reinterpret_cast<const void*>(kern));
  if (!at_zero) return -1;
  if (shmem > 48 * 1024)
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
  const int64_t nitems = nq * nsplit;
  // persistent workgroups: as many as are resident at once on the 256 CUs, each walks over items
  int per_cu = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, NT, shmem) != hipSuccess || per_cu < 1)
    per_cu = 1;
  const int64_t grid = std::min<int64_t>(nitems, 256ll * per_cu);
  launch_fill_u64(counter, 1, 0ull, st);
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(NT), shmem, st, q, centroids, codebooks,
                     probes, cdist, nprobe, ppb, nsplit, nitems, list_off, codes, norms, cnorm, list_tables,
                     ntotal, k, tot, sink, reinterpret_cast<unsigned long long*>(counter), item_list, item_count);
  return 0;
}

template <int M, int DSUB>
static int launch_scan_bank_any(const IvfpqDims& g, const float* q, int64_t nq,
                                 const float* centroids, const float* codebooks,
                                 const int32_t* probes, const float* cdist, int nprobe, int ppb,
                                 int nsplit, const int64_t* list_off, const uint8_t* codes,
                                 const float* norms, const float* cnorm, const float* list_tables,
                                 int mode, int64_t ntotal, int k, int tot, KeySink sink, u64* counter,
                                 hipStream_t st) {
#define GO(MET, RR)                                                                               \
  return launch_scan_bank<M, DSUB, MET, RR>(g, q, nq, centroids, codebooks, probes, cdist, nprobe, ppb,  \
                                            nsplit, list_off, codes, norms, cnorm, list_tables, ntotal, k, tot, sink, counter, st)
  const int r = tot <= 128 ? 2 : (tot <= 256 ? 4 : 0);   // register-sort width covering the slots
  if (mode == 1)      { if (r == 2) GO(1, 2); else if (r == 4) GO(1, 4); else GO(1, 0); }
  else if (mode == 2) { if (r == 2) GO(2, 2); else if (r == 4) GO(2, 4); else GO(2, 0); }
  else if (mode == 3) { if (r == 2) GO(3, 2); else if (r == 4) GO(3, 4); else GO(3, 0); }
  else                { if (r == 2) GO(0, 2); else if (r == 4) GO(0, 4); else GO(0, 0); }
#undef GO
}

// Work space the wavefront-private kernel needs: one table per query, [nq][K][M] floats.
size_t ivfpq_query_table_bytes(const IvfpqDims& g, int64_t nq) {
  return (size_t)nq * g.K * g.M * sizeof(float);
}
static size_t wave_scan_lds_bytes(const IvfpqDims& g, int mode, int tot, int ppb) {
  const int nw = mode == 3 ? 1 : kWaveScanShare;
  return (size_t)g.K * g.M * sizeof(float) + (size_t)nw * ((size_t)tot * sizeof(u64) + (size_t)ppb * 16);
}
template <int M, int DSUB, int MODE>
static int launch_scan_wave(const IvfpqDims& g, const float* q, int64_t nq, const float* codebooks,
                             float* query_tables, const float* list_tables, const int32_t* probes,
                             const float* cdist, int nprobe, int ppb, int nsplit, const int64_t* list_off,
                             const uint8_t* codes, const float* norms, const float* cnorm, int64_t ntotal,
                             int k, KeySink sink, hipStream_t st) {
  hipLaunchKernelGGL((pq_query_tables_kernel<DSUB>), dim3((unsigned)((nq + kQtQueries - 1) / kQtQueries)),
                     dim3(256), (size_t)kQtQueries * g.d * sizeof(float), st, q, nq,
                     codebooks + (size_t)g.M * g.K * g.dsub, g.d, g.M, g.K, MODE == 1 ? 1.f : -2.f, query_tables);
  const int tot = select_slots_for_k(k);
  const size_t shmem = wave_scan_lds_bytes(g, MODE, tot, ppb);
  const dim3 grid((unsigned)(nq * nsplit)), block(MODE == 3 ? 64 : 64 * kWaveScanShare);
#define GO(RR)                                                                                        \
  do {                                                                                                \
    auto kern = &ivfpq_scan_wave_kernel<M, MODE, RR>;                                                 \
    static const bool at_zero = dynamic_lds_starts_at_zero(reinterpret_cast<const void*>(kern));      \
    if (!at_zero) return -1;                                                                          \
    if (shmem > 48 * 1024)                                                                            \
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                                  \
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);              \
    hipLaunchKernelGGL(kern, grid, block, shmem, st, query_tables, list_tables, probes, cdist, nprobe, \
                       ppb, nsplit, list_off, codes, norms, cnorm, ntotal, k, tot, sink);             \
  } while (0)
  const int r = select_regs_for_slots(tot);
  if (r == 2) GO(2); else if (r == 4) GO(4); else GO(0);
#undef GO
  return 0;
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
                      const float* norms, const float* cnorm, const float* list_tables,
                      float* query_tables, int64_t ntotal, int k, u64* partial, u64* counter,
                      const int64_t* ids, float* out_dist, int64_t* out_ids, hipStream_t st) {
  if (nq <= 0) return 0;
  // table form: 1 inner product; 2 L2 through the stored norms (norms non-null; cnorm = the
  // centroids' squared norms); 0 L2 with one table of squared residual distances per (query, list)
  // 3: L2 with per-list terms of the tables precomputed (list_tables non-null; bank kernel shapes only)
  const int mode = g.metric == 1 ? 1 : (norms ? 2 : (list_tables && ivfpq_codes_rotated(g) ? 3 : 0));
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
  if (mode != 0 && query_tables && ivfpq_wave_scan_applies(g, ntotal)) {
    if (wave_scan_lds_bytes(g, mode, select_slots_for_k(k), ppb) > 160 * 1024) return -1;
#define WAVE(MM, DS, MODE)                                                                             \
  return launch_scan_wave<MM, DS, MODE>(g, q, nq, codebooks, query_tables, list_tables, probes, cdist, nprobe, \
                                 ppb, nsplit, list_off, codes, norms, cnorm, ntotal, k, sink, st)
    if (g.M == 16) { if (mode == 1) WAVE(16, 8, 1); else if (mode == 2) WAVE(16, 8, 2); else WAVE(16, 8, 3); }
    else           { if (mode == 1) WAVE(8, 4, 1); else if (mode == 2) WAVE(8, 4, 2); else WAVE(8, 4, 3); }
#undef WAVE
  }
  if (ivfpq_codes_rotated(g)) {   // (the stored codes are rotated: no other kernel reads them)
    const int btot = bank_slots_for_k(k, ppb);
    if (bank_scan_lds_bytes(btot, ppb) > 160 * 1024) return -1;
#define BANK(MM, DS)                                                                              \
  if (g.M == MM && g.dsub == DS) {                                                                \
    return launch_scan_bank_any<MM, DS>(g, q, nq, centroids, codebooks, probes, cdist, nprobe, ppb, \
                                        nsplit, list_off, codes, norms, cnorm, list_tables, mode, ntotal, k, btot, sink, counter, st); \
  }
    BANK(16, 8)   // PQ16x8 on d = 128
    BANK(32, 3)   // PQ32x8 on d = 96
    BANK(8, 4)    // PQ8x8 on d = 32
#undef BANK
    return -1;
  }
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


// ---- list-major scan: work space and launches ---------------------------------------------
// The work space behind `lm`: bounds [nq] f32, candidate counts [nq] u32, overflow flags [nq] u32,
// the queries to scan again [nq] u32 and their number,
// pairs per list / fill cursors [nlist] u32, their sums per 1024 lists, pair offsets [nlist + 1] u32, pairs [nq * nprobe]
// u32, candidates [nq][cap] u64.
namespace {
struct LmLayout { size_t o_bound, o_count, o_flag, o_rlist, o_rcount, o_lcount, o_bsum, o_poff, o_pairs, o_cand, bytes; };
LmLayout lm_layout(int64_t nq, int nprobe, int nlist, int cap) {
  auto up = [](size_t v) { return (v + 255) / 256 * 256; };
  LmLayout L;
  size_t o = 0;
  L.o_bound = o; o += up((size_t)nq * sizeof(float));
  L.o_count = o; o += up((size_t)nq * sizeof(u32));
  L.o_flag = o; o += up((size_t)nq * sizeof(u32));
  L.o_rlist = o; o += up((size_t)nq * sizeof(u32));
  L.o_rcount = o; o += up(sizeof(u32));
  L.o_lcount = o; o += up((size_t)nlist * sizeof(u32));
  L.o_bsum = o; o += up((size_t)((nlist + 1023) / 1024) * sizeof(u32));
  L.o_poff = o; o += up((size_t)(nlist + 1) * sizeof(u32));
  L.o_pairs = o; o += up((size_t)nq * nprobe * sizeof(u32));
  L.o_cand = o; o += up((size_t)nq * cap * sizeof(u64));
  L.bytes = o;
  return L;
}
size_t lm_scan_lds_bytes() { return (size_t)kBankTableBytes + 16 + (size_t)3 * kLmGroup * 4; }
}  // namespace

bool ivfpq_listmajor_shape(const IvfpqDims& g) {
  return ivfpq_codes_rotated(g) && g.metric == 0 &&
         ((g.M == 32 && g.dsub == 3) || (g.M == 16 && g.dsub == 8) || (g.M == 8 && g.dsub == 4));
}
size_t ivfpq_listmajor_bytes(const IvfpqDims& g, int64_t nq, int nprobe, int cap) {
  return lm_layout(nq, nprobe, g.nlist, cap).bytes;
}

// The three parts of a list-major search, launched one after the other by the caller (which times
// them apart): `part` 0 = the first p_first probes of every query, query-major, k best keys per
// query into `first`, then the bounds and the pairs of the remaining probes grouped by list;
// 1 = the list-major scan; 2 = k best of first-stage keys and candidates per query, then the
// query-major kernel over all probes of the queries whose candidate buffer overflowed.
template <int M, int DSUB>
static int launch_listmajor_t(int part, const IvfpqDims& g, const float* q, int64_t nq, const float* centroids,
                              const float* codebooks, const int32_t* probes, const float* cdist, int nprobe,
                              int p_first, int cap, const int64_t* list_off, const uint8_t* codes,
                              int64_t ntotal, int k, u64* first, u64* counter, char* lm, const int64_t* ids,
                              float* out_dist, int64_t* out_ids, hipStream_t st) {
  const LmLayout L = lm_layout(nq, nprobe, g.nlist, cap);
  float* qbound = reinterpret_cast<float*>(lm + L.o_bound);
  u32* cand_count = reinterpret_cast<u32*>(lm + L.o_count);
  u32* flag = reinterpret_cast<u32*>(lm + L.o_flag);
  u32* rlist = reinterpret_cast<u32*>(lm + L.o_rlist);
  u32* rcount = reinterpret_cast<u32*>(lm + L.o_rcount);
  u32* lcount = reinterpret_cast<u32*>(lm + L.o_lcount);
  u32* bsum = reinterpret_cast<u32*>(lm + L.o_bsum);
  u32* poff = reinterpret_cast<u32*>(lm + L.o_poff);
  u32* pairs = reinterpret_cast<u32*>(lm + L.o_pairs);
  u64* cand = reinterpret_cast<u64*>(lm + L.o_cand);
  const int tot_a = bank_slots_for_k(k, p_first), tot_b = bank_slots_for_k(k, nprobe);
  if (bank_scan_lds_bytes(tot_a, p_first) > 160 * 1024 || bank_scan_lds_bytes(tot_b, nprobe) > 160 * 1024) return -1;
  auto scan_kern = &ivfpq_scan_listmajor_kernel<M, DSUB, kBankThreads>;
  static const bool at_zero = dynamic_lds_starts_at_zero(reinterpret_cast<const void*>(scan_kern));
  if (!at_zero) return -1;
  if (part == 0) {
    KeySink keys;
    keys.metric = 0; keys.keys = first; keys.val = nullptr; keys.id64 = nullptr; keys.idx32 = nullptr; keys.idmap = nullptr;
    const int ra = tot_a <= 128 ? 2 : (tot_a <= 256 ? 4 : 0);
#define BANK_A(RR) launch_scan_bank<M, DSUB, 0, RR>(g, q, nq, centroids, codebooks, probes, cdist, nprobe, p_first, 1, \
                                                    list_off, codes, nullptr, nullptr, nullptr, ntotal, k, tot_a, keys, counter, st)
    const int rc = ra == 2 ? BANK_A(2) : (ra == 4 ? BANK_A(4) : BANK_A(0));
#undef BANK_A
    if (rc != 0) return rc;
    launch_fill_u64(reinterpret_cast<u64*>(lcount), (int64_t)((g.nlist + 1) / 2), 0ull, st);
    const unsigned gp = (unsigned)((nq * nprobe + 255) / 256);
    hipLaunchKernelGGL(lm_prepare_kernel, dim3(gp), dim3(256), 0, st, probes, nq, nprobe, p_first, list_off, first, k,
                       qbound, cand_count, flag, lcount, rcount);
    const unsigned nblk = (unsigned)((g.nlist + 1023) / 1024);
    hipLaunchKernelGGL(lm_block_sums_kernel, dim3(nblk), dim3(1024), 0, st, lcount, g.nlist, bsum);
    hipLaunchKernelGGL(lm_offsets_kernel, dim3(nblk), dim3(1024), 0, st, lcount, g.nlist, bsum, poff);
    hipLaunchKernelGGL(lm_scatter_kernel, dim3(gp), dim3(256), 0, st, probes, nq, nprobe, p_first, list_off, poff,
                       lcount, pairs);
    launch_fill_u64(counter, 1, 0ull, st);   // (the work counter of the scan that follows)
    return 0;
  }
  if (part == 1) {
    const size_t shmem = lm_scan_lds_bytes();
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(scan_kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)shmem);
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, scan_kern, kBankThreads, shmem) != hipSuccess || per_cu < 1)
      per_cu = 1;
    const int64_t grid = std::min<int64_t>(g.nlist, 256ll * per_cu);
    hipLaunchKernelGGL(scan_kern, dim3((unsigned)grid), dim3(kBankThreads), shmem, st, q, centroids, codebooks, cdist,
                       nprobe, poff, pairs, g.nlist, list_off, codes, qbound, cand_count, cand, cap, flag,
                       reinterpret_cast<unsigned long long*>(counter));
    return 0;
  }
  {
    const int tot = select_slots_for_k(k);
    const size_t shmem = (size_t)tot * sizeof(u64);
    const dim3 grid((unsigned)nq), block(64);
    switch (select_regs_for_slots(tot)) {
      case 2: hipLaunchKernelGGL((lm_merge_kernel<2>), grid, block, shmem, st, first, cand_count, cand, cap, k, tot, ids, out_dist, out_ids, flag, rlist, rcount); break;
      case 4: hipLaunchKernelGGL((lm_merge_kernel<4>), grid, block, shmem, st, first, cand_count, cand, cap, k, tot, ids, out_dist, out_ids, flag, rlist, rcount); break;
      default: hipLaunchKernelGGL((lm_merge_kernel<0>), grid, block, shmem, st, first, cand_count, cand, cap, k, tot, ids, out_dist, out_ids, flag, rlist, rcount); break;
    }
  }
  KeySink fin;
  fin.metric = 0; fin.keys = nullptr; fin.val = out_dist; fin.id64 = out_ids; fin.idx32 = nullptr; fin.idmap = ids;
  const int rb = tot_b <= 128 ? 2 : (tot_b <= 256 ? 4 : 0);
#define BANK_B(RR) launch_scan_bank<M, DSUB, 0, RR>(g, q, nq, centroids, codebooks, probes, cdist, nprobe, nprobe, 1, \
                                                    list_off, codes, nullptr, nullptr, nullptr, ntotal, k, tot_b, fin, counter, st, rlist, rcount)
  return rb == 2 ? BANK_B(2) : (rb == 4 ? BANK_B(4) : BANK_B(0));
#undef BANK_B
}

// L2 search with residual tables, list-major (see ivfpq_scan_listmajor_kernel), in three parts
// (0, 1, 2: see launch_listmajor_t).  `first`: nq * k keys; `lm`: ivfpq_listmajor_bytes().
// Returns -1 where the shape or the LDS does not fit (then from part 0 on: nothing was launched).
int launch_ivfpq_scan_listmajor(int part, const IvfpqDims& g, const float* q, int64_t nq, const float* centroids,
                                const float* codebooks, const int32_t* probes, const float* cdist, int nprobe,
                                int p_first, int cap, const int64_t* list_off, const uint8_t* codes,
                                int64_t ntotal, int k, u64* first, u64* counter, char* lm, const int64_t* ids,
                                float* out_dist, int64_t* out_ids, hipStream_t st) {
  if (nq <= 0) return 0;
  if (!ivfpq_listmajor_shape(g) || p_first < 1 || p_first >= nprobe) return -1;
#define LMGO(MM, DS)                                                                                      \
  if (g.M == MM && g.dsub == DS)                                                                          \
    return launch_listmajor_t<MM, DS>(part, g, q, nq, centroids, codebooks, probes, cdist, nprobe, p_first, cap, \
                                      list_off, codes, ntotal, k, first, counter, lm, ids, out_dist, out_ids, st)
  LMGO(32, 3);
  LMGO(16, 8);
  LMGO(8, 4);
#undef LMGO
  return -1;
}
// where the number of queries scanned again by the last part lies (one u32, device memory)
const unsigned* ivfpq_listmajor_rescan_count(const IvfpqDims& g, int64_t nq, int nprobe, int cap, const char* lm) {
  return reinterpret_cast<const unsigned*>(lm + lm_layout(nq, nprobe, g.nlist, cap).o_rcount);
}

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
