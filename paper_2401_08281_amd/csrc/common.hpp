// Device-side helpers shared by the gfx950 kernels: ordered keys and the
// wavefront-level k-selection.  gfx950 only: wavefronts are 64 lanes wide.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef unsigned long long u64;
typedef unsigned int u32;

#define VS_WAVE 64
#define KEY_EMPTY 0xFFFFFFFFFFFFFFFFull

// ---- ordered keys ----------------------------------------------------------
// A candidate is one 64-bit key: (order-preserving image of the fp32 value)
// in the high word, a 32-bit index in the low word.  A smaller key is a
// better candidate under both metrics (for the inner product the value word
// is complemented), and among equal values the smaller index wins, which
// makes every selection below deterministic.

__device__ __forceinline__ u32 order_f32(float f) {
  u32 u = __float_as_uint(f);
  return u ^ ((u >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}
__device__ __forceinline__ float unorder_f32(u32 o) {
  u32 u = (o & 0x80000000u) ? (o ^ 0x80000000u) : ~o;
  return __uint_as_float(u);
}
__device__ __forceinline__ u64 make_key(float v, u32 idx, int metric) {
  u32 o = order_f32(v);
  if (metric) o = ~o;
  return ((u64)o << 32) | (u64)idx;
}
__device__ __forceinline__ float key_value(u64 key, int metric) {
  u32 o = (u32)(key >> 32);
  if (metric) o = ~o;
  return unorder_f32(o);
}
__device__ __forceinline__ u32 key_index(u64 key) { return (u32)(key & 0xFFFFFFFFull); }

__device__ __forceinline__ int lane_id() { return threadIdx.x & (VS_WAVE - 1); }

// Orders the LDS traffic of one wavefront: earlier LDS writes of any lane are
// visible to later LDS reads of any lane of the same wavefront.
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Workgroup barrier that orders LDS traffic only.  Unlike __syncthreads() it
// does not wait for outstanding global loads or stores, so prefetches that
// were issued before the barrier stay in flight across it.  Use it where the
// data exchanged between wavefronts lives in LDS.
__device__ __forceinline__ void block_sync_lds() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Waits until every global load issued so far by this wavefront has returned.  Placed
// after a prologue that fills long-lived registers (codebooks, MFMA operand fragments), it
// lets the loop that follows keep its own prefetches in flight: without it the compiler has
// to assume, at every use of those registers inside the loop, that the prologue's loads may
// still be pending, and waits for everything -- the loop's prefetches included.
__device__ __forceinline__ void wait_all_global_loads() {
  __builtin_amdgcn_s_waitcnt(0x0F70);   // gfx9 encoding: vmcnt(0), expcnt and lgkmcnt unconstrained
}

// ---- cross-lane exchange and register-resident bitonic sort ------------------
// lane i receives the value held by lane i ^ X.  X = 1, 2, 4, 8 stay inside a
// row of 16 lanes and use DPP modifiers (no LDS traffic); 16 and 32 cross rows
// and go through ds_bpermute.
template <int X>
__device__ __forceinline__ u32 lane_xor_u32(u32 v) {
  const int s = (int)v;
  if constexpr (X == 1) {
    return (u32)__builtin_amdgcn_update_dpp(0, s, 0xB1, 0xF, 0xF, false);   // quad_perm [1,0,3,2]
  } else if constexpr (X == 2) {
    return (u32)__builtin_amdgcn_update_dpp(0, s, 0x4E, 0xF, 0xF, false);   // quad_perm [2,3,0,1]
  } else if constexpr (X == 4) {
    // lanes with bit 2 clear (banks 0, 2 of each row) read lane + 4, the others lane - 4
    int r = __builtin_amdgcn_update_dpp(0, s, 0x104, 0xF, 0x5, false);      // row_shl:4
    r = __builtin_amdgcn_update_dpp(r, s, 0x114, 0xF, 0xA, false);          // row_shr:4
    return (u32)r;
  } else if constexpr (X == 8) {
    return (u32)__builtin_amdgcn_update_dpp(0, s, 0x128, 0xF, 0xF, false);  // row_ror:8
  } else {
    return (u32)__shfl_xor(s, X);
  }
}
template <int X>
__device__ __forceinline__ u64 lane_xor(u64 v) {
  const u32 lo = lane_xor_u32<X>((u32)v), hi = lane_xor_u32<X>((u32)(v >> 32));
  return ((u64)hi << 32) | lo;
}
template <int X>
__device__ __forceinline__ u32 lane_xor(u32 v) { return lane_xor_u32<X>(v); }

// One compare-exchange step of the bitonic network at lane distance X for
// element index e (ascending block when (e & size) == 0).
template <int X, typename T>
__device__ __forceinline__ T bitonic_lane_step(T v, int e, int stride, int size) {
  const T o = lane_xor<X>(v);
  const bool keep_min = ((e & stride) == 0) == ((e & size) == 0);
  const T lo = v < o ? v : o, hi = v < o ? o : v;
  return keep_min ? lo : hi;
}

// Sorts the 64 * R keys (u32 or u64) held by one wavefront, ascending in element order
// e = lane * R + r.  Strides below R are register-to-register; the rest cross lanes.
template <int R, typename T>
__device__ __forceinline__ void wave_sort_regs(T (&v)[R]) {
  const int lane = lane_id();
#pragma unroll
  for (int size = 2; size <= 64 * R; size <<= 1) {
#pragma unroll
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      if (stride >= R) {
        const int X = stride / R;
#pragma unroll
        for (int r = 0; r < R; ++r) {
          const int e = lane * R + r;
          switch (X) {
            case 1: v[r] = bitonic_lane_step<1>(v[r], e, stride, size); break;
            case 2: v[r] = bitonic_lane_step<2>(v[r], e, stride, size); break;
            case 4: v[r] = bitonic_lane_step<4>(v[r], e, stride, size); break;
            case 8: v[r] = bitonic_lane_step<8>(v[r], e, stride, size); break;
            case 16: v[r] = bitonic_lane_step<16>(v[r], e, stride, size); break;
            default: v[r] = bitonic_lane_step<32>(v[r], e, stride, size); break;
          }
        }
      } else {
#pragma unroll
        for (int r = 0; r < R; ++r) {
          if ((r & stride) == 0) {
            const int e = lane * R + r;
            const bool up = (e & size) == 0;
            const T a = v[r], b = v[r | stride];
            const bool sw = (a > b) == up;
            v[r] = sw ? b : a;
            v[r | stride] = sw ? a : b;
          }
        }
      }
    }
  }
}

// ---- wavefront-level k-selection ------------------------------------------
// One wavefront keeps the k smallest keys of a stream (App. A.3 "GPU Faiss": k-selection
// is the critical GPU stage; Sec. 3.1: for larger k use an unordered reservoir
// that is trimmed back to k when it overflows).  State: TOT 64-bit slots in
// LDS owned by the wavefront.  Slots [0, k) hold the best k seen so far,
// ascending after every trim; slots [k, TOT) are the reservoir.  A candidate
// enters the reservoir only if it beats the current k-th best (`thresh`), so
// once the threshold has tightened almost every candidate costs one compare.
// When the reservoir cannot take another full wavefront of candidates, the
// live slots are sorted and the reservoir is emptied.  TOT is a power of two
// >= k + 64.  R > 0: TOT <= 64 * R (any size >= k + 64) and the sort runs in registers (R keys
// per lane, DPP exchanges); R == 0: TOT a power of two, bitonic network through LDS.
// LDS pointers carry their address space in the type, so that every access below is
// a ds_* instruction (not a flat access that has to discover its aperture at run time).
typedef __attribute__((address_space(3))) volatile u64* lds_u64_ptr;
__device__ __forceinline__ lds_u64_ptr to_lds(u64* p) { return (lds_u64_ptr)p; }

template <int R>
struct WaveSelect {
  lds_u64_ptr s;         // this wavefront's TOT slots
  lds_u64_ptr shared;    // optional: a bound shared by the wavefronts of a workgroup, or null
  bool has_shared;
  int tot, k, cnt;       // cnt: reservoir fill (wave-uniform)
  u64 thresh;            // k-th best key this wavefront holds (wave-uniform)
  u64 seen;              // the workgroup bound as last read by refresh_shared() (wave-uniform)
  u64 bound;             // min(thresh, seen): what push_cached() and push_value() test against
  float bound_f;         // the value in `bound`, in a scalar register (NaN while nothing bounds)
  int metric;            // how push_value() orders values: 0 smaller is better, 1 larger is better

  // attach to existing state (slots hold k sorted keys plus cnt_ reservoir entries)
  __device__ __forceinline__ void attach(u64* slots, int tot_, int k_, int cnt_, u64 thresh_) {
    s = to_lds(slots); shared = (lds_u64_ptr)0; has_shared = false;
    tot = tot_; k = k_; cnt = cnt_; thresh = thresh_; seen = KEY_EMPTY; metric = 0;
    rebound();
  }

  __device__ __forceinline__ void init(u64* slots, int tot_, int k_, u64* shared_ = nullptr) {
    s = to_lds(slots); has_shared = shared_ != nullptr;
    shared = has_shared ? to_lds(shared_) : (lds_u64_ptr)0;
    tot = tot_; k = k_; cnt = 0; thresh = KEY_EMPTY; seen = KEY_EMPTY; metric = 0;
    rebound();
    for (int i = lane_id(); i < k; i += VS_WAVE) s[i] = KEY_EMPTY;
    wave_lds_sync();
  }
  // values are ordered as make_key(v, i, metric_) orders them (call right after init / attach)
  __device__ __forceinline__ void set_metric(int metric_) { metric = metric_; rebound(); }
  // bound and bound_f follow thresh and seen.  The value of the all-ones key is a NaN under both
  // metrics, and no value compares greater or smaller than a NaN: nothing is rejected by it.
  __device__ __forceinline__ void rebound() {
    bound = seen < thresh ? seen : thresh;
    bound_f = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(
                                            __builtin_bit_cast(int, key_value(bound, metric))));
  }

  __device__ __forceinline__ void sort_lds() {
    const int lane = lane_id();
    for (int i = k + cnt + lane; i < tot; i += VS_WAVE) s[i] = KEY_EMPTY;
    wave_lds_sync();
    for (int size = 2; size <= tot; size <<= 1) {
      for (int stride = size >> 1; stride > 0; stride >>= 1) {
        for (int i = lane; i < (tot >> 1); i += VS_WAVE) {
          int lo = ((i & ~(stride - 1)) << 1) | (i & (stride - 1));
          int hi = lo + stride;
          bool up = (lo & size) == 0;
          u64 a = s[lo], b = s[hi];
          if ((a > b) == up) { s[lo] = b; s[hi] = a; }
        }
        wave_lds_sync();
      }
    }
  }

  __device__ __forceinline__ void sort_regs() {
    // live slots are [0, k + cnt); the rest count as empty
    const int lane = lane_id(), live = k + cnt;
    wave_lds_sync();   // reservoir writes of this wavefront are visible to all its lanes
    u64 v[R > 0 ? R : 1];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int e = lane * R + r;
      v[r] = e < live ? s[e] : KEY_EMPTY;
    }
    wave_sort_regs(v);
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int e = lane * R + r;
      if (e < k) s[e] = v[r];
    }
    wave_lds_sync();
  }

  // Sorts the live slots, keeps the best k, empties the reservoir.
  __device__ __forceinline__ void trim() {
    if constexpr (R > 0) sort_regs(); else sort_lds();
    cnt = 0;
    thresh = s[k - 1];
    rebound();
    // The k-th best key of ANY subset bounds the k-th best of the whole: publish it so
    // that sibling wavefronts reject candidates that cannot make the workgroup's top k.
    if (has_shared && lane_id() == 0 && thresh != KEY_EMPTY)
      __hip_atomic_fetch_min((__attribute__((address_space(3))) u64*)shared, thresh,
                             __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  }

  // Every lane of the wavefront must call this together.  use_shared: also
  // reject against the workgroup bound.
  __device__ __forceinline__ void push(bool valid, u64 key, bool use_shared = false) {
    u64 th = thresh;
    if (use_shared) { const u64 sh = *shared; th = sh < th ? sh : th; }
    bool pass = valid && key < th;
    u64 mask = __ballot(pass);
    if (mask == 0) return;
    int pos = k + cnt + __popcll(mask & ((1ull << lane_id()) - 1ull));
    if (pass) s[pos] = key;
    cnt += __popcll(mask);
    if (k + cnt + VS_WAVE > tot) trim();
  }

  // The same with the workgroup bound taken from the copy that refresh_shared() made: a bound only
  // ever tightens, so an old copy is still a valid (weaker) bound, and reading it once per list
  // instead of once per push takes an LDS round trip off every push.
  __device__ __forceinline__ void refresh_shared() {
    if (has_shared) { const u64 sh = *shared; seen = sh < seen ? sh : seen; rebound(); }
  }
  __device__ __forceinline__ void push_cached(bool valid, u64 key) {
    bool pass = valid && key < bound;
    u64 mask = __ballot(pass);
    if (mask == 0) return;
    int pos = k + cnt + __popcll(mask & ((1ull << lane_id()) - 1ull));
    if (pass) s[pos] = key;
    cnt += __popcll(mask);
    if (k + cnt + VS_WAVE > tot) { trim(); refresh_shared(); }
  }
  // push_cached(valid, make_key(v, idx, metric)) with a cheaper way out for the usual case that no
  // lane holds a candidate: a key below the bound has a value that is not worse than the bound's,
  // so one float compare against a scalar rejects a whole wavefront before any key is formed.
  __device__ __forceinline__ void push_value(bool valid, float v, u32 idx) {
    const bool maybe = valid && (metric ? !(v < bound_f) : !(v > bound_f));
    if (__ballot(maybe) == 0) return;
    push_cached(valid, make_key(v, idx, metric));
  }

  // After finish(), slots [0, k) hold the k best keys in ascending order.
  __device__ __forceinline__ void finish() {
    if (cnt > 0) trim();
    wave_lds_sync();
  }
};

// Total slots a wavefront needs for a given k, and the register-sort width
// (keys per lane) that goes with it: 0 = sort through LDS.
static inline int select_slots_for_k(int k) {
  int tot = 128;
  while (tot < k + 64) tot <<= 1;
  return tot;
}
static inline int select_regs_for_slots(int tot) { return tot <= 256 ? tot / 64 : 0; }

// four 32-bit words as one register tuple (HIP's own uint4 / float4 arrays are placed in
// scratch memory by the compiler; an ext-vector type stays in registers)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// ---- inverted-list storage ------------------------------------------------------
// list that owns storage position p: the l with off[l] <= p < off[l+1]
__device__ __forceinline__ int list_of_position(const int64_t* __restrict__ off, int nlist,
                                                int64_t p) {
  int lo = 0, hi = nlist;  // invariant: off[lo] <= p < off[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (off[mid] <= p) lo = mid; else hi = mid;
  }
  return lo;
}

// ---- canon distance of one pair ------------------------------------------------
// The fp32 chain every exact decision of the library is defined in: dimension order,
// diff = a - b rounded, acc = fma(diff, diff, acc) (inner product: acc = fma(a, b, acc)).
// qs may live in LDS (read as broadcasts); b is a row in global memory; vec: d % 4 == 0.
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

// The same value for 64 rows at once, one per lane of a wavefront, with memory read in runs of
// 128 bytes (d a multiple of 32): per chunk of 32 dimensions eight lanes fetch the 128 bytes
// of one row (8 rows per load instruction), the chunk goes through a wavefront-private LDS
// tile (row stride 36 floats: aligned, conflict-free) and lane r continues the chain of row
// `row` of lane r in dimension order; the next chunk is in flight in registers meanwhile.
// row: any valid row of B in every lane (lanes without a row pass 0 and drop the result).
// ids_s: 64 int64 and tile: 64 * 36 floats of LDS owned by this wavefront.
template <int METRIC>
__device__ __forceinline__ float wave_canon_rows_tiled(const float* __restrict__ qs,
                                                       const float* __restrict__ B, int d, int64_t row,
                                                       int64_t* __restrict__ ids_s,
                                                       float* __restrict__ tile) {
  constexpr int DC = 32, LD = 36;
  const int lane = lane_id(), r_ld = lane >> 3, c_ld = lane & 7;
  wave_lds_sync();                                   // earlier users of ids_s and the tile are done
  ids_s[lane] = row;
  wave_lds_sync();
  const float* rp[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) rp[i] = B + ids_s[r_ld + 8 * i] * d + c_ld * 4;
  u32x4 stg[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) stg[i] = *reinterpret_cast<const u32x4*>(rp[i]);
  float acc = 0.f;
  const int nch = d / DC;
  for (int ch = 0; ch < nch; ++ch) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
      *reinterpret_cast<u32x4*>(tile + (r_ld + 8 * i) * LD + c_ld * 4) = stg[i];
    wave_lds_sync();
    if (ch + 1 < nch) {
#pragma unroll
      for (int i = 0; i < 8; ++i) stg[i] = *reinterpret_cast<const u32x4*>(rp[i] + (ch + 1) * DC);
    }
    const float* __restrict__ tr = tile + lane * LD;
    const float* __restrict__ qc = qs + ch * DC;
#pragma unroll
    for (int cc = 0; cc < DC / 4; ++cc) {
      const float4 xv = *reinterpret_cast<const float4*>(tr + cc * 4);
      const float4 qv = *reinterpret_cast<const float4*>(qc + cc * 4);
      const float xs[4] = {xv.x, xv.y, xv.z, xv.w}, qq[4] = {qv.x, qv.y, qv.z, qv.w};
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (METRIC == 0) { const float diff = qq[u] - xs[u]; acc = __builtin_fmaf(diff, diff, acc); }
        else acc = __builtin_fmaf(qq[u], xs[u], acc);
      }
    }
    wave_lds_sync();                                 // the tile is free for the next chunk
  }
  return acc;
}

// ---- merge of sorted key lists by ranking -----------------------------------
// `nl` ascending lists of k keys each (padded with KEY_EMPTY) sit at
// base + w * stride.  Keys are unique, so the number of keys smaller than x over
// all lists is x's position in the merged order; every key whose rank is below
// k goes straight to out[rank].  All lanes of the workgroup take part; no
// sorting.  out must not alias the lists.
__device__ __forceinline__ int count_less(const u64* __restrict__ L, int k, u64 x) {
  if (k <= 16) {
    int c = 0;
    for (int j = 0; j < k; ++j) c += L[j] < x ? 1 : 0;
    return c;
  }
  int lo = 0, hi = k;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (L[mid] < x) lo = mid + 1; else hi = mid;
  }
  return lo;
}

// Where selected keys go: raw keys (to be merged again later) and / or final
// results (value, 64-bit id through an optional id map, 32-bit index).  Null
// members are skipped.  Empty slots become id -1 and value +inf (L2) / -inf (IP).
struct KeySink {
  u64* keys;
  float* val;
  int64_t* id64;
  int32_t* idx32;
  const int64_t* idmap;
  int metric;
  __device__ __forceinline__ void put(int64_t at, u64 key) const {
    if (keys) keys[at] = key;
    const bool empty = key == KEY_EMPTY;
    if (val) val[at] = empty ? (metric ? -__builtin_inff() : __builtin_inff()) : key_value(key, metric);
    if (id64) id64[at] = empty ? -1 : (idmap ? idmap[key_index(key)] : (int64_t)key_index(key));
    if (idx32) idx32[at] = empty ? -1 : (int32_t)key_index(key);
  }
};

// Call after a workgroup barrier (the lists are read as ordinary, stable memory).
// Output slot of rank r is sink[at0 + r].
__device__ __forceinline__ void block_rank_merge(const u64* __restrict__ base, int stride, int nl,
                                                 int k, const KeySink& sink, int64_t at0) {
  const int nthreads = blockDim.x;
  for (int c = threadIdx.x; c < nl * k; c += nthreads) {
    const int w = c / k, j = c - w * k;
    const u64 x = base[w * stride + j];
    if (x == KEY_EMPTY) continue;
    int rank = j;
    for (int w2 = 0; w2 < nl; ++w2)
      if (w2 != w) rank += count_less(base + w2 * stride, k, x);
    if (rank < k) sink.put(at0 + rank, x);
  }
  if (threadIdx.x < k) {   // pad the ranks that no real key fills
    int total = 0;
    for (int w = 0; w < nl; ++w) total += count_less(base + w * stride, k, KEY_EMPTY);
    for (int r = total + threadIdx.x; r < k; r += nthreads) sink.put(at0 + r, KEY_EMPTY);
  }
}
