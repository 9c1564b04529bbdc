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

// ---- wavefront-level k-selection ------------------------------------------
// One wavefront keeps the k smallest keys of a stream (App. A.4: k-selection
// is the critical GPU stage; Sec. 3.2: for larger k use an unordered reservoir
// that is trimmed back to k when it overflows).  State: TOT 64-bit slots in
// LDS owned by the wavefront.  Slots [0, k) hold the best k seen so far,
// ascending after every trim; slots [k, TOT) are the reservoir.  A candidate
// enters the reservoir only if it beats the current k-th best (`thresh`), so
// once the threshold has tightened almost every candidate costs one compare.
// When the reservoir cannot take another full wavefront of candidates, all
// TOT slots are sorted with a bitonic network and the reservoir is emptied.
// TOT is a power of two >= k + 64.
struct WaveSelect {
  volatile u64* s;       // this wavefront's TOT slots
  volatile u64* shared;  // optional: a bound shared by the wavefronts of a workgroup (LDS), or null
  int tot, k, cnt;       // cnt: reservoir fill (wave-uniform)
  u64 thresh;            // k-th best key this wavefront holds (wave-uniform)

  __device__ __forceinline__ void init(u64* slots, int tot_, int k_, u64* shared_ = nullptr) {
    s = slots; shared = shared_; tot = tot_; k = k_; cnt = 0; thresh = KEY_EMPTY;
    for (int i = lane_id(); i < tot; i += VS_WAVE) s[i] = KEY_EMPTY;
    wave_lds_sync();
  }

  __device__ __forceinline__ void sort_all() {
    const int lane = lane_id();
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

  // Sorts everything, keeps the best k, empties the reservoir.
  __device__ __forceinline__ void trim() {
    for (int i = k + cnt + lane_id(); i < tot; i += VS_WAVE) s[i] = KEY_EMPTY;
    wave_lds_sync();
    sort_all();
    cnt = 0;
    thresh = s[k - 1];
    // The k-th best key of ANY subset bounds the k-th best of the whole: publish it so
    // that sibling wavefronts reject candidates that cannot make the workgroup's top k.
    if (shared && lane_id() == 0 && thresh != KEY_EMPTY)
      atomicMin(const_cast<u64*>(shared), thresh);
  }

  // Every lane of the wavefront must call this together.  use_shared: also
  // reject against the workgroup bound.  It must be false when re-inserting
  // keys that other wavefronts already hold (one of them IS the bound).
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

  // After finish(), slots [0, k) hold the k best keys in ascending order.
  __device__ __forceinline__ void finish() {
    wave_lds_sync();
    trim();
  }
};

// Total slots a wavefront needs for a given k.
static inline int select_slots_for_k(int k) {
  int tot = 128;
  while (tot < k + 64) tot <<= 1;
  return tot;
}
