// Host runtime and C ABI of libvs (see include/vs.h for the contract).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/vs.h"
#include "internal.hpp"

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

#define HIP_TRY(expr)                                                                     \
  do {                                                                                    \
    hipError_t e_ = (expr);                                                               \
    if (e_ != hipSuccess)                                                                 \
      return fail(e_ == hipErrorOutOfMemory ? VS_ERR_OOM : VS_ERR_DEVICE, "%s: %s", #expr, \
                  hipGetErrorString(e_));                                                 \
  } while (0)

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

// Grow-only device scratch buffer, with what it takes to hand it from one user to the next:
// a mutex for the host side and an event recorded behind the last user's launches.
struct Scratch {
  void* p = nullptr;
  size_t bytes = 0;
  std::mutex mu;
  hipEvent_t done = nullptr;     // recorded behind the last launches that use the buffer
  hipStream_t last = nullptr;    // ... on this stream
  int reserve(size_t need) {
    if (need <= bytes) return VS_OK;
    if (p) { HIP_TRY(hipFree(p)); p = nullptr; bytes = 0; }   // (hipFree waits for the device)
    HIP_TRY(hipMalloc(&p, need));
    bytes = need;
    return VS_OK;
  }
  void release() {
    if (p) (void)hipFree(p);
    p = nullptr; bytes = 0;
    if (done) (void)hipEventDestroy(done);
    done = nullptr; last = nullptr;
  }
};

// One user of a scratch buffer at a time, also on the device: holds the mutex while a call
// enqueues its work, makes a call on ANOTHER stream wait for the event that the previous user
// recorded behind its last launch, and records its own when it leaves.  (Calls on one stream are
// ordered by the stream.  A stream under graph capture neither waits nor records: a captured call
// must not be mixed with calls on other streams that use the same buffer.)
struct ScratchUse {
  Scratch& sc;
  std::unique_lock<std::mutex> lock;
  hipStream_t st;
  bool live;
  ScratchUse(Scratch& sc_, hipStream_t st_) : sc(sc_), lock(sc_.mu), st(st_), live(true) {
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cs) != hipSuccess || cs != hipStreamCaptureStatusNone) { live = false; return; }
    if (sc.done && sc.last != st) (void)hipStreamWaitEvent(st, sc.done, 0);
  }
  ~ScratchUse() {
    if (!live) return;
    if (!sc.done && hipEventCreateWithFlags(&sc.done, hipEventDisableTiming) != hipSuccess) {
      sc.done = nullptr;
      return;
    }
    if (hipEventRecord(sc.done, st) == hipSuccess) sc.last = st;
  }
};

// Carves aligned sub-buffers out of one allocation.
struct Carver {
  size_t off = 0;
  size_t take(size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; }
};

// The file-scope device array behind vs_ivfpq_search_static.  Its name is a host-side stand-in,
// not a device address: host code uses the per-device pointer that hipGetSymbolAddress returns
// (every GPU holds its own copy of the array at its own address).
constexpr size_t kStaticScratchBytes = VS_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
std::mutex g_static_mu;
void* g_static_ptr[16] = {nullptr};

// Address of the current device's copy of `scratch` (looked up once per device, with that device
// current); null + error on failure.
int static_scratch(char** out) {
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= 16) return fail(VS_ERR_UNSUPPORTED, "static scratch: device %d", dev);
  std::lock_guard<std::mutex> lock(g_static_mu);
  if (!g_static_ptr[dev]) {
    void* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr)
      return fail(VS_ERR_DEVICE, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
    g_static_ptr[dev] = ptr;
  }
  *out = static_cast<char*>(g_static_ptr[dev]);
  return VS_OK;
}

// scratch of vs_flat_search, vs_flat_index_search, vs_kmeans and vs_ivfpq_train, one per device
Scratch g_flat_scratch[16];

// ---- optional stage timing ---------------------------------------------------
struct ProfRec { int stage; hipEvent_t a, b; };
std::mutex g_prof_mu;
std::vector<ProfRec> g_prof;
bool g_prof_on = false;

// Brackets the launches made inside its scope with two events on the stream.
struct StageTimer {
  int stage; hipStream_t st; hipEvent_t a = nullptr, b = nullptr; bool on;
  StageTimer(int stage_, hipStream_t st_) : stage(stage_), st(st_), on(g_prof_on && stage_ >= 0) {
    if (!on) return;
    if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) { on = false; return; }
    (void)hipEventRecord(a, st);
  }
  ~StageTimer() {
    if (!on) return;
    (void)hipEventRecord(b, st);
    std::lock_guard<std::mutex> lock(g_prof_mu);
    g_prof.push_back({stage, a, b});
  }
};

// Budget for a materialised distance tile: small enough to live in the
// 256 MB last-level cache between the kernel that writes it and the
// selection kernel that reads it back.
constexpr size_t kTileBytes = 128ull << 20;

// ---- run-time options (vs_set_option) -----------------------------------------
std::atomic<int> g_knn_path{0};          // 0 auto, 1 canon tiles only, 2 MFMA shortlist whenever supported
// List-major IVF-PQ scan: 0 where it pays (large batch, long code store), 1 wherever the shape
// allows it, -1 never; and its two sizes: probes scanned query-major first, candidates per query.
std::atomic<int> g_list_major{0};
std::atomic<int> g_lm_first{4};
std::atomic<int> g_lm_cap{1024};
std::atomic<float> g_knn_eps_scale{1.f}; // multiplies the error bound of the MFMA shortlist test
std::atomic<long long> g_knn_mfma_rows{0};

void tile_shape(int64_t na, int64_t nb, int64_t* rows, int64_t* cols) {
  int64_t c = std::min<int64_t>(nb, 16384);
  c = (c + 63) / 64 * 64;
  int64_t r = (int64_t)(kTileBytes / sizeof(float)) / c;
  r = std::max<int64_t>(64, r / 64 * 64);
  r = std::min(r, (na + 63) / 64 * 64);
  *rows = r;
  *cols = c;
}

// Device buffers of one prepared MFMA operand, carved from scratch or owned by an index.
struct Planes {
  unsigned short* hi = nullptr;
  unsigned short* lo = nullptr;
  unsigned short* h16 = nullptr;   // fp16 heads, at lo + (padded rows) * d
  float* norm = nullptr;
  PrepInfo* info = nullptr;
  int known_bf16 = -1;          // info->all_bf16 once the host has read it back, else -1
  bool try_heads_only = false;  // prepared with PrepInfo::heads_only set (an index's own operand)
};
size_t planes_bytes(int64_t n, int d) {
  n = mfma_padded_rows(n);
  return align_up((size_t)n * d * sizeof(unsigned short)) + align_up((size_t)2 * n * d * sizeof(unsigned short)) +
         align_up((size_t)n * sizeof(float)) + align_up(sizeof(PrepInfo));
}
Planes carve_planes(char* base, int64_t n, int d) {
  Planes p;
  n = mfma_padded_rows(n);
  size_t o = 0;
  p.hi = reinterpret_cast<unsigned short*>(base + o); o += align_up((size_t)n * d * sizeof(unsigned short));
  // (operand preparation writes the fp16 heads right behind the bf16 tails: one block of two planes)
  p.lo = reinterpret_cast<unsigned short*>(base + o); o += align_up((size_t)2 * n * d * sizeof(unsigned short));
  p.h16 = p.lo + (size_t)n * d;
  p.norm = reinterpret_cast<float*>(base + o); o += align_up((size_t)n * sizeof(float));
  p.info = reinterpret_cast<PrepInfo*>(base + o);
  return p;
}
MfmaOperand operand(const float* x, int64_t n, const Planes& p) {
  MfmaOperand m;
  m.x = x; m.hi = p.hi; m.lo = p.lo; m.h16 = p.h16; m.norm = p.norm; m.info = p.info; m.n = n;
  m.known_bf16 = p.known_bf16;
  m.try_heads_only = p.try_heads_only;
  return m;
}
// After the preparation of an index's own operand has completed: tell the host whether the
// rows are exactly bf16, so that searches enqueue only the sweep variant that will run.
hipError_t learn_planes(Planes* p) {
  PrepInfo h;
  const hipError_t e = hipMemcpy(&h, p->info, sizeof(PrepInfo), hipMemcpyDeviceToHost);
  if (e == hipSuccess) p->known_bf16 = h.all_bf16 ? 1 : 0;
  return e;
}

// Exact k best rows of B for every row of A (canon values, ties to the smaller index),
// written best first to `out`.  Two routes with identical results:
//   canon tiles:    canon_matrix + row_select over (row tile, column tile) pairs;
//   MFMA shortlist: bf16 matrix-core contraction -> kp candidates per row -> canon re-rank,
//                   with a per-row sufficiency test and an exact fallback.
struct KnnPlan {
  bool mfma = false;
  int nsplit = 1;
  int64_t rows = 0, cols = 0;     // canon tile shape
  size_t bytes = 0;               // scratch needed
};
KnnPlan knn_plan(int64_t na, int64_t nb, int d, int k, bool b_prepared) {
  KnnPlan p;
  const int path = g_knn_path.load();
  p.mfma = path != 1 && nb > 0 && mfma_knn_supported(d, k);
  if (p.mfma) {
    size_t b = planes_bytes(na, d);
    if (!b_prepared) b += planes_bytes(nb, d);
    b += align_up(mfma_knn_shortlist_bytes(na, nb, d, k, &p.nsplit));
    b += align_up(sizeof(int)) + align_up((size_t)na * sizeof(int));
    b += align_up(mfma_knn_fallback_bytes(na, nb, k));
    p.bytes = b;
  } else {
    tile_shape(na, std::max<int64_t>(nb, 1), &p.rows, &p.cols);
    p.bytes = align_up((size_t)p.rows * p.cols * sizeof(float)) + align_up((size_t)na * k * sizeof(u64));
  }
  return p;
}

// Plan for n rows of A processed in pieces of at most `piece` rows: the work space covers the
// full pieces and the shorter last one (a shorter piece may be laid out with more splits of B,
// so its work space is not bounded by that of a longer one).
KnnPlan knn_plan_pieces(int64_t n, int64_t piece, int64_t nb, int d, int k, bool b_prepared) {
  KnnPlan p = knn_plan(std::min(n, piece), nb, d, k, b_prepared);
  if (n > piece && n % piece != 0) {
    const KnnPlan last = knn_plan(n % piece, nb, d, k, b_prepared);
    p.bytes = std::max(p.bytes, last.bytes);
  }
  return p;
}

// `plan` must come from knn_plan / knn_plan_pieces for these shapes: a work space smaller than
// what na rows need is refused here, before any kernel is launched on it.
int knn_run(const KnnPlan& plan, char* ws, const float* A, int64_t na, const float* B, int64_t nb,
            int d, int metric, int k, const Planes* b_planes, const SelectOut& out, hipStream_t st,
            int stage_dist, int stage_select, const int** fallback_count = nullptr) {
  // fallback_count: receives the device address of this call's count of rows that took the exact
  // fallback (valid once the call's kernels have run), or null when the canon tiles served the call
  if (fallback_count) *fallback_count = nullptr;
  {
    const KnnPlan need = knn_plan(na, nb, d, k, b_planes != nullptr);
    if (need.mfma != plan.mfma || (plan.mfma && need.bytes > plan.bytes))
      return fail(VS_ERR_DEVICE, "k-nearest-rows: work space of %zu bytes planned, %zu needed for %lld rows",
                  plan.bytes, need.bytes, (long long)na);
  }
  if (plan.mfma) {
    size_t o = 0;
    Planes pa = carve_planes(ws + o, na, d); o += planes_bytes(na, d);
    Planes pb;
    if (b_planes) pb = *b_planes;
    else { pb = carve_planes(ws + o, nb, d); o += planes_bytes(nb, d); }
    int ns = 1;
    const size_t sl = align_up(mfma_knn_shortlist_bytes(na, nb, d, k, &ns));
    u64* shortlist = reinterpret_cast<u64*>(ws + o); o += sl;
    int* fb_count = reinterpret_cast<int*>(ws + o); o += align_up(sizeof(int));
    int* fb_rows = reinterpret_cast<int*>(ws + o); o += align_up((size_t)na * sizeof(int));
    u64* fb_partial = reinterpret_cast<u64*>(ws + o);
    const MfmaOperand oa = operand(A, na, pa), ob = operand(B, nb, pb);
    {
      StageTimer t(stage_dist, st);
      launch_prep(A, na, d, pa.hi, pa.lo, pa.norm, pa.info, st);
      if (!b_planes) launch_prep(B, nb, d, pb.hi, pb.lo, pb.norm, pb.info, st);
      launch_mfma_shortlist(oa, ob, d, metric, k, plan.nsplit, shortlist, fb_count, st);
    }
    {
      StageTimer t(stage_select, st);
      launch_rerank(oa, ob, d, metric, k, plan.nsplit, shortlist, g_knn_eps_scale.load(), out,
                    fb_count, fb_rows, fb_partial, st);
    }
    g_knn_mfma_rows += na;
    if (fallback_count) *fallback_count = fb_count;
    return VS_OK;
  }
  float* mat = reinterpret_cast<float*>(ws);
  u64* keys = reinterpret_cast<u64*>(ws + align_up((size_t)plan.rows * plan.cols * sizeof(float)));
  for (int64_t a0 = 0; a0 < na; a0 += plan.rows) {
    const int64_t ra = std::min(plan.rows, na - a0);
    SelectOut o;
    o.val = out.val ? out.val + a0 * k : nullptr;
    o.id64 = out.id64 ? out.id64 + a0 * k : nullptr;
    o.idx32 = out.idx32 ? out.idx32 + a0 * k : nullptr;
    for (int64_t b0 = 0; b0 < nb; b0 += plan.cols) {
      const int64_t cb = std::min(plan.cols, nb - b0);
      {
        StageTimer t(stage_dist, st);
        launch_canon_matrix(A + a0 * d, ra, B + b0 * d, cb, d, metric, mat, plan.cols, st);
      }
      {
        StageTimer t(stage_select, st);
        launch_row_select(mat, plan.cols, ra, cb, (u32)b0, metric, k, keys + a0 * k, b0 == 0,
                          b0 + cb >= nb, o, st);
      }
    }
  }
  return VS_OK;
}

}  // namespace

struct vs_ivfpq {
  IvfpqDims g{};
  int device = 0;
  float* centroids = nullptr;   // [nlist, d]
  float* codebooks = nullptr;   // [M, K, dsub]
  int64_t ntotal = 0;
  uint8_t* codes = nullptr;     // [ntotal, code_size], list-contiguous
  int64_t* ids = nullptr;       // [ntotal]
  float* norms = nullptr;       // [ntotal] squared norms of the decoded vectors, search_type 1 only
  float* cnorm = nullptr;       // [nlist] squared norms of the centroids (IVF-PQ only)
  float* list_tables = nullptr; // [nlist, K, M] per-list terms of the split tables (search type 2, once computed)
  int search_type = VS_ST_RESIDUAL_TABLES;
  int64_t* list_off = nullptr;  // device [nlist + 1]
  std::vector<int64_t> h_off;   // host copy
  void* plane_mem = nullptr;    // bf16 head/tail planes + norms of the centroids (MFMA route)
  Planes c_planes;
  bool has_planes = false;
  bool assign_probed = false;   // an add has run its assignment through the matrix-core route
  int coarse_metric = -1;       // metric of list assignment and probing; -1: the index metric (g.metric)
  mutable Scratch scratch;
};

// IVF-Flat shares the lists, the coarse quantizer and the bookkeeping of the IVF-PQ index
struct vs_ivfflat {
  vs_ivfpq core;
};

// Flat index: the rows as given, plus the prepared operand of the matrix-core route
struct vs_flat {
  int d = 0, metric = 0, device = 0;
  int64_t ntotal = 0, cap = 0;  // rows stored / rows the buffers hold
  float* x = nullptr;           // [cap, d]
  void* plane_mem = nullptr;    // planes_bytes(cap, d), laid out for ntotal rows
  Planes planes;
  bool has_planes = false;
};

inline int coarse_metric_of(const vs_ivfpq* ix) { return ix->coarse_metric < 0 ? ix->g.metric : ix->coarse_metric; }

// IVF-SQ8 likewise; core.codes holds d bytes per vector (core.g: M = d, nbits = 8)
struct vs_ivfsq8 {
  vs_ivfpq core;
  float* vmin = nullptr;   // [d] first cell's lower end per component
  float* step = nullptr;   // [d] cell width per component
};

extern "C" {

const char* vs_last_error(void) { return g_err; }

int vs_profile_enable(int on) {
  std::lock_guard<std::mutex> lock(g_prof_mu);
  g_prof_on = on != 0;
  return VS_OK;
}

int vs_profile_read(double* stage_ms, int64_t* launches) {
  if (!stage_ms || !launches) return fail(VS_ERR_INVALID_ARG, "vs_profile_read: null pointer");
  std::lock_guard<std::mutex> lock(g_prof_mu);
  for (int s = 0; s < VS_NUM_STAGES; ++s) { stage_ms[s] = 0.0; launches[s] = 0; }
  int rc = VS_OK;
  for (const ProfRec& r : g_prof) {
    float ms = 0.f;
    hipError_t e = hipEventSynchronize(r.b);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.a, r.b);
    if (e != hipSuccess) rc = fail(VS_ERR_DEVICE, "vs_profile_read: %s", hipGetErrorString(e));
    else if (r.stage >= 0 && r.stage < VS_NUM_STAGES) { stage_ms[r.stage] += ms; ++launches[r.stage]; }
    (void)hipEventDestroy(r.a);
    (void)hipEventDestroy(r.b);
  }
  g_prof.clear();
  return rc;
}
const char* vs_version(void) { return "vs 0.2 (gfx950)"; }

int vs_set_option(const char* name, double value) {
  if (!name) return fail(VS_ERR_INVALID_ARG, "vs_set_option: name is null");
  if (!strcmp(name, "knn_path")) {
    if (value != 0 && value != 1 && value != 2) return fail(VS_ERR_INVALID_ARG, "vs_set_option: knn_path must be 0, 1 or 2");
    g_knn_path = (int)value;
    return VS_OK;
  }
  if (!strcmp(name, "knn_eps_scale")) { g_knn_eps_scale = (float)value; return VS_OK; }
  if (!strcmp(name, "list_major")) {
    if (value != 0 && value != 1 && value != -1) return fail(VS_ERR_INVALID_ARG, "vs_set_option: list_major must be -1, 0 or 1");
    g_list_major = (int)value;
    return VS_OK;
  }
  if (!strcmp(name, "list_major_first")) {
    if (value < 1 || value > 64) return fail(VS_ERR_INVALID_ARG, "vs_set_option: list_major_first outside [1, 64]");
    g_lm_first = (int)value;
    return VS_OK;
  }
  if (!strcmp(name, "list_major_candidates")) {
    if (value < 64 || value > 65536) return fail(VS_ERR_INVALID_ARG, "vs_set_option: list_major_candidates outside [64, 65536]");
    g_lm_cap = (int)value;
    return VS_OK;
  }
  return fail(VS_ERR_INVALID_ARG, "vs_set_option: unknown option '%s'", name);
}

int64_t vs_knn_workspace_bytes(int64_t na, int64_t nb, int32_t d, int32_t k, int64_t piece,
                               int32_t b_prepared) {
  if (na < 0 || nb < 0 || d < 1 || k < 1) {
    fail(VS_ERR_INVALID_ARG, "vs_knn_workspace_bytes: na = %lld, nb = %lld, d = %d, k = %d", (long long)na,
         (long long)nb, d, k);
    return -1;
  }
  if (na == 0) return 0;
  const KnnPlan p = piece > 0 ? knn_plan_pieces(na, piece, nb, d, k, b_prepared != 0)
                              : knn_plan(na, nb, d, k, b_prepared != 0);
  return (int64_t)p.bytes;
}

int vs_counters_read(int64_t* counters) {
  if (!counters) return fail(VS_ERR_INVALID_ARG, "vs_counters_read: null pointer");
  HIP_TRY(hipDeviceSynchronize());
  unsigned long long fb = 0;
  if (read_fallback_total(&fb) != 0) return fail(VS_ERR_DEVICE, "vs_counters_read: cannot read the device counter");
  counters[0] = g_knn_mfma_rows.exchange(0);
  counters[1] = (int64_t)fb;
  return VS_OK;
}

int vs_flat_search(const float* x, int64_t nb, const float* q, int64_t nq, int32_t d,
                   int32_t metric, int32_t k, float* out_dist, int64_t* out_ids,
                   void* hip_stream) {
  if (nq < 0 || nb < 0) return fail(VS_ERR_INVALID_ARG, "vs_flat_search: negative size");
  if (d < 1) return fail(VS_ERR_INVALID_ARG, "vs_flat_search: d = %d < 1", d);
  if (k < 1 || k > VS_MAX_K) return fail(VS_ERR_INVALID_ARG, "vs_flat_search: k = %d outside [1, %d]", k, VS_MAX_K);
  if (metric != VS_METRIC_L2 && metric != VS_METRIC_IP) return fail(VS_ERR_INVALID_ARG, "vs_flat_search: unknown metric %d", metric);
  if (nb >= (1ll << 31)) return fail(VS_ERR_INVALID_ARG, "vs_flat_search: nb must be < 2^31");
  if (nq == 0) return VS_OK;
  if (!q || !out_dist || !out_ids || (nb > 0 && !x)) return fail(VS_ERR_INVALID_ARG, "vs_flat_search: null pointer");
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= 16) return fail(VS_ERR_UNSUPPORTED, "vs_flat_search: device %d", dev);

  const KnnPlan plan = knn_plan(nq, nb, d, k, false);
  ScratchUse guard(g_flat_scratch[dev], st);
  Scratch& sc = g_flat_scratch[dev];
  if (int rc = sc.reserve(plan.bytes + (size_t)nq * k * sizeof(u64))) return rc;
  char* base = static_cast<char*>(sc.p);
  SelectOut out;
  out.val = out_dist;
  out.id64 = out_ids;
  if (nb == 0) {   // nothing to select from: all slots empty
    u64* keys = reinterpret_cast<u64*>(base);
    launch_fill_u64(keys, nq * k, 0xFFFFFFFFFFFFFFFFull, st);
    launch_keys_to_results(keys, nq * k, metric, out_dist, out_ids, nullptr, st);
  } else {
    if (int rc = knn_run(plan, base, q, nq, x, nb, d, metric, k, nullptr, out, st, VS_STAGE_FLAT_DIST,
                         VS_STAGE_FLAT_SELECT))
      return rc;
  }
  HIP_TRY(hipGetLastError());
  return VS_OK;
}

int vs_flat_create(vs_flat** out, int32_t d, int32_t metric) {
  if (!out) return fail(VS_ERR_INVALID_ARG, "vs_flat_create: out is null");
  *out = nullptr;
  if (d < 1) return fail(VS_ERR_INVALID_ARG, "vs_flat_create: d = %d < 1", d);
  if (metric != VS_METRIC_L2 && metric != VS_METRIC_IP) return fail(VS_ERR_INVALID_ARG, "vs_flat_create: unknown metric %d", metric);
  vs_flat* ix = new (std::nothrow) vs_flat();
  if (!ix) return fail(VS_ERR_OOM, "vs_flat_create: host allocation failed");
  ix->d = d; ix->metric = metric;
  if (hipError_t e = hipGetDevice(&ix->device); e != hipSuccess) {
    delete ix;
    return fail(VS_ERR_DEVICE, "vs_flat_create: %s", hipGetErrorString(e));
  }
  *out = ix;
  return VS_OK;
}

void vs_flat_destroy(vs_flat* ix) {
  if (!ix) return;
  if (ix->x) (void)hipFree(ix->x);
  if (ix->plane_mem) (void)hipFree(ix->plane_mem);
  delete ix;
}

int64_t vs_flat_ntotal(const vs_flat* ix) { return ix ? ix->ntotal : -1; }

int vs_flat_add(vs_flat* ix, const float* x, int64_t n, void* hip_stream) {
  if (!ix) return fail(VS_ERR_INVALID_ARG, "vs_flat_add: index is null");
  if (n < 0) return fail(VS_ERR_INVALID_ARG, "vs_flat_add: negative size");
  if (n == 0) return VS_OK;
  if (!x) return fail(VS_ERR_INVALID_ARG, "vs_flat_add: null pointer");
  if (ix->ntotal + n >= (1ll << 31)) return fail(VS_ERR_INVALID_ARG, "vs_flat_add: ntotal must stay below 2^31");
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int d = ix->d;
  const bool planes = mfma_knn_supported(d, 1);
  const int64_t total = ix->ntotal + n;
  if (total > ix->cap) {   // grow both buffers (at least doubling), keep the stored rows
    const int64_t cap = std::max(total, 2 * ix->cap);
    float* nx = nullptr;
    void* np = nullptr;
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&nx), (size_t)cap * d * sizeof(float));
    if (e == hipSuccess && planes) e = hipMalloc(&np, planes_bytes(cap, d));
    if (e == hipSuccess && ix->ntotal > 0)
      e = hipMemcpyAsync(nx, ix->x, (size_t)ix->ntotal * d * sizeof(float), hipMemcpyDeviceToDevice, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) {
      if (nx) (void)hipFree(nx);
      if (np) (void)hipFree(np);
      (void)hipGetLastError();
      return fail(e == hipErrorOutOfMemory ? VS_ERR_OOM : VS_ERR_DEVICE, "vs_flat_add: %s", hipGetErrorString(e));
    }
    if (ix->x) (void)hipFree(ix->x);
    if (ix->plane_mem) (void)hipFree(ix->plane_mem);
    ix->x = nx; ix->plane_mem = np; ix->cap = cap;
  }
  HIP_TRY(hipMemcpyAsync(ix->x + ix->ntotal * d, x, (size_t)n * d * sizeof(float), hipMemcpyDeviceToDevice, st));
  ix->ntotal = total;
  if (planes) {   // (the panel layout of the planes depends on the row count: prepared anew)
    ix->planes = carve_planes(static_cast<char*>(ix->plane_mem), total, d);
    launch_prep(ix->x, total, d, ix->planes.hi, ix->planes.lo, ix->planes.norm, ix->planes.info, st, true);
    ix->planes.try_heads_only = true;
    ix->has_planes = true;
  }
  HIP_TRY(hipStreamSynchronize(st));
  if (planes) HIP_TRY(learn_planes(&ix->planes));
  HIP_TRY(hipGetLastError());
  return VS_OK;
}

int vs_flat_index_search(const vs_flat* ix, const float* q, int64_t nq, int32_t k, float* out_dist,
                         int64_t* out_ids, void* hip_stream) {
  if (!ix) return fail(VS_ERR_INVALID_ARG, "vs_flat_index_search: index is null");
  if (nq < 0) return fail(VS_ERR_INVALID_ARG, "vs_flat_index_search: negative size");
  if (k < 1 || k > VS_MAX_K) return fail(VS_ERR_INVALID_ARG, "vs_flat_index_search: k = %d outside [1, %d]", k, VS_MAX_K);
  if (nq == 0) return VS_OK;
  if (!q || !out_dist || !out_ids) return fail(VS_ERR_INVALID_ARG, "vs_flat_index_search: null pointer");
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int dev = ix->device;
  if (dev < 0 || dev >= 16) return fail(VS_ERR_UNSUPPORTED, "vs_flat_index_search: device %d", dev);
  const int64_t nb = ix->ntotal;
  const int d = ix->d, metric = ix->metric;
  const Planes* bp = ix->has_planes ? &ix->planes : nullptr;
  const KnnPlan plan = knn_plan(nq, nb, d, k, bp != nullptr);
  ScratchUse guard(g_flat_scratch[dev], st);
  Scratch& sc = g_flat_scratch[dev];
  if (int rc = sc.reserve(plan.bytes + (size_t)nq * k * sizeof(u64))) return rc;
  char* base = static_cast<char*>(sc.p);
  SelectOut out;
  out.val = out_dist;
  out.id64 = out_ids;
  if (nb == 0) {   // nothing to select from: all slots empty
    u64* keys = reinterpret_cast<u64*>(base);
    launch_fill_u64(keys, nq * k, 0xFFFFFFFFFFFFFFFFull, st);
    launch_keys_to_results(keys, nq * k, metric, out_dist, out_ids, nullptr, st);
  } else {
    if (int rc = knn_run(plan, base, q, nq, ix->x, nb, d, metric, k, bp, out, st, VS_STAGE_FLAT_DIST,
                         VS_STAGE_FLAT_SELECT))
      return rc;
  }
  HIP_TRY(hipGetLastError());
  return VS_OK;
}

int vs_trim(void) {
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= 16) return fail(VS_ERR_UNSUPPORTED, "vs_trim: device %d", dev);
  std::lock_guard<std::mutex> lock(g_flat_scratch[dev].mu);
  HIP_TRY(hipDeviceSynchronize());   // nothing may still be using the buffer
  g_flat_scratch[dev].release();
  return VS_OK;
}

int vs_refine(const float* x, int64_t nb, const float* q, int64_t nq, int32_t d, int32_t metric,
              const int64_t* cand_ids, int32_t kc, int32_t k, float* out_dist, int64_t* out_ids,
              void* hip_stream) {
  if (nq < 0 || nb < 0) return fail(VS_ERR_INVALID_ARG, "vs_refine: negative size");
  if (d < 1) return fail(VS_ERR_INVALID_ARG, "vs_refine: d = %d < 1", d);
  if (k < 1 || k > VS_MAX_K) return fail(VS_ERR_INVALID_ARG, "vs_refine: k = %d outside [1, %d]", k, VS_MAX_K);
  if (kc < 1) return fail(VS_ERR_INVALID_ARG, "vs_refine: kc = %d < 1", kc);
  if (metric != VS_METRIC_L2 && metric != VS_METRIC_IP) return fail(VS_ERR_INVALID_ARG, "vs_refine: unknown metric %d", metric);
  if (nb >= (1ll << 32)) return fail(VS_ERR_INVALID_ARG, "vs_refine: nb must be < 2^32");
  if (nq == 0) return VS_OK;
  if (!q || !cand_ids || !out_dist || !out_ids || (nb > 0 && !x)) return fail(VS_ERR_INVALID_ARG, "vs_refine: null pointer");
  // per wavefront: the selection slots and the query, four wavefronts per workgroup
  const size_t lds = refine_lds_bytes(d, k);
  if (lds > 160 * 1024) return fail(VS_ERR_UNSUPPORTED, "vs_refine: d = %d with k = %d needs %zu bytes of LDS", d, k, lds);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  {
    StageTimer t(VS_STAGE_REFINE, st);
    launch_refine(x, nb, q, nq, d, metric, cand_ids, kc, k, out_dist, out_ids, st);
  }
  HIP_TRY(hipGetLastError());
  return VS_OK;
}

namespace {

// Best row of B [nb, d] for every row of A [n, d] (k-nearest-rows with k = 1, in pieces of 2^20
// rows): idx [n] and, if asked for, the canon value val [n].  `sc` is grown as needed.
int nearest_rows(const float* A, int64_t n, const float* B, int64_t nb, int d, int metric,
                 int32_t* idx, float* val, Scratch& sc, hipStream_t st) {
  constexpr int64_t kPiece = 1 << 20;
  const KnnPlan plan = knn_plan_pieces(n, kPiece, nb, d, 1, false);
  if (!plan.mfma) {
    // shapes the matrix-core kernels do not cover (sub-vectors of a few dimensions): fused canon
    // distance + arg-best tiles, one 64-bit key (value, row of B) per row of A
    if (int rc = sc.reserve((size_t)n * sizeof(u64))) return rc;
    u64* keys = static_cast<u64*>(sc.p);
    launch_fill_u64(keys, n, 0xFFFFFFFFFFFFFFFFull, st);
    launch_canon_argbest(A, n, B, nb, d, metric, keys, st);
    launch_keys_to_probes(keys, n, metric, idx, val, st);
    return VS_OK;
  }
  if (int rc = sc.reserve(plan.bytes)) return rc;
  for (int64_t i0 = 0; i0 < n; i0 += kPiece) {
    const int64_t ni = std::min(kPiece, n - i0);
    SelectOut o;
    o.idx32 = idx + i0;
    o.val = val ? val + i0 : nullptr;
    if (int rc = knn_run(plan, static_cast<char*>(sc.p), A + i0 * d, ni, B, nb, d, metric, 1, nullptr, o,
                         st, -1, -1))
      return rc;
  }
  return VS_OK;
}

struct DeviceBuf {   // a plain allocation released on scope exit
  void* p = nullptr;
  ~DeviceBuf() { if (p) (void)hipFree(p); }
  int alloc(size_t bytes) { HIP_TRY(hipMalloc(&p, std::max<size_t>(bytes, 256))); return VS_OK; }
};

// niter rounds of Lloyd's iteration on device data.  dev_buf: idx [n] int32 | val [n] fp32 |
// order [n] int32 | off [K + 1] int64, carved by the caller; sc: scratch of the assignment.
int kmeans_rounds(const float* x, int64_t n, int d, int K, int niter, float* centroids,
                  double* objective, int32_t* idx, float* val, int32_t* order, int64_t* off,
                  Scratch& sc, hipStream_t st) {
  // Up to 16384 centroids the bookkeeping of a round (the objective, and every centroid's
  // vectors in ascending order) stays on the device; beyond, the host does it.
  const bool on_device = K <= 16384 && n > 0;
  DeviceBuf sortbuf;
  if (on_device) { if (int rc = sortbuf.alloc(kmeans_sort_bytes(n, K))) return rc; }
  std::vector<int32_t> h_idx(on_device ? 0 : (size_t)n), h_order(on_device ? 0 : (size_t)n);
  std::vector<float> h_val(on_device ? 0 : (size_t)n);
  std::vector<int64_t> h_off((size_t)K + 1), cursor((size_t)K);
  for (int r = 0; r < niter; ++r) {
    // (1) nearest centroid of every vector: canon L2, ties to the smaller centroid number
    if (int rc = nearest_rows(x, n, centroids, K, d, VS_METRIC_L2, idx, val, sc, st)) return rc;
    if (on_device) {
      int64_t* scal = nullptr;
      double* partial = nullptr;
      launch_kmeans_sort(idx, val, n, K, static_cast<char*>(sortbuf.p), order, off, &scal, &partial, st);
      int64_t h_scal[2];
      double h_part[256];
      HIP_TRY(hipMemcpyAsync(h_scal, scal, sizeof(h_scal), hipMemcpyDeviceToHost, st));
      HIP_TRY(hipMemcpyAsync(h_part, partial, sizeof(h_part), hipMemcpyDeviceToHost, st));
      HIP_TRY(hipStreamSynchronize(st));
      if (h_scal[1] != 0) return fail(VS_ERR_DEVICE, "k-means: assignment produced a centroid outside [0, %d)", K);
      double obj = 0.0;
      for (int t = 0; t < 256; ++t) obj += h_part[t];
      if (objective) objective[r] = obj / (double)n;
      if (int rc = sc.reserve(segmented_mean_partial_bytes(n, d, K, h_scal[0]))) return rc;
      launch_segmented_mean(x, d, order, off, K, h_scal[0], centroids, static_cast<double*>(sc.p), st);
      continue;
    }
    HIP_TRY(hipMemcpyAsync(h_idx.data(), idx, (size_t)n * sizeof(int32_t), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipMemcpyAsync(h_val.data(), val, (size_t)n * sizeof(float), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    // host bookkeeping, one pass over n numbers: the objective, and the vectors of every
    // centroid in ascending order (a stable counting sort)
    double obj = 0.0;
    std::fill(h_off.begin(), h_off.end(), 0);
    for (int64_t i = 0; i < n; ++i) {
      const int32_t j = h_idx[(size_t)i];
      if (j < 0 || j >= K) return fail(VS_ERR_DEVICE, "k-means: assignment produced centroid %d", j);
      obj += (double)h_val[(size_t)i];
      ++h_off[(size_t)j + 1];
    }
    if (objective) objective[r] = n > 0 ? obj / (double)n : 0.0;
    int64_t largest = 0;
    for (int j = 0; j < K; ++j) largest = std::max(largest, h_off[(size_t)j + 1]);
    for (int j = 0; j < K; ++j) { h_off[(size_t)j + 1] += h_off[(size_t)j]; cursor[(size_t)j] = h_off[(size_t)j]; }
    for (int64_t i = 0; i < n; ++i) h_order[(size_t)cursor[(size_t)h_idx[(size_t)i]]++] = (int32_t)i;
    HIP_TRY(hipMemcpyAsync(order, h_order.data(), (size_t)n * sizeof(int32_t), hipMemcpyHostToDevice, st));
    HIP_TRY(hipMemcpyAsync(off, h_off.data(), h_off.size() * sizeof(int64_t), hipMemcpyHostToDevice, st));
    // (2) every centroid moves to the mean of its vectors (the assignment's scratch is free
    // again: it holds the block sums of clusters longer than one summation block)
    if (int rc = sc.reserve(segmented_mean_partial_bytes(n, d, K, largest))) return rc;
    launch_segmented_mean(x, d, order, off, K, largest, centroids, static_cast<double*>(sc.p), st);
    HIP_TRY(hipStreamSynchronize(st));   // the host arrays are reused by the next round
  }
  HIP_TRY(hipStreamSynchronize(st));     // the centroids are final when the call returns
  HIP_TRY(hipGetLastError());
  return VS_OK;
}

}  // namespace

int vs_kmeans(const float* x, int64_t n, int32_t d, int32_t K, int32_t niter, float* centroids,
              double* objective, int32_t* assign, void* hip_stream) {
  if (n < 0 || n >= (1ll << 31)) return fail(VS_ERR_INVALID_ARG, "vs_kmeans: n outside [0, 2^31)");
  if (d < 1 || K < 1) return fail(VS_ERR_INVALID_ARG, "vs_kmeans: d = %d, K = %d must be >= 1", d, K);
  if (niter < 0) return fail(VS_ERR_INVALID_ARG, "vs_kmeans: niter < 0");
  if (!centroids || (n > 0 && !x)) return fail(VS_ERR_INVALID_ARG, "vs_kmeans: null pointer");
  if (niter == 0) return VS_OK;
  if (n == 0) {   // nothing to assign: every centroid stays, the objective is 0
    if (objective) for (int r = 0; r < niter; ++r) objective[r] = 0.0;
    return VS_OK;
  }
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= 16) return fail(VS_ERR_UNSUPPORTED, "vs_kmeans: device %d", dev);
  Carver cv;
  const size_t o_idx = cv.take((size_t)n * sizeof(int32_t));
  const size_t o_val = cv.take((size_t)n * sizeof(float));
  const size_t o_order = cv.take((size_t)n * sizeof(int32_t));
  const size_t o_off = cv.take(((size_t)K + 1) * sizeof(int64_t));
  DeviceBuf buf;
  if (int rc = buf.alloc(cv.off)) return rc;
  char* b = static_cast<char*>(buf.p);
  ScratchUse guard(g_flat_scratch[dev], st);
  if (int rc = kmeans_rounds(x, n, d, K, niter, centroids, objective, reinterpret_cast<int32_t*>(b + o_idx),
                             reinterpret_cast<float*>(b + o_val), reinterpret_cast<int32_t*>(b + o_order),
                             reinterpret_cast<int64_t*>(b + o_off), g_flat_scratch[dev], st))
    return rc;
  if (assign) {   // idx still holds the last round's step (1)
    HIP_TRY(hipMemcpyAsync(assign, b + o_idx, (size_t)n * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
    HIP_TRY(hipStreamSynchronize(st));   // the work buffer is released on return
  }
  return VS_OK;
}

int vs_ivfpq_train(const float* x, int64_t n, int32_t d, int32_t metric, int32_t nlist, int32_t M,
                   int32_t nbits, int32_t niter, float* centroids, float* codebooks,
                   double* objective, void* hip_stream) {
  if (n < 1 || n >= (1ll << 31)) return fail(VS_ERR_INVALID_ARG, "vs_ivfpq_train: n outside [1, 2^31)");
  if (d < 1 || nlist < 1 || M < 1) return fail(VS_ERR_INVALID_ARG, "vs_ivfpq_train: d, nlist, M must be >= 1");
  if (d % M != 0) return fail(VS_ERR_INVALID_ARG, "vs_ivfpq_train: d = %d is not a multiple of M = %d", d, M);
  if (metric != VS_METRIC_L2 && metric != VS_METRIC_IP) return fail(VS_ERR_INVALID_ARG, "vs_ivfpq_train: unknown metric %d", metric);
  if (nbits != 4 && nbits != 8) return fail(VS_ERR_UNSUPPORTED, "vs_ivfpq_train: nbits = %d (only 4 and 8)", nbits);
  if (niter < 0) return fail(VS_ERR_INVALID_ARG, "vs_ivfpq_train: niter < 0");
  if (!x || !centroids || !codebooks) return fail(VS_ERR_INVALID_ARG, "vs_ivfpq_train: null pointer");
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= 16) return fail(VS_ERR_UNSUPPORTED, "vs_ivfpq_train: device %d", dev);
  const int K = 1 << nbits, dsub = d / M, kmax = std::max(nlist, K);
  Carver cv;
  const size_t o_idx = cv.take((size_t)n * sizeof(int32_t));
  const size_t o_val = cv.take((size_t)n * sizeof(float));
  const size_t o_order = cv.take((size_t)n * sizeof(int32_t));
  const size_t o_off = cv.take(((size_t)kmax + 1) * sizeof(int64_t));
  const size_t o_res = cv.take((size_t)n * d * sizeof(float));
  DeviceBuf buf;
  if (int rc = buf.alloc(cv.off)) return rc;
  char* b = static_cast<char*>(buf.p);
  int32_t* idx = reinterpret_cast<int32_t*>(b + o_idx);
  float* val = reinterpret_cast<float*>(b + o_val);
  int32_t* order = reinterpret_cast<int32_t*>(b + o_order);
  int64_t* off = reinterpret_cast<int64_t*>(b + o_off);
  float* res = reinterpret_cast<float*>(b + o_res);
  ScratchUse guard(g_flat_scratch[dev], st);
  Scratch& sc = g_flat_scratch[dev];
  // 1. coarse quantizer: k-means on the training vectors
  if (int rc = kmeans_rounds(x, n, d, nlist, niter, centroids, objective, idx, val, order, off, sc, st)) return rc;
  // 2. + 3. list of every training vector under the index metric (as vs_ivfpq_add), residuals
  if (int rc = nearest_rows(x, n, centroids, nlist, d, metric, idx, nullptr, sc, st)) return rc;
  launch_residual_slices(x, n, d, dsub, centroids, idx, res, st);
  // 4. one k-means per sub-quantizer on its slice of the residuals
  for (int m = 0; m < M; ++m) {
    if (int rc = kmeans_rounds(res + (size_t)m * n * dsub, n, dsub, K, niter,
                               codebooks + (size_t)m * K * dsub,
                               objective ? objective + (size_t)(1 + m) * niter : nullptr, idx, val,
                               order, off, sc, st))
      return rc;
  }
  HIP_TRY(hipStreamSynchronize(st));
  HIP_TRY(hipGetLastError());
  return VS_OK;
}

int vs_ivfpq_create(vs_ivfpq** out, int32_t d, int32_t metric, int32_t nlist, int32_t M,
                    int32_t nbits, const float* centroids, const float* codebooks,
                    void* hip_stream) {
  if (!out) return fail(VS_ERR_INVALID_ARG, "vs_ivfpq_create: out is null");
  *out = nullptr;
  if (!centroids || !codebooks) return fail(VS_ERR_INVALID_ARG, "vs_ivfpq_create: null pointer");
  if (d < 1 || nlist < 1 || M < 1) return fail(VS_ERR_INVALID_ARG, "vs_ivfpq_create: d, nlist, M must be >= 1");
  if (d % M != 0) return fail(VS_ERR_INVALID_ARG, "vs_ivfpq_create: d = %d is not a multiple of M = %d", d, M);
  if (metric != VS_METRIC_L2 && metric != VS_METRIC_IP) return fail(VS_ERR_INVALID_ARG, "vs_ivfpq_create: unknown metric %d", metric);
  if (nbits != 4 && nbits != 8) return fail(VS_ERR_UNSUPPORTED, "vs_ivfpq_create: nbits = %d (only 4 and 8)", nbits);
  if (nbits == 4 && (M & 1)) return fail(VS_ERR_INVALID_ARG, "vs_ivfpq_create: M must be even with 4-bit codes");
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  vs_ivfpq* ix = new (std::nothrow) vs_ivfpq();
  if (!ix) return fail(VS_ERR_OOM, "vs_ivfpq_create: host allocation failed");
  ix->g.d = d; ix->g.metric = metric; ix->g.nlist = nlist; ix->g.M = M; ix->g.nbits = nbits;
  ix->g.K = 1 << nbits; ix->g.dsub = d / M; ix->g.code_size = M * nbits / 8;
  ix->h_off.assign((size_t)nlist + 1, 0);
  auto cleanup = [&](int rc) { vs_ivfpq_destroy(ix); return rc; };
#define TRY_C(expr)                                                                         \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess)                                                                   \
      return cleanup(fail(e_ == hipErrorOutOfMemory ? VS_ERR_OOM : VS_ERR_DEVICE, "%s: %s", \
                          #expr, hipGetErrorString(e_)));                                   \
  } while (0)
  TRY_C(hipGetDevice(&ix->device));
  const size_t cb = (size_t)nlist * d * sizeof(float);
  const size_t tb = (size_t)M * ix->g.K * ix->g.dsub * sizeof(float);
  TRY_C(hipMalloc(reinterpret_cast<void**>(&ix->centroids), cb));
  // (the codebooks twice: [M, K, dsub] as given, and behind it [K, M, dsub], the order in which the
  // per-query tables of the wavefront-private scan are computed)
  TRY_C(hipMalloc(reinterpret_cast<void**>(&ix->codebooks), 2 * tb));
  TRY_C(hipMalloc(reinterpret_cast<void**>(&ix->list_off), ((size_t)nlist + 1) * sizeof(int64_t)));
  TRY_C(hipMemcpyAsync(ix->centroids, centroids, cb, hipMemcpyDeviceToDevice, st));
  TRY_C(hipMemcpyAsync(ix->codebooks, codebooks, tb, hipMemcpyDeviceToDevice, st));
  launch_pq_codebooks_by_entry(ix->g, ix->codebooks, ix->codebooks + tb / sizeof(float), st);
  TRY_C(hipMalloc(reinterpret_cast<void**>(&ix->cnorm), (size_t)nlist * sizeof(float)));
  launch_row_norms(ix->centroids, nlist, d, ix->cnorm, st);
  TRY_C(hipMemsetAsync(ix->list_off, 0, ((size_t)nlist + 1) * sizeof(int64_t), st));
  if (mfma_knn_supported(d, 1)) {
    TRY_C(hipMalloc(&ix->plane_mem, planes_bytes(nlist, d)));
    ix->c_planes = carve_planes(static_cast<char*>(ix->plane_mem), nlist, d);
    launch_prep(ix->centroids, nlist, d, ix->c_planes.hi, ix->c_planes.lo, ix->c_planes.norm,
                ix->c_planes.info, st, true);
    ix->c_planes.try_heads_only = true;
    ix->has_planes = true;
  }
  TRY_C(hipStreamSynchronize(st));
  if (ix->has_planes) TRY_C(learn_planes(&ix->c_planes));
#undef TRY_C
  {   // set-up for vs_ivfpq_search_static: this device's address of the static work space
    char* unused = nullptr;
    if (int rc = static_scratch(&unused)) return cleanup(rc);
  }
  *out = ix;
  return VS_OK;
}

static void ivf_free_device_memory(vs_ivfpq* ix) {
  if (ix->centroids) (void)hipFree(ix->centroids);
  if (ix->codebooks) (void)hipFree(ix->codebooks);
  if (ix->list_off) (void)hipFree(ix->list_off);
  if (ix->codes) (void)hipFree(ix->codes);
  if (ix->ids) (void)hipFree(ix->ids);
  if (ix->norms) (void)hipFree(ix->norms);
  if (ix->cnorm) (void)hipFree(ix->cnorm);
  if (ix->list_tables) (void)hipFree(ix->list_tables);
  if (ix->plane_mem) (void)hipFree(ix->plane_mem);
  ix->scratch.release();
}

void vs_ivfpq_destroy(vs_ivfpq* ix) {
  if (!ix) return;
  ivf_free_device_memory(ix);
  delete ix;
}

int64_t vs_ivfpq_ntotal(const vs_ivfpq* ix) { return ix ? ix->ntotal : -1; }
int32_t vs_ivfpq_code_size(const vs_ivfpq* ix) { return ix ? ix->g.code_size : -1; }

namespace {

// Where the n new vectors of an add go: list of every vector (device), its position in the
// grown list-contiguous storage (device), the grown offsets (device and host), and `extra`
// bytes of scratch for the caller.  Steps: (1) best centroid on the canon chain, ties to the
// smaller list; (2) stable placement -- the new entries of a list follow its old ones, in the
// order given (a stable sort of the batch by list on the device: launch_ivf_place).
struct Placement {
  int32_t* list_of = nullptr;
  int64_t* dest = nullptr;
  int64_t* new_off = nullptr;
  char* extra = nullptr;
  std::vector<int64_t> h_new;
};

int ivf_assign_and_place(vs_ivfpq* ix, const float* x, int64_t n, size_t extra, Placement* pl,
                         hipStream_t st, const char* who) {
  const IvfpqDims& g = ix->g;
  const int cmetric = ix->coarse_metric < 0 ? g.metric : ix->coarse_metric;   // lists are chosen under the coarse metric
  if (n >= (1ll << 31)) return fail(VS_ERR_UNSUPPORTED, "%s: at most 2^31 - 1 vectors per call", who);
  // scratch: work space of the MFMA assignment (pieces of at most kAssignPiece vectors) |
  // best keys [n] | list_of [n] | caller's extra | dest [n] | new offsets | work space of the placement
  constexpr int64_t kAssignPiece = 1 << 20;
  // The first piece of an index's first large add is a short one: the sweeps start out on the
  // fp16 heads alone and learn from a call's fallback count whether that does for this data; a
  // short first call keeps the price of finding out small.
  constexpr int64_t kProbePiece = 8192;
  const int64_t first_piece = !ix->assign_probed && n > 4 * kProbePiece ? kProbePiece : 0;
  KnnPlan plan = knn_plan_pieces(n - first_piece, kAssignPiece, g.nlist, g.d, 1, ix->has_planes);
  if (first_piece > 0) {
    const KnnPlan probe = knn_plan(first_piece, g.nlist, g.d, 1, ix->has_planes);
    plan.bytes = std::max(plan.bytes, probe.bytes);
  }
  if (!plan.mfma) plan.bytes = 0;
  Carver cv;
  const size_t o_knn = cv.take(plan.bytes);
  const size_t o_keys = cv.take((size_t)n * sizeof(u64));
  const size_t o_list = cv.take((size_t)n * sizeof(int32_t));
  const size_t o_extra = cv.take(extra);
  const size_t o_dest = cv.take((size_t)n * sizeof(int64_t));
  const size_t o_off = cv.take(((size_t)g.nlist + 1) * sizeof(int64_t));
  const size_t o_place = cv.take(ivf_place_work_bytes(n, g.nlist));
  if (int rc = ix->scratch.reserve(cv.off)) return rc;
  char* base = static_cast<char*>(ix->scratch.p);
  u64* keys = reinterpret_cast<u64*>(base + o_keys);
  pl->list_of = reinterpret_cast<int32_t*>(base + o_list);
  pl->extra = base + o_extra;
  pl->dest = reinterpret_cast<int64_t*>(base + o_dest);
  pl->new_off = reinterpret_cast<int64_t*>(base + o_off);

  if (plan.mfma) {
    for (int64_t i0 = 0; i0 < n;) {
      const int64_t ni = i0 == 0 && first_piece > 0 ? first_piece : std::min(kAssignPiece, n - i0);
      SelectOut o;
      o.idx32 = pl->list_of + i0;
      if (int rc = knn_run(plan, base + o_knn, x + i0 * g.d, ni, ix->centroids, g.nlist, g.d, cmetric, 1,
                           ix->has_planes ? &ix->c_planes : nullptr, o, st, -1, -1))
        return rc;
      i0 += ni;
    }
    ix->assign_probed = true;
  } else {
    launch_fill_u64(keys, n, 0xFFFFFFFFFFFFFFFFull, st);
    launch_canon_argbest(x, n, ix->centroids, g.nlist, g.d, cmetric, keys, st);
    launch_keys_to_index32(keys, n, pl->list_of, st);
  }

  // slots in the grown lists: a stable sort of the batch by list, on the device; only the new
  // offsets (nlist + 1 numbers) and one flag come back to the host
  int* bad = launch_ivf_place(pl->list_of, n, g.nlist, ix->list_off, base + o_place, pl->dest, pl->new_off, st);
  pl->h_new.assign((size_t)g.nlist + 1, 0);
  int h_bad = 0;
  HIP_TRY(hipMemcpyAsync(pl->h_new.data(), pl->new_off, pl->h_new.size() * sizeof(int64_t), hipMemcpyDeviceToHost, st));
  HIP_TRY(hipMemcpyAsync(&h_bad, bad, sizeof(int), hipMemcpyDeviceToHost, st));
  HIP_TRY(hipStreamSynchronize(st));
  HIP_TRY(hipGetLastError());
  if (h_bad) return fail(VS_ERR_DEVICE, "%s: the assignment kernel produced a list outside [0, %d)", who, g.nlist);
  if (pl->h_new[(size_t)g.nlist] != ix->ntotal + n)
    return fail(VS_ERR_DEVICE, "%s: %lld slots placed for %lld stored + %lld new vectors", who,
                (long long)pl->h_new[(size_t)g.nlist], (long long)ix->ntotal, (long long)n);
  return VS_OK;
}

// Installs the grown storage (already filled on the stream) in place of the old one.
int ivf_commit_storage(vs_ivfpq* ix, uint8_t* codes, int64_t* new_ids, float* new_norms,
                       int64_t total, Placement* pl, hipStream_t st, const char* who) {
  hipError_t e = hipMemcpyAsync(ix->list_off, pl->new_off, pl->h_new.size() * sizeof(int64_t), hipMemcpyDeviceToDevice, st);
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  if (e == hipSuccess) e = hipGetLastError();
  if (e != hipSuccess) {
    (void)hipFree(codes); (void)hipFree(new_ids);
    if (new_norms) (void)hipFree(new_norms);
    return fail(VS_ERR_DEVICE, "%s: %s", who, hipGetErrorString(e));
  }
  if (ix->codes) (void)hipFree(ix->codes);
  if (ix->ids) (void)hipFree(ix->ids);
  if (ix->norms) (void)hipFree(ix->norms);
  ix->codes = codes; ix->ids = new_ids; ix->norms = new_norms; ix->ntotal = total;
  ix->h_off.swap(pl->h_new);
  return VS_OK;
}

}  // namespace

int vs_ivfpq_add(vs_ivfpq* ix, const float* x, int64_t n, const int64_t* ids, void* hip_stream) {
  if (!ix) return fail(VS_ERR_INVALID_ARG, "vs_ivfpq_add: index is null");
  if (n < 0) return fail(VS_ERR_INVALID_ARG, "vs_ivfpq_add: n < 0");
  if (n == 0) return VS_OK;
  if (!x) return fail(VS_ERR_INVALID_ARG, "vs_ivfpq_add: x is null");
  if (ix->ntotal + n >= (1ll << 32)) return fail(VS_ERR_UNSUPPORTED, "vs_ivfpq_add: more than 2^32 - 1 stored vectors");
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const IvfpqDims& g = ix->g;
  Placement pl;
  // one byte per (vector, m) for the codes before they are packed into their lists, and
  // (search type "stored norms") one float per vector
  const bool with_norms = ix->search_type == VS_ST_STORED_NORMS;
  const size_t code_bytes = align_up((size_t)n * g.M);
  if (int rc = ivf_assign_and_place(ix, x, n, code_bytes + (with_norms ? (size_t)n * sizeof(float) : 0),
                                    &pl, st, "vs_ivfpq_add"))
    return rc;
  uint8_t* tmp_codes = reinterpret_cast<uint8_t*>(pl.extra);
  float* tmp_norms = with_norms ? reinterpret_cast<float*>(pl.extra + code_bytes) : nullptr;
  launch_pq_encode(g, x, n, pl.list_of, ix->centroids, ix->codebooks, tmp_codes, st);
  if (with_norms)
    launch_pq_norms(g, tmp_codes, n, pl.list_of, ix->centroids, ix->codebooks, tmp_norms, st);

  const int64_t total = ix->ntotal + n;
  uint8_t* codes = nullptr;
  int64_t* new_ids = nullptr;
  float* new_norms = nullptr;
  HIP_TRY(hipMalloc(reinterpret_cast<void**>(&codes), (size_t)total * g.code_size));
  if (hipMalloc(reinterpret_cast<void**>(&new_ids), (size_t)total * sizeof(int64_t)) != hipSuccess ||
      (with_norms && hipMalloc(reinterpret_cast<void**>(&new_norms), (size_t)total * sizeof(float)) != hipSuccess)) {
    (void)hipFree(codes);
    if (new_ids) (void)hipFree(new_ids);
    return fail(VS_ERR_OOM, "vs_ivfpq_add: id / norm storage allocation failed");
  }
  launch_relayout(g, ix->codes, ix->ids, ix->norms, ix->ntotal, ix->list_off, pl.new_off, tmp_codes,
                  ids, ix->ntotal, tmp_norms, pl.dest, pl.list_of, n, codes, new_ids, new_norms, st);
  return ivf_commit_storage(ix, codes, new_ids, new_norms, total, &pl, st, "vs_ivfpq_add");
}

int vs_ivfpq_set_search_type(vs_ivfpq* ix, int32_t search_type) {
  if (!ix) return fail(VS_ERR_INVALID_ARG, "vs_ivfpq_set_search_type: index is null");
  if (search_type != VS_ST_RESIDUAL_TABLES && search_type != VS_ST_STORED_NORMS &&
      search_type != VS_ST_PRECOMPUTED_TABLES)
    return fail(VS_ERR_INVALID_ARG, "vs_ivfpq_set_search_type: unknown search type %d", search_type);
  if (search_type != VS_ST_RESIDUAL_TABLES && ix->g.metric != VS_METRIC_L2)
    return fail(VS_ERR_INVALID_ARG, "vs_ivfpq_set_search_type: stored norms and precomputed tables serve the L2 metric only");
  if (ix->ntotal > 0 && search_type == VS_ST_STORED_NORMS && !ix->norms) {
    // the index holds vectors without norms: compute them from the stored codes, with the kernel
    // that vs_ivfpq_add uses (it takes codes in their canonical byte order and the list of each)
    const IvfpqDims& g = ix->g;
    const int64_t n = ix->ntotal;
    const bool rotated = ivfpq_codes_rotated(g);
    float* norms = nullptr;
    int32_t* list_of = nullptr;
    uint8_t* canon = nullptr;
    auto release = [&] {
      if (list_of) (void)hipFree(list_of);
      if (canon) (void)hipFree(canon);
    };
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&norms), (size_t)n * sizeof(float));
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&list_of), (size_t)n * sizeof(int32_t));
    if (e == hipSuccess && rotated) e = hipMalloc(reinterpret_cast<void**>(&canon), (size_t)n * g.code_size);
    if (e == hipSuccess) {
      launch_list_of_storage(ix->list_off, g.nlist, n, list_of, nullptr);
      if (rotated) launch_codes_canonical(g, ix->codes, ix->list_off, n, canon, nullptr);
      launch_pq_norms(g, rotated ? canon : ix->codes, n, list_of, ix->centroids, ix->codebooks, norms, nullptr,
                      true);
      e = hipStreamSynchronize(nullptr);
      if (e == hipSuccess) e = hipGetLastError();
    }
    release();
    if (e != hipSuccess) {
      if (norms) (void)hipFree(norms);
      return fail(e == hipErrorOutOfMemory ? VS_ERR_OOM : VS_ERR_DEVICE, "vs_ivfpq_set_search_type: %s",
                  hipGetErrorString(e));
    }
    ix->norms = norms;
  }
  if (search_type == VS_ST_PRECOMPUTED_TABLES && !ix->list_tables) {
    const IvfpqDims& g = ix->g;
    if (!ivfpq_codes_rotated(g))
      return fail(VS_ERR_UNSUPPORTED, "vs_ivfpq_set_search_type: precomputed tables exist for 8-bit codes of "
                  "8 x 4, 16 x 8 and 32 x 3 dimensions only (M = %d, d / M = %d, nbits = %d)", g.M, g.dsub, g.nbits);
    // one table of M * K floats per list (the centroids and codebooks never change after create)
    float* t = nullptr;
    HIP_TRY(hipMalloc(reinterpret_cast<void**>(&t), (size_t)g.nlist * g.K * g.M * sizeof(float)));
    launch_pq_list_tables(g, ix->centroids, ix->codebooks, t, nullptr);
    hipError_t e = hipStreamSynchronize(nullptr);
    if (e == hipSuccess) e = hipGetLastError();
    if (e != hipSuccess) { (void)hipFree(t); return fail(VS_ERR_DEVICE, "vs_ivfpq_set_search_type: %s", hipGetErrorString(e)); }
    ix->list_tables = t;
  }
  ix->search_type = search_type;   // norms and tables already stored are kept, so one can switch back and forth
  return VS_OK;
}

int vs_ivfpq_set_coarse_metric(vs_ivfpq* ix, int32_t metric) {
  if (!ix) return fail(VS_ERR_INVALID_ARG, "vs_ivfpq_set_coarse_metric: index is null");
  if (metric != VS_METRIC_L2 && metric != VS_METRIC_IP)
    return fail(VS_ERR_INVALID_ARG, "vs_ivfpq_set_coarse_metric: unknown metric %d", metric);
  if (ix->g.metric == VS_METRIC_L2 && metric != VS_METRIC_L2)
    return fail(VS_ERR_INVALID_ARG, "vs_ivfpq_set_coarse_metric: an L2 index chooses its lists by L2");
  if (ix->ntotal > 0 && metric != coarse_metric_of(ix))
    return fail(VS_ERR_INVALID_ARG, "vs_ivfpq_set_coarse_metric: the index already holds vectors assigned under the other metric");
  ix->coarse_metric = metric;
  return VS_OK;
}

int vs_ivfpq_get_norms(const vs_ivfpq* ix, float* norms, void* hip_stream) {
  if (!ix || !norms) return fail(VS_ERR_INVALID_ARG, "vs_ivfpq_get_norms: null pointer");
  if (ix->ntotal == 0) return VS_OK;
  if (!ix->norms) return fail(VS_ERR_INVALID_ARG, "vs_ivfpq_get_norms: the index stores no norms");
  HIP_TRY(hipMemcpyAsync(norms, ix->norms, (size_t)ix->ntotal * sizeof(float), hipMemcpyDeviceToDevice,
                         static_cast<hipStream_t>(hip_stream)));
  return VS_OK;
}

// coarse quantizer: the npr best lists per query, best first, with their canon values (under the
// coarse metric)
static int coarse_select(const vs_ivfpq* ix, const KnnPlan& plan, char* ws, const float* q,
                         int64_t nq, int npr, int32_t* probes, float* cdist, hipStream_t st,
                         bool timed = true, const int** fallback_count = nullptr) {
  SelectOut out;
  out.val = cdist;
  out.idx32 = probes;
  return knn_run(plan, ws, q, nq, ix->centroids, ix->g.nlist, ix->g.d, coarse_metric_of(ix), npr,
                 ix->has_planes ? &ix->c_planes : nullptr, out, st, timed ? VS_STAGE_COARSE_DIST : -1,
                 timed ? VS_STAGE_COARSE_SELECT : -1, fallback_count);
}

int vs_ivfpq_coarse(const vs_ivfpq* ix, const float* q, int64_t nq, int32_t nprobe,
                    int32_t* probes, float* coarse_dist, void* hip_stream) {
  if (!ix) return fail(VS_ERR_INVALID_ARG, "vs_ivfpq_coarse: index is null");
  if (nq < 0) return fail(VS_ERR_INVALID_ARG, "vs_ivfpq_coarse: nq < 0");
  if (nprobe < 1 || nprobe > VS_MAX_K) return fail(VS_ERR_INVALID_ARG, "vs_ivfpq_coarse: nprobe = %d outside [1, %d]", nprobe, VS_MAX_K);
  if (nq == 0) return VS_OK;
  if (!q || !probes) return fail(VS_ERR_INVALID_ARG, "vs_ivfpq_coarse: null pointer");
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int npr = std::min<int>(nprobe, ix->g.nlist);
  const KnnPlan plan = knn_plan(nq, ix->g.nlist, ix->g.d, npr, ix->has_planes);
  ScratchUse use(ix->scratch, st);
  if (int rc = ix->scratch.reserve(plan.bytes)) return rc;
  if (int rc = coarse_select(ix, plan, static_cast<char*>(ix->scratch.p), q, nq, npr, probes, coarse_dist, st)) return rc;
  HIP_TRY(hipGetLastError());
  return VS_OK;
}

namespace {

// Work space of one search, carved from one buffer.
struct SearchLayout {
  int npr = 0, nsplit = 1;
  KnnPlan plan;
  size_t o_knn = 0, o_pr = 0, o_cd = 0, o_part = 0, o_cnt = 0, o_qt = 0, o_lm = 0, bytes = 0;
  bool query_tables = false;
  bool list_major = false;      // the scan runs list-major (see ivfpq_scan_listmajor_kernel)
  int lm_first = 0, lm_cap = 0;
};
void search_layout(const vs_ivfpq* ix, int64_t nq, int k, int nprobe, SearchLayout* out, bool allow_list_major = true) {
  SearchLayout& L = *out;
  const IvfpqDims& g = ix->g;
  L.npr = std::min<int>(nprobe, g.nlist);
  // probe splits: enough workgroups to fill the chip when nq is small
  L.nsplit = (int)std::min<int64_t>(L.npr, std::max<int64_t>(1, (4096 + nq - 1) / nq));
  // List-major scan: L2 with residual tables on the shapes of the bank-private kernel, when every
  // list is probed several times by the batch, the codes do not fit the caches anyway and the
  // lists are long (a list of one or two chunks leaves the list-major kernel, which builds two
  // tables and then scans, with nothing to overlap the builds with: measured slower at 244 codes).
  const int lm = g_list_major.load();
  const int first = std::min(g_lm_first.load(), L.npr - 1);
  const bool residual_tables = !(ix->search_type == VS_ST_STORED_NORMS && ix->norms) &&
                               !(ix->search_type == VS_ST_PRECOMPUTED_TABLES && ix->list_tables);
  if (allow_list_major && lm >= 0 && ivfpq_listmajor_shape(g) && residual_tables && first >= 1 &&
      ix->ntotal > 0 && nq * (int64_t)L.npr < (1ll << 32) &&
      (lm == 1 || (L.nsplit == 1 && L.npr >= 16 && nq * (int64_t)(L.npr - first) >= 3 * (int64_t)g.nlist &&
                   ix->ntotal * (int64_t)g.code_size >= (512ll << 20) && ix->ntotal >= 1024 * (int64_t)g.nlist))) {
    L.list_major = true;
    L.lm_first = first;
    L.lm_cap = g_lm_cap.load();
    L.nsplit = 1;
  }
  const int ppb = (L.npr + L.nsplit - 1) / L.nsplit;
  L.nsplit = (L.npr + ppb - 1) / ppb;
  L.plan = knn_plan(nq, g.nlist, g.d, L.npr, ix->has_planes);
  Carver cv;
  L.o_knn = cv.take(L.plan.bytes);
  L.o_pr = cv.take((size_t)nq * L.npr * sizeof(int32_t));
  L.o_cd = cv.take((size_t)nq * L.npr * sizeof(float));
  L.o_part = cv.take((size_t)nq * L.nsplit * k * sizeof(u64));
  L.o_cnt = cv.take(sizeof(u64));
  // (every table form but the residual tables: inner product, stored norms, precomputed tables)
  L.query_tables = ivfpq_wave_scan_applies(g, ix->ntotal) &&
                   (g.metric == VS_METRIC_IP || (ix->search_type == VS_ST_STORED_NORMS && ix->norms) ||
                    (ix->search_type == VS_ST_PRECOMPUTED_TABLES && ix->list_tables));
  if (L.query_tables) L.o_qt = cv.take(ivfpq_query_table_bytes(g, nq));
  if (L.list_major) L.o_lm = cv.take(ivfpq_listmajor_bytes(g, nq, L.npr, L.lm_cap));
  L.bytes = cv.off;
}

int search_check_args(const char* who, const vs_ivfpq* ix, const float* q, int64_t nq, int32_t k,
                      int32_t nprobe, const float* out_dist, const int64_t* out_ids) {
  if (!ix) return fail(VS_ERR_INVALID_ARG, "%s: index is null", who);
  if (nq < 0) return fail(VS_ERR_INVALID_ARG, "%s: nq < 0", who);
  if (k < 1 || k > VS_MAX_K) return fail(VS_ERR_INVALID_ARG, "%s: k = %d outside [1, %d]", who, k, VS_MAX_K);
  if (nprobe < 1 || nprobe > VS_MAX_K) return fail(VS_ERR_INVALID_ARG, "%s: nprobe = %d outside [1, %d]", who, nprobe, VS_MAX_K);
  if (nq > 0 && (!q || !out_dist || !out_ids)) return fail(VS_ERR_INVALID_ARG, "%s: null pointer", who);
  return VS_OK;
}

// The search itself on a work space of L.bytes at `base`: kernel launches only.
int search_run(const char* who, const vs_ivfpq* ix, const SearchLayout& L, char* base, const float* q,
               int64_t nq, int k, float* out_dist, int64_t* out_ids, hipStream_t st, bool timed,
               vs_search_stats* stats = nullptr) {
  const IvfpqDims& g = ix->g;
  int32_t* probes = reinterpret_cast<int32_t*>(base + L.o_pr);
  float* cdist = reinterpret_cast<float*>(base + L.o_cd);
  u64* partial = reinterpret_cast<u64*>(base + L.o_part);
  u64* counter = reinterpret_cast<u64*>(base + L.o_cnt);
  const int* fallback_count = nullptr;
  if (int rc = coarse_select(ix, L.plan, base + L.o_knn, q, nq, L.npr, probes, cdist, st, timed, &fallback_count))
    return rc;
  // an inner-product index that chooses its lists by L2: the scan's per-list term is <q, c_l>,
  // not the L2 distance the coarse quantizer returned
  if (g.metric == VS_METRIC_IP && coarse_metric_of(ix) == VS_METRIC_L2)
    launch_probe_inner_products(q, nq, g.d, ix->centroids, probes, L.npr, cdist, st);
  if (stats)
    launch_search_stats(probes, nq * L.npr, ix->list_off, fallback_count, L.plan.mfma ? nq : 0, L.npr,
                        L.list_major ? L.lm_first : 0, reinterpret_cast<long long*>(stats), st);
  // search type "stored norms": the per-(query, list) number is |q|^2 - 2 <q, c_l> = coarse
  // distance - |c_l|^2, and the scan adds the stored |x'|^2 of every code (Sec. 4.3)
  const bool with_norms = ix->search_type == VS_ST_STORED_NORMS && ix->norms;
  const bool split = ix->search_type == VS_ST_PRECOMPUTED_TABLES && ix->list_tables;
  bool scanned = false;
  if (L.list_major) {   // (where its selection state does not fit the LDS: the query-major scan below)
    auto part = [&](int which) {
      return launch_ivfpq_scan_listmajor(which, g, q, nq, ix->centroids, ix->codebooks, probes, cdist, L.npr,
                                         L.lm_first, L.lm_cap, ix->list_off, ix->codes, ix->ntotal, k, partial,
                                         counter, base + L.o_lm, ix->ids, out_dist, out_ids, st);
    };
    {
      StageTimer t(timed ? VS_STAGE_SCAN_FIRST : -1, st);
      scanned = part(0) == 0;
    }
    if (scanned) {
      {
        StageTimer t(timed ? VS_STAGE_SCAN : -1, st);
        (void)part(1);
      }
      StageTimer t(timed ? VS_STAGE_MERGE : -1, st);
      (void)part(2);
      if (stats)
        launch_search_stats_rescan(ivfpq_listmajor_rescan_count(g, nq, L.npr, L.lm_cap, base + L.o_lm),
                                   reinterpret_cast<long long*>(stats), st);
    }
  }
  if (!scanned) {
    StageTimer t(timed ? VS_STAGE_SCAN : -1, st);
    if (launch_ivfpq_scan(g, q, nq, ix->centroids, ix->codebooks, probes, cdist, L.npr, L.nsplit,
                          ix->list_off, ix->codes, with_norms ? ix->norms : nullptr, ix->cnorm,
                          split ? ix->list_tables : nullptr,
                          L.query_tables ? reinterpret_cast<float*>(base + L.o_qt) : nullptr, ix->ntotal, k,
                          partial, counter, ix->ids,
                          out_dist, out_ids, st) != 0)
      return fail(VS_ERR_UNSUPPORTED, "%s: look-up tables of M * 2^nbits = %d floats plus selection state for k = %d exceed the LDS", who, g.M * g.K, k);
  }
  if (L.nsplit > 1) {
    StageTimer t(timed ? VS_STAGE_MERGE : -1, st);
    launch_ivfpq_merge(partial, nq, L.nsplit, k, g.metric, ix->ids, out_dist, out_ids, st);
  }
  HIP_TRY(hipGetLastError());
  return VS_OK;
}

}  // namespace

int vs_ivfpq_search(const vs_ivfpq* ix, const float* q, int64_t nq, int32_t k, int32_t nprobe,
                    float* out_dist, int64_t* out_ids, void* hip_stream) {
  if (int rc = search_check_args("vs_ivfpq_search", ix, q, nq, k, nprobe, out_dist, out_ids)) return rc;
  if (nq == 0) return VS_OK;
  SearchLayout L;
  search_layout(ix, nq, k, nprobe, &L);
  ScratchUse use(ix->scratch, static_cast<hipStream_t>(hip_stream));
  if (int rc = ix->scratch.reserve(L.bytes)) return rc;
  return search_run("vs_ivfpq_search", ix, L, static_cast<char*>(ix->scratch.p), q, nq, k, out_dist, out_ids,
                    static_cast<hipStream_t>(hip_stream), true);
}

int vs_ivfpq_search_stats(const vs_ivfpq* ix, const float* q, int64_t nq, int32_t k, int32_t nprobe,
                          float* out_dist, int64_t* out_ids, vs_search_stats* stats, void* hip_stream) {
  if (int rc = search_check_args("vs_ivfpq_search_stats", ix, q, nq, k, nprobe, out_dist, out_ids)) return rc;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (nq == 0) {
    if (stats) launch_fill_u64(reinterpret_cast<u64*>(stats), sizeof(vs_search_stats) / sizeof(u64), 0ull, st);
    return VS_OK;
  }
  SearchLayout L;
  search_layout(ix, nq, k, nprobe, &L);
  ScratchUse use(ix->scratch, st);
  if (int rc = ix->scratch.reserve(L.bytes)) return rc;
  return search_run("vs_ivfpq_search_stats", ix, L, static_cast<char*>(ix->scratch.p), q, nq, k, out_dist, out_ids,
                    st, true, stats);
}

int vs_ivfpq_search_static(const vs_ivfpq* ix, const float* q, int64_t nq, int32_t k, int32_t nprobe,
                           float* out_dist, int64_t* out_ids, void* hip_stream) {
  if (int rc = search_check_args("vs_ivfpq_search_static", ix, q, nq, k, nprobe, out_dist, out_ids)) return rc;
  if (nq == 0) return VS_OK;
  SearchLayout L;
  search_layout(ix, nq, k, nprobe, &L, false);   // (the list-major scan's buffers are not for a fixed work space)
  if (L.bytes > kStaticScratchBytes)
    return fail(VS_ERR_INVALID_ARG,
                "vs_ivfpq_search_static: %lld queries with k = %d, nprobe = %d need %zu bytes of work space, "
                "the static buffer holds %zu; search fewer queries per call or use vs_ivfpq_search",
                (long long)nq, k, nprobe, L.bytes, kStaticScratchBytes);
  char* base = nullptr;
  if (int rc = static_scratch(&base)) return rc;
  return search_run("vs_ivfpq_search_static", ix, L, base, q, nq, k, out_dist, out_ids,
                    static_cast<hipStream_t>(hip_stream), false);
}

// ---- IVF-Flat: the same inverted lists with the vectors stored as they are --------------
// (core.codes holds the rows [ntotal, d] fp32, core.g.code_size = 4 d, no codebooks)

int vs_ivfflat_create(vs_ivfflat** out, int32_t d, int32_t metric, int32_t nlist,
                      const float* centroids, void* hip_stream) {
  if (!out) return fail(VS_ERR_INVALID_ARG, "vs_ivfflat_create: out is null");
  *out = nullptr;
  if (!centroids) return fail(VS_ERR_INVALID_ARG, "vs_ivfflat_create: null pointer");
  if (d < 1 || nlist < 1) return fail(VS_ERR_INVALID_ARG, "vs_ivfflat_create: d, nlist must be >= 1");
  if (metric != VS_METRIC_L2 && metric != VS_METRIC_IP) return fail(VS_ERR_INVALID_ARG, "vs_ivfflat_create: unknown metric %d", metric);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  vs_ivfflat* fx = new (std::nothrow) vs_ivfflat();
  if (!fx) return fail(VS_ERR_OOM, "vs_ivfflat_create: host allocation failed");
  vs_ivfpq* ix = &fx->core;
  ix->g.d = d; ix->g.metric = metric; ix->g.nlist = nlist; ix->g.M = 0; ix->g.nbits = 0;
  ix->g.K = 0; ix->g.dsub = 0; ix->g.code_size = d * (int)sizeof(float);
  ix->h_off.assign((size_t)nlist + 1, 0);
  auto cleanup = [&](int rc) { vs_ivfflat_destroy(fx); return rc; };
#define TRY_C(expr)                                                                         \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess)                                                                   \
      return cleanup(fail(e_ == hipErrorOutOfMemory ? VS_ERR_OOM : VS_ERR_DEVICE, "%s: %s", \
                          #expr, hipGetErrorString(e_)));                                   \
  } while (0)
  TRY_C(hipGetDevice(&ix->device));
  const size_t cb = (size_t)nlist * d * sizeof(float);
  TRY_C(hipMalloc(reinterpret_cast<void**>(&ix->centroids), cb));
  TRY_C(hipMalloc(reinterpret_cast<void**>(&ix->list_off), ((size_t)nlist + 1) * sizeof(int64_t)));
  TRY_C(hipMemcpyAsync(ix->centroids, centroids, cb, hipMemcpyDeviceToDevice, st));
  TRY_C(hipMemsetAsync(ix->list_off, 0, ((size_t)nlist + 1) * sizeof(int64_t), st));
  if (mfma_knn_supported(d, 1)) {
    TRY_C(hipMalloc(&ix->plane_mem, planes_bytes(nlist, d)));
    ix->c_planes = carve_planes(static_cast<char*>(ix->plane_mem), nlist, d);
    launch_prep(ix->centroids, nlist, d, ix->c_planes.hi, ix->c_planes.lo, ix->c_planes.norm,
                ix->c_planes.info, st, true);
    ix->c_planes.try_heads_only = true;
    ix->has_planes = true;
  }
  TRY_C(hipStreamSynchronize(st));
  if (ix->has_planes) TRY_C(learn_planes(&ix->c_planes));
#undef TRY_C
  *out = fx;
  return VS_OK;
}

void vs_ivfflat_destroy(vs_ivfflat* fx) {
  if (!fx) return;
  ivf_free_device_memory(&fx->core);
  delete fx;
}

int64_t vs_ivfflat_ntotal(const vs_ivfflat* fx) { return fx ? fx->core.ntotal : -1; }

int vs_ivfflat_add(vs_ivfflat* fx, const float* x, int64_t n, const int64_t* ids, void* hip_stream) {
  if (!fx) return fail(VS_ERR_INVALID_ARG, "vs_ivfflat_add: index is null");
  if (n < 0) return fail(VS_ERR_INVALID_ARG, "vs_ivfflat_add: n < 0");
  if (n == 0) return VS_OK;
  if (!x) return fail(VS_ERR_INVALID_ARG, "vs_ivfflat_add: x is null");
  vs_ivfpq* ix = &fx->core;
  if (ix->ntotal + n >= (1ll << 32)) return fail(VS_ERR_UNSUPPORTED, "vs_ivfflat_add: more than 2^32 - 1 stored vectors");
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const IvfpqDims& g = ix->g;
  Placement pl;
  if (int rc = ivf_assign_and_place(ix, x, n, 0, &pl, st, "vs_ivfflat_add")) return rc;
  const int64_t total = ix->ntotal + n;
  uint8_t* rows = nullptr;
  int64_t* new_ids = nullptr;
  HIP_TRY(hipMalloc(reinterpret_cast<void**>(&rows), (size_t)total * g.code_size));
  if (hipMalloc(reinterpret_cast<void**>(&new_ids), (size_t)total * sizeof(int64_t)) != hipSuccess) {
    (void)hipFree(rows);
    return fail(VS_ERR_OOM, "vs_ivfflat_add: id storage allocation failed");
  }
  launch_ivfflat_relayout(g.d, g.nlist, reinterpret_cast<const float*>(ix->codes), ix->ids, ix->ntotal,
                          ix->list_off, pl.new_off, x, ids, ix->ntotal, pl.dest, n,
                          reinterpret_cast<float*>(rows), new_ids, st);
  return ivf_commit_storage(ix, rows, new_ids, nullptr, total, &pl, st, "vs_ivfflat_add");
}

int vs_ivfflat_search(const vs_ivfflat* fx, const float* q, int64_t nq, int32_t k, int32_t nprobe,
                      float* out_dist, int64_t* out_ids, void* hip_stream) {
  if (!fx) return fail(VS_ERR_INVALID_ARG, "vs_ivfflat_search: index is null");
  if (nq < 0) return fail(VS_ERR_INVALID_ARG, "vs_ivfflat_search: nq < 0");
  if (k < 1 || k > VS_MAX_K) return fail(VS_ERR_INVALID_ARG, "vs_ivfflat_search: k = %d outside [1, %d]", k, VS_MAX_K);
  if (nprobe < 1 || nprobe > VS_MAX_K) return fail(VS_ERR_INVALID_ARG, "vs_ivfflat_search: nprobe = %d outside [1, %d]", nprobe, VS_MAX_K);
  if (nq == 0) return VS_OK;
  if (!q || !out_dist || !out_ids) return fail(VS_ERR_INVALID_ARG, "vs_ivfflat_search: null pointer");
  const vs_ivfpq* ix = &fx->core;
  const IvfpqDims& g = ix->g;
  if (ivfflat_scan_lds_bytes(g.d, k) > 160 * 1024)
    return fail(VS_ERR_UNSUPPORTED, "vs_ivfflat_search: d = %d with k = %d exceeds the LDS", g.d, k);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int npr = std::min<int>(nprobe, g.nlist);
  // probe splits: enough workgroups to fill the chip when nq is small
  int nsplit = (int)std::min<int64_t>(npr, std::max<int64_t>(1, (4096 + nq - 1) / nq));
  const int ppb = (npr + nsplit - 1) / nsplit;
  nsplit = (npr + ppb - 1) / ppb;
  const KnnPlan plan = knn_plan(nq, g.nlist, g.d, npr, ix->has_planes);
  Carver cv;
  const size_t o_knn = cv.take(plan.bytes);
  const size_t o_pr = cv.take((size_t)nq * npr * sizeof(int32_t));
  const size_t o_part = cv.take((size_t)nq * nsplit * k * sizeof(u64));
  ScratchUse use(ix->scratch, st);
  if (int rc = ix->scratch.reserve(cv.off)) return rc;
  char* base = static_cast<char*>(ix->scratch.p);
  int32_t* probes = reinterpret_cast<int32_t*>(base + o_pr);
  u64* partial = reinterpret_cast<u64*>(base + o_part);
  if (int rc = coarse_select(ix, plan, base + o_knn, q, nq, npr, probes, nullptr, st)) return rc;
  {
    StageTimer t(VS_STAGE_SCAN, st);
    launch_ivfflat_scan(g.d, g.metric, q, nq, probes, npr, nsplit, ix->list_off,
                        reinterpret_cast<const float*>(ix->codes), k, partial, ix->ids, out_dist,
                        out_ids, st);
  }
  if (nsplit > 1) {
    StageTimer t(VS_STAGE_MERGE, st);
    launch_ivfpq_merge(partial, nq, nsplit, k, g.metric, ix->ids, out_dist, out_ids, st);
  }
  HIP_TRY(hipGetLastError());
  return VS_OK;
}

int vs_ivfflat_get_list_sizes(const vs_ivfflat* fx, int64_t* sizes, void* hip_stream) {
  if (!fx || !sizes) return fail(VS_ERR_INVALID_ARG, "vs_ivfflat_get_list_sizes: null pointer");
  launch_list_sizes(fx->core.list_off, fx->core.g.nlist, sizes, static_cast<hipStream_t>(hip_stream));
  HIP_TRY(hipGetLastError());
  return VS_OK;
}

int vs_ivfflat_get_storage(const vs_ivfflat* fx, int64_t* ids, int32_t* list_of, float* rows,
                           void* hip_stream) {
  if (!fx) return fail(VS_ERR_INVALID_ARG, "vs_ivfflat_get_storage: index is null");
  const vs_ivfpq* ix = &fx->core;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (ix->ntotal == 0) return VS_OK;
  if (ids) HIP_TRY(hipMemcpyAsync(ids, ix->ids, (size_t)ix->ntotal * sizeof(int64_t), hipMemcpyDeviceToDevice, st));
  if (list_of) launch_list_of_storage(ix->list_off, ix->g.nlist, ix->ntotal, list_of, st);
  if (rows) HIP_TRY(hipMemcpyAsync(rows, ix->codes, (size_t)ix->ntotal * ix->g.code_size, hipMemcpyDeviceToDevice, st));
  HIP_TRY(hipGetLastError());
  return VS_OK;
}

// ---- IVF-SQ8 ---------------------------------------------------------------------------

int vs_ivfsq8_create(vs_ivfsq8** out, int32_t d, int32_t metric, int32_t nlist,
                     const float* centroids, const float* vmin, const float* step,
                     void* hip_stream) {
  if (!out) return fail(VS_ERR_INVALID_ARG, "vs_ivfsq8_create: out is null");
  *out = nullptr;
  if (!centroids || !vmin || !step) return fail(VS_ERR_INVALID_ARG, "vs_ivfsq8_create: null pointer");
  if (d < 1 || nlist < 1) return fail(VS_ERR_INVALID_ARG, "vs_ivfsq8_create: d, nlist must be >= 1");
  if (metric != VS_METRIC_L2 && metric != VS_METRIC_IP) return fail(VS_ERR_INVALID_ARG, "vs_ivfsq8_create: unknown metric %d", metric);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  vs_ivfsq8* sx = new (std::nothrow) vs_ivfsq8();
  if (!sx) return fail(VS_ERR_OOM, "vs_ivfsq8_create: host allocation failed");
  vs_ivfpq* ix = &sx->core;
  ix->g.d = d; ix->g.metric = metric; ix->g.nlist = nlist; ix->g.M = d; ix->g.nbits = 8;
  ix->g.K = 0; ix->g.dsub = 0; ix->g.code_size = d;
  ix->h_off.assign((size_t)nlist + 1, 0);
  auto cleanup = [&](int rc) { vs_ivfsq8_destroy(sx); return rc; };
#define TRY_C(expr)                                                                         \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess)                                                                   \
      return cleanup(fail(e_ == hipErrorOutOfMemory ? VS_ERR_OOM : VS_ERR_DEVICE, "%s: %s", \
                          #expr, hipGetErrorString(e_)));                                   \
  } while (0)
  TRY_C(hipGetDevice(&ix->device));
  const size_t cb = (size_t)nlist * d * sizeof(float), pb = (size_t)d * sizeof(float);
  TRY_C(hipMalloc(reinterpret_cast<void**>(&ix->centroids), cb));
  TRY_C(hipMalloc(reinterpret_cast<void**>(&ix->list_off), ((size_t)nlist + 1) * sizeof(int64_t)));
  TRY_C(hipMalloc(reinterpret_cast<void**>(&sx->vmin), pb));
  TRY_C(hipMalloc(reinterpret_cast<void**>(&sx->step), pb));
  TRY_C(hipMemcpyAsync(ix->centroids, centroids, cb, hipMemcpyDeviceToDevice, st));
  TRY_C(hipMemcpyAsync(sx->vmin, vmin, pb, hipMemcpyDeviceToDevice, st));
  TRY_C(hipMemcpyAsync(sx->step, step, pb, hipMemcpyDeviceToDevice, st));
  TRY_C(hipMemsetAsync(ix->list_off, 0, ((size_t)nlist + 1) * sizeof(int64_t), st));
  if (mfma_knn_supported(d, 1)) {
    TRY_C(hipMalloc(&ix->plane_mem, planes_bytes(nlist, d)));
    ix->c_planes = carve_planes(static_cast<char*>(ix->plane_mem), nlist, d);
    launch_prep(ix->centroids, nlist, d, ix->c_planes.hi, ix->c_planes.lo, ix->c_planes.norm,
                ix->c_planes.info, st, true);
    ix->c_planes.try_heads_only = true;
    ix->has_planes = true;
  }
  TRY_C(hipStreamSynchronize(st));
  if (ix->has_planes) TRY_C(learn_planes(&ix->c_planes));
#undef TRY_C
  *out = sx;
  return VS_OK;
}

void vs_ivfsq8_destroy(vs_ivfsq8* sx) {
  if (!sx) return;
  ivf_free_device_memory(&sx->core);
  if (sx->vmin) (void)hipFree(sx->vmin);
  if (sx->step) (void)hipFree(sx->step);
  delete sx;
}

int64_t vs_ivfsq8_ntotal(const vs_ivfsq8* sx) { return sx ? sx->core.ntotal : -1; }

int vs_ivfsq8_add(vs_ivfsq8* sx, const float* x, int64_t n, const int64_t* ids, void* hip_stream) {
  if (!sx) return fail(VS_ERR_INVALID_ARG, "vs_ivfsq8_add: index is null");
  if (n < 0) return fail(VS_ERR_INVALID_ARG, "vs_ivfsq8_add: n < 0");
  if (n == 0) return VS_OK;
  if (!x) return fail(VS_ERR_INVALID_ARG, "vs_ivfsq8_add: x is null");
  vs_ivfpq* ix = &sx->core;
  if (ix->ntotal + n >= (1ll << 32)) return fail(VS_ERR_UNSUPPORTED, "vs_ivfsq8_add: more than 2^32 - 1 stored vectors");
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const IvfpqDims& g = ix->g;
  Placement pl;
  if (int rc = ivf_assign_and_place(ix, x, n, (size_t)n * g.d, &pl, st, "vs_ivfsq8_add")) return rc;
  uint8_t* tmp_codes = reinterpret_cast<uint8_t*>(pl.extra);
  launch_sq8_encode(x, n, g.d, sx->vmin, sx->step, tmp_codes, st);
  const int64_t total = ix->ntotal + n;
  uint8_t* codes = nullptr;
  int64_t* new_ids = nullptr;
  HIP_TRY(hipMalloc(reinterpret_cast<void**>(&codes), (size_t)total * g.code_size));
  if (hipMalloc(reinterpret_cast<void**>(&new_ids), (size_t)total * sizeof(int64_t)) != hipSuccess) {
    (void)hipFree(codes);
    return fail(VS_ERR_OOM, "vs_ivfsq8_add: id storage allocation failed");
  }
  launch_relayout(g, ix->codes, ix->ids, nullptr, ix->ntotal, ix->list_off, pl.new_off, tmp_codes,
                  ids, ix->ntotal, nullptr, pl.dest, pl.list_of, n, codes, new_ids, nullptr, st);
  return ivf_commit_storage(ix, codes, new_ids, nullptr, total, &pl, st, "vs_ivfsq8_add");
}

int vs_ivfsq8_search(const vs_ivfsq8* sx, const float* q, int64_t nq, int32_t k, int32_t nprobe,
                     float* out_dist, int64_t* out_ids, void* hip_stream) {
  if (!sx) return fail(VS_ERR_INVALID_ARG, "vs_ivfsq8_search: index is null");
  if (nq < 0) return fail(VS_ERR_INVALID_ARG, "vs_ivfsq8_search: nq < 0");
  if (k < 1 || k > VS_MAX_K) return fail(VS_ERR_INVALID_ARG, "vs_ivfsq8_search: k = %d outside [1, %d]", k, VS_MAX_K);
  if (nprobe < 1 || nprobe > VS_MAX_K) return fail(VS_ERR_INVALID_ARG, "vs_ivfsq8_search: nprobe = %d outside [1, %d]", nprobe, VS_MAX_K);
  if (nq == 0) return VS_OK;
  if (!q || !out_dist || !out_ids) return fail(VS_ERR_INVALID_ARG, "vs_ivfsq8_search: null pointer");
  const vs_ivfpq* ix = &sx->core;
  const IvfpqDims& g = ix->g;
  if (ivfsq8_scan_lds_bytes(g.d, k) > 160 * 1024)
    return fail(VS_ERR_UNSUPPORTED, "vs_ivfsq8_search: d = %d with k = %d exceeds the LDS", g.d, k);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int npr = std::min<int>(nprobe, g.nlist);
  int nsplit = (int)std::min<int64_t>(npr, std::max<int64_t>(1, (4096 + nq - 1) / nq));
  const int ppb = (npr + nsplit - 1) / nsplit;
  nsplit = (npr + ppb - 1) / ppb;
  const KnnPlan plan = knn_plan(nq, g.nlist, g.d, npr, ix->has_planes);
  Carver cv;
  const size_t o_knn = cv.take(plan.bytes);
  const size_t o_pr = cv.take((size_t)nq * npr * sizeof(int32_t));
  const size_t o_part = cv.take((size_t)nq * nsplit * k * sizeof(u64));
  ScratchUse use(ix->scratch, st);
  if (int rc = ix->scratch.reserve(cv.off)) return rc;
  char* base = static_cast<char*>(ix->scratch.p);
  int32_t* probes = reinterpret_cast<int32_t*>(base + o_pr);
  u64* partial = reinterpret_cast<u64*>(base + o_part);
  if (int rc = coarse_select(ix, plan, base + o_knn, q, nq, npr, probes, nullptr, st)) return rc;
  {
    StageTimer t(VS_STAGE_SCAN, st);
    launch_ivfsq8_scan(g.d, g.metric, q, nq, sx->vmin, sx->step, probes, npr, nsplit, ix->list_off,
                       ix->codes, k, partial, ix->ids, out_dist, out_ids, st);
  }
  if (nsplit > 1) {
    StageTimer t(VS_STAGE_MERGE, st);
    launch_ivfpq_merge(partial, nq, nsplit, k, g.metric, ix->ids, out_dist, out_ids, st);
  }
  HIP_TRY(hipGetLastError());
  return VS_OK;
}

int vs_ivfsq8_get_list_sizes(const vs_ivfsq8* sx, int64_t* sizes, void* hip_stream) {
  if (!sx || !sizes) return fail(VS_ERR_INVALID_ARG, "vs_ivfsq8_get_list_sizes: null pointer");
  launch_list_sizes(sx->core.list_off, sx->core.g.nlist, sizes, static_cast<hipStream_t>(hip_stream));
  HIP_TRY(hipGetLastError());
  return VS_OK;
}

int vs_ivfsq8_get_storage(const vs_ivfsq8* sx, int64_t* ids, int32_t* list_of, uint8_t* codes,
                          void* hip_stream) {
  if (!sx) return fail(VS_ERR_INVALID_ARG, "vs_ivfsq8_get_storage: index is null");
  const vs_ivfpq* ix = &sx->core;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (ix->ntotal == 0) return VS_OK;
  if (ids) HIP_TRY(hipMemcpyAsync(ids, ix->ids, (size_t)ix->ntotal * sizeof(int64_t), hipMemcpyDeviceToDevice, st));
  if (list_of) launch_list_of_storage(ix->list_off, ix->g.nlist, ix->ntotal, list_of, st);
  if (codes) HIP_TRY(hipMemcpyAsync(codes, ix->codes, (size_t)ix->ntotal * ix->g.code_size, hipMemcpyDeviceToDevice, st));
  HIP_TRY(hipGetLastError());
  return VS_OK;
}

int vs_ivfpq_get_list_sizes(const vs_ivfpq* ix, int64_t* sizes, void* hip_stream) {
  if (!ix || !sizes) return fail(VS_ERR_INVALID_ARG, "vs_ivfpq_get_list_sizes: null pointer");
  launch_list_sizes(ix->list_off, ix->g.nlist, sizes, static_cast<hipStream_t>(hip_stream));
  HIP_TRY(hipGetLastError());
  return VS_OK;
}

int vs_ivfpq_get_assignments(const vs_ivfpq* ix, int64_t* ids, int32_t* list_of,
                             void* hip_stream) {
  if (!ix) return fail(VS_ERR_INVALID_ARG, "vs_ivfpq_get_assignments: index is null");
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (ix->ntotal == 0) return VS_OK;
  if (ids) HIP_TRY(hipMemcpyAsync(ids, ix->ids, (size_t)ix->ntotal * sizeof(int64_t), hipMemcpyDeviceToDevice, st));
  if (list_of) launch_list_of_storage(ix->list_off, ix->g.nlist, ix->ntotal, list_of, st);
  HIP_TRY(hipGetLastError());
  return VS_OK;
}

int vs_ivfpq_get_codes(const vs_ivfpq* ix, uint8_t* codes, void* hip_stream) {
  if (!ix || !codes) return fail(VS_ERR_INVALID_ARG, "vs_ivfpq_get_codes: null pointer");
  if (ix->ntotal == 0) return VS_OK;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (ivfpq_codes_rotated(ix->g)) {   // the store keeps these shapes' codes rotated for the scan
    launch_codes_canonical(ix->g, ix->codes, ix->list_off, ix->ntotal, codes, st);
    HIP_TRY(hipGetLastError());
    return VS_OK;
  }
  HIP_TRY(hipMemcpyAsync(codes, ix->codes, (size_t)ix->ntotal * ix->g.code_size, hipMemcpyDeviceToDevice, st));
  return VS_OK;
}

}  // extern "C"
