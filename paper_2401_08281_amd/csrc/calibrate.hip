// Calibration kernels for the benchmark (not part of libvs.so): what this GPU reaches on the two
// resources the search kernels are priced against, measured in the same process as the benchmark,
// and a copy kernel of known size under a name of its own for the HBM traffic counters.
//   vsc_read_stream   a read-only stream over a buffer larger than every cache (HBM read rate)
//   vsc_mfma_loop     back-to-back v_mfma_f32_32x32x16_bf16 on registers (matrix-core issue rate)
//   vsc_copy          dst = src, one 16-byte load and store per thread and step
// Built into libvs_calibrate.so; plain C entry points, device pointers, HIP events for the timing.
#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

namespace {

// A workgroup reads 32 KB of consecutive memory per step (eight 16-byte non-temporal loads per
// thread, all requested before the first is used) and the grid walks the buffer front to back: the
// fastest of the read patterns tried on this chip.  `sink` is written only if the data xor to a
// value that the host chose not to be there, so the loads cannot be dropped and nothing is stored.
__global__ __launch_bounds__(256) void vs_calibrate_read_kernel(const u32x4* __restrict__ src, size_t n16,
                                                                unsigned magic, unsigned* __restrict__ sink) {
  constexpr int U = 8;
  const size_t span = (size_t)256 * U;
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (size_t b = (size_t)blockIdx.x * span; b + span <= n16; b += (size_t)gridDim.x * span) {
    u32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(src + b + u * 256 + threadIdx.x);
#pragma unroll
    for (int u = 0; u < U; ++u) acc ^= v[u];
  }
  const unsigned v = acc.x ^ acc.y ^ acc.z ^ acc.w;
  if (v == magic) sink[0] = v;
}

__global__ __launch_bounds__(256) void vs_calibrate_copy_kernel(const u32x4* __restrict__ src,
                                                                u32x4* __restrict__ dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// Four independent accumulator tiles per wavefront, so that an instruction never waits for the
// one before it; operands are register constants.  2 * 32 * 32 * 16 flop per instruction.
__global__ __launch_bounds__(256) void vs_calibrate_mfma_kernel(int iters, float* __restrict__ out) {
  bf16x8 a, b;
  for (int i = 0; i < 8; ++i) {
    a[i] = (__bf16)(float)((threadIdx.x + i) & 7);
    b[i] = (__bf16)(float)((threadIdx.x * 3 + i) & 3);
  }
  floatx16 c0 = {}, c1 = {}, c2 = {}, c3 = {};
  for (int it = 0; it < iters; ++it) {
    c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
    c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
    c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
    c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
  }
  float s = 0.f;
  for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
  out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

struct Events {
  hipEvent_t a = nullptr, b = nullptr;
  bool ok = false;
  Events() { ok = hipEventCreate(&a) == hipSuccess && hipEventCreate(&b) == hipSuccess; }
  ~Events() {
    if (a) (void)hipEventDestroy(a);
    if (b) (void)hipEventDestroy(b);
  }
};

}  // namespace

extern "C" {

// dst = src (device pointers, bytes a multiple of 16), enqueued on `stream`.  0, or -1 on bad arguments.
__attribute__((visibility("default"))) int vsc_copy(const void* src, void* dst, size_t bytes, void* stream) {
  if (!src || !dst || bytes % 16 != 0) return -1;
  hipLaunchKernelGGL(vs_calibrate_copy_kernel, dim3(256 * 8), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const u32x4*>(src), static_cast<u32x4*>(dst), bytes / 16);
  return hipGetLastError() == hipSuccess ? 0 : -2;
}

// Reads `bytes` (a multiple of 32 KB) at src `iters` times after one untimed pass; *gbs = 1e-9 *
// bytes * iters / seconds between two events on `stream`.  sink: one device word (never written
// unless the data xor to `magic`).  Synchronises the stream.
__attribute__((visibility("default"))) int vsc_read_stream(const void* src, size_t bytes, int iters,
                                                           unsigned* sink, double* gbs, void* stream) {
  if (!src || !sink || !gbs || bytes % (32 * 1024) != 0 || bytes == 0 || iters < 1) return -1;
  hipStream_t st = static_cast<hipStream_t>(stream);
  Events ev;
  if (!ev.ok) return -2;
  const unsigned magic = 0x9e3779b9u;
  auto go = [&] {
    hipLaunchKernelGGL(vs_calibrate_read_kernel, dim3(256 * 8), dim3(256), 0, st, static_cast<const u32x4*>(src),
                       bytes / 16, magic, sink);
  };
  go();
  if (hipEventRecord(ev.a, st) != hipSuccess) return -2;
  for (int i = 0; i < iters; ++i) go();
  if (hipEventRecord(ev.b, st) != hipSuccess || hipEventSynchronize(ev.b) != hipSuccess) return -2;
  float ms = 0.f;
  if (hipEventElapsedTime(&ms, ev.a, ev.b) != hipSuccess || ms <= 0.f) return -2;
  *gbs = 1e-9 * (double)bytes * iters / (ms * 1e-3);
  return 0;
}

// 256 CUs x 2 workgroups of 4 wavefronts, each 4 * iters matrix instructions; *tflops from the
// time of three launches after one untimed.  out: device, 256 * 2 * 256 floats.  Synchronises.
__attribute__((visibility("default"))) int vsc_mfma_loop(int iters, float* out, double* tflops, void* stream) {
  if (!out || !tflops || iters < 1) return -1;
  hipStream_t st = static_cast<hipStream_t>(stream);
  Events ev;
  if (!ev.ok) return -2;
  const int blocks = 256 * 2, launches = 3;
  auto go = [&] { hipLaunchKernelGGL(vs_calibrate_mfma_kernel, dim3(blocks), dim3(256), 0, st, iters, out); };
  go();
  if (hipEventRecord(ev.a, st) != hipSuccess) return -2;
  for (int i = 0; i < launches; ++i) go();
  if (hipEventRecord(ev.b, st) != hipSuccess || hipEventSynchronize(ev.b) != hipSuccess) return -2;
  float ms = 0.f;
  if (hipEventElapsedTime(&ms, ev.a, ev.b) != hipSuccess || ms <= 0.f) return -2;
  const double flop = 2.0 * 32 * 32 * 16 * 4.0 * iters * 4.0 /*wavefronts*/ * blocks * launches;
  *tflops = 1e-12 * flop / (ms * 1e-3);
  return 0;
}

}  // extern "C"
