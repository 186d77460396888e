// Machine probes: what this GPU sustains on the two resources the step's kernels are
// judged against, measured with the same compiler and launch path as the kernels.
//   kv_probe_mfma_bf16 : a register-resident loop of v_mfma_f32_32x32x16_bf16 on every SIMD
//                        (no memory traffic, four independent accumulators per wave),
//   kv_probe_copy      : a streaming device-to-device copy of a given size, which is also
//                        the known-size launch that HBM byte counters are scaled by.
// Both time their launches with HIP events stamped by the runtime around the kernel.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include <algorithm>

#include "../../include/kvx.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kProbeThreads = 512;        // two waves per SIMD
constexpr int kProbeAccs = 4;

__global__ __launch_bounds__(kProbeThreads) void mfma_probe_kernel(float* out, int iters) {
  const int lane = threadIdx.x & 63;
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    // small values of both signs, different per lane and element, exact in bf16
    a[e] = (__bf16)(0.125f * (float)(((lane * 5 + e * 3) % 7) - 3));
    b[e] = (__bf16)(0.125f * (float)(((lane * 3 + e * 5 + (int)blockIdx.x) % 7) - 3));
  }
  f32x16 acc[kProbeAccs];
#pragma unroll
  for (int k = 0; k < kProbeAccs; ++k)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[k][e] = 0.f;
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int k = 0; k < kProbeAccs; ++k) acc[k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[k], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int k = 0; k < kProbeAccs; ++k)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += acc[k][e];
  out[(int64_t)blockIdx.x * kProbeThreads + threadIdx.x] = s;
}

// Each workgroup moves one contiguous 16 KiB piece: four 16-byte loads per lane in flight, then
// the four stores.  (Of the shapes tried - grid-stride loops with 2048 to 65536 workgroups, with
// and without non-temporal accesses, 32 KiB pieces, the runtime's own device-to-device copy - this
// one moved 1 to 4 GiB fastest on this machine.)
constexpr int kCopyUnroll = 4;
__global__ __launch_bounds__(256) void copy_probe_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, int64_t n16) {
  const int64_t base = (int64_t)blockIdx.x * (256 * kCopyUnroll) + threadIdx.x;
  uint4 v[kCopyUnroll];
#pragma unroll
  for (int u = 0; u < kCopyUnroll; ++u)
    if (base + u * 256 < n16) v[u] = src[base + u * 256];
#pragma unroll
  for (int u = 0; u < kCopyUnroll; ++u)
    if (base + u * 256 < n16) dst[base + u * 256] = v[u];
}

struct EventPair {
  hipEvent_t a = nullptr, b = nullptr;
  bool ok = false;
  EventPair() { ok = hipEventCreate(&a) == hipSuccess && hipEventCreate(&b) == hipSuccess; }
  ~EventPair() {
    if (a) hipEventDestroy(a);
    if (b) hipEventDestroy(b);
  }
};

}  // namespace

extern "C" {

int kv_probe_mfma_bf16(int32_t iters, int32_t repeats, void* hip_stream, double* tflops) {
  if (!tflops || iters < 1 || iters > (1 << 22) || repeats < 1 || repeats > 1024) return KV_E_INVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
    return KV_E_HIP;
  const int blocks = cus;                   // one workgroup of eight waves per compute unit
  float* out = nullptr;
  if (hipMalloc((void**)&out, (size_t)blocks * kProbeThreads * sizeof(float)) != hipSuccess) return KV_E_NOMEM;
  EventPair ev;
  int rc = ev.ok ? KV_OK : KV_E_HIP;
  double total_ms = 0.0, total_flops = 0.0;
  for (int r = 0; r < repeats + 1 && rc == KV_OK; ++r) {      // the first launch warms up
    hipExtLaunchKernelGGL(mfma_probe_kernel, dim3(blocks), dim3(kProbeThreads), 0, st, ev.a, ev.b, 0, out, (int)iters);
    float ms = 0.f;
    if (hipEventSynchronize(ev.b) != hipSuccess || hipEventElapsedTime(&ms, ev.a, ev.b) != hipSuccess || !(ms > 0.f)) {
      rc = KV_E_HIP;
      break;
    }
    if (r == 0) continue;
    const double flops = 2.0 * 32 * 32 * 16 * (double)kProbeAccs * iters * (kProbeThreads / 64) * blocks;
    total_ms += ms;
    total_flops += flops;
  }
  hipFree(out);
  *tflops = total_ms > 0.0 ? total_flops / (total_ms * 1e-3) / 1e12 : 0.0;
  return rc;
}

int kv_probe_copy(int64_t bytes, int32_t repeats, void* hip_stream, double* gbytes_per_s) {
  if (!gbytes_per_s || bytes < 4096 || bytes > (1ll << 34) || (bytes & 15) || repeats < 1 || repeats > 1024) return KV_E_INVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  uint4 *src = nullptr, *dst = nullptr;
  if (hipMalloc((void**)&src, (size_t)bytes) != hipSuccess) return KV_E_NOMEM;
  if (hipMalloc((void**)&dst, (size_t)bytes) != hipSuccess) {
    hipFree(src);
    return KV_E_NOMEM;
  }
  EventPair ev;
  int rc = ev.ok ? KV_OK : KV_E_HIP;
  if (rc == KV_OK && hipMemsetAsync(src, 0x5a, (size_t)bytes, st) != hipSuccess) rc = KV_E_HIP;
  const int64_t n16 = bytes / 16;
  const int blocks = (int)((n16 + 256 * kCopyUnroll - 1) / (256 * kCopyUnroll));      // <= 2^20 for 16 GiB
  double total_ms = 0.0;
  for (int r = 0; r < repeats + 1 && rc == KV_OK; ++r) {
    hipExtLaunchKernelGGL(copy_probe_kernel, dim3(blocks), dim3(256), 0, st, ev.a, ev.b, 0, (const uint4*)src, dst, n16);
    float ms = 0.f;
    if (hipEventSynchronize(ev.b) != hipSuccess || hipEventElapsedTime(&ms, ev.a, ev.b) != hipSuccess || !(ms > 0.f)) {
      rc = KV_E_HIP;
      break;
    }
    if (r == 0) continue;
    total_ms += ms;
  }
  hipFree(src);
  hipFree(dst);
  // bytes read + bytes written over the launches after the first
  *gbytes_per_s = total_ms > 0.0 ? 2.0 * (double)bytes * repeats / (total_ms * 1e-3) / 1e9 : 0.0;
  return rc;
}

}  // extern "C"
