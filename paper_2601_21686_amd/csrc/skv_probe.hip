// Measuring sticks, not part of the attention path; built into a library of their own (libskv_probe.so).
// First a kernel that only reads.  Every workgroup streams a
// contiguous slice with four 16-byte loads in flight per lane and writes nothing (one guarded store that never
// fires keeps the loads alive).  What it reaches is what this memory system gives a plain streaming read of
// that size; the range kernels are judged against it as well as against the published peak.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "skv_probe.h"

namespace skv {
namespace {

constexpr int kProbeThreads = 256;
constexpr int kProbeUnroll = 4;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// NT: streaming (non-temporal) loads, as the range kernels use them for rows that exceed the last-level cache.
template <bool NT>
__global__ __launch_bounds__(kProbeThreads) void stream_read_kernel(const u32x4* __restrict__ src, size_t per_wg,
                                                                  float* sink) {
  const u32x4* p = src + (size_t)blockIdx.x * per_wg;
  float acc = 0.f;
  for (size_t i = threadIdx.x; i < per_wg; i += kProbeThreads * kProbeUnroll) {   // per_wg is a multiple of the stride
    u32x4 v[kProbeUnroll];
#pragma unroll
    for (int u = 0; u < kProbeUnroll; ++u) {
      if constexpr (NT) v[u] = __builtin_nontemporal_load(p + i + (size_t)u * kProbeThreads);
      else v[u] = p[i + (size_t)u * kProbeThreads];
    }
#pragma unroll
    for (int u = 0; u < kProbeUnroll; ++u) acc += __uint_as_float(v[u].x ^ v[u].y ^ v[u].z ^ v[u].w);
  }
  if (acc == 12345.678f) sink[blockIdx.x] = acc;   // practically never: the sum of xor-ed words is not this value
}

// The same for a stream that reads two bytes for each byte it writes, the mix of the chunk append at
// ranks that add up to the head size: c = a ^ b over contiguous slices.
__global__ __launch_bounds__(kProbeThreads) void stream_mix_kernel(const uint4* __restrict__ a, const uint4* __restrict__ b,
                                                                 uint4* __restrict__ c, size_t per_wg) {
  const size_t base = (size_t)blockIdx.x * per_wg;
  for (size_t i = threadIdx.x; i < per_wg; i += kProbeThreads * kProbeUnroll) {   // per_wg is a multiple of the stride
    uint4 x[kProbeUnroll], y[kProbeUnroll];
#pragma unroll
    for (int u = 0; u < kProbeUnroll; ++u) {
      x[u] = a[base + i + (size_t)u * kProbeThreads];
      y[u] = b[base + i + (size_t)u * kProbeThreads];
    }
#pragma unroll
    for (int u = 0; u < kProbeUnroll; ++u)
      c[base + i + (size_t)u * kProbeThreads] = make_uint4(x[u].x ^ y[u].x, x[u].y ^ y[u].y, x[u].z ^ y[u].z, x[u].w ^ y[u].w);
  }
}

}  // namespace

}  // namespace skv

using namespace skv;

extern "C" {

skv_status skv_probe_stream_read(const void* src, size_t bytes, int32_t workgroups, int32_t streaming, void* sink,
                                 size_t* bytes_read, void* stream) {
  if (!src || !sink || !bytes_read) return SKV_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(src) & 15u) || (reinterpret_cast<uintptr_t>(sink) & 3u)) return SKV_ERR_ALIGN;
  if (workgroups < 1 || workgroups > 65535) return SKV_ERR_SHAPE;
  const size_t stride = (size_t)kProbeThreads * kProbeUnroll;        // 16-byte pieces one turn of the loop covers
  const size_t per_wg = bytes / 16 / (size_t)workgroups / stride * stride;
  if (per_wg == 0) return SKV_ERR_SHAPE;
  *bytes_read = per_wg * (size_t)workgroups * 16;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  if (streaming)
    hipLaunchKernelGGL(stream_read_kernel<true>, dim3((unsigned)workgroups), dim3(kProbeThreads), 0, hs,
                       static_cast<const u32x4*>(src), per_wg, static_cast<float*>(sink));
  else
    hipLaunchKernelGGL(stream_read_kernel<false>, dim3((unsigned)workgroups), dim3(kProbeThreads), 0, hs,
                       static_cast<const u32x4*>(src), per_wg, static_cast<float*>(sink));
  return hipGetLastError() == hipSuccess ? SKV_OK : SKV_ERR_HIP;
}

skv_status skv_probe_stream_mix(const void* a, const void* b, void* c, size_t bytes, int32_t workgroups,
                                size_t* bytes_each, void* stream) {
  if (!a || !b || !c || !bytes_each) return SKV_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b) | reinterpret_cast<uintptr_t>(c)) & 15u)
    return SKV_ERR_ALIGN;
  if (workgroups < 1 || workgroups > 65535) return SKV_ERR_SHAPE;
  const size_t stride = (size_t)kProbeThreads * kProbeUnroll;
  const size_t per_wg = bytes / 16 / (size_t)workgroups / stride * stride;
  if (per_wg == 0) return SKV_ERR_SHAPE;
  *bytes_each = per_wg * (size_t)workgroups * 16;
  hipLaunchKernelGGL(stream_mix_kernel, dim3((unsigned)workgroups), dim3(kProbeThreads), 0, static_cast<hipStream_t>(stream),
                     static_cast<const uint4*>(a), static_cast<const uint4*>(b), static_cast<uint4*>(c), per_wg);
  return hipGetLastError() == hipSuccess ? SKV_OK : SKV_ERR_HIP;
}

}  // extern "C"
