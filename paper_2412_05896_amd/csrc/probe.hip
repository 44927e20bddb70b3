// xkv_probe_stream_read: a plain streaming read of a device buffer, shaped like
// the attention kernels' K/V read (workgroups of 256 threads, each reading
// 128 KiB with 16-byte loads, all issued before any is used), optionally with a
// small record store per workgroup.  It computes nothing of the method: it
// exists so that the benchmark can quote, on the box it runs on, the read
// bandwidth a kernel of this shape can reach, next to what the path achieves.
#include <hip/hip_runtime.h>

#include "device_util.h"
#include "xkv_internal.h"

namespace xkv {
namespace {

constexpr int kProbeThreads = 256;
constexpr int kProbeLoads = 32;            // 16-byte loads per thread: 128 KiB per workgroup

// kStore: 0 ordinary stores, 1 non-temporal stores, 2 the library's system-scope stores.
template <bool kNonTemporal, int kStore>
__global__ __launch_bounds__(kProbeThreads) void probe_read(const uint4* __restrict__ src,
                                                            float* __restrict__ sink,
                                                            int store_floats, unsigned never) {
  const size_t base = static_cast<size_t>(blockIdx.x) * kProbeThreads * kProbeLoads;
  uint4 r[kProbeLoads];
#pragma unroll
  for (int i = 0; i < kProbeLoads; ++i) {
    const uint4* p = src + base + static_cast<size_t>(i) * kProbeThreads + threadIdx.x;
    r[i] = kNonTemporal ? load_stream16(p) : *p;
  }
  unsigned x = 0;
#pragma unroll
  for (int i = 0; i < kProbeLoads; ++i) x ^= r[i].x ^ r[i].y ^ r[i].z ^ r[i].w;
  const float f = __uint_as_float(x);
  // `never` is a value the data cannot fold to: the store keeps the loads alive without happening.
  if (x == never) sink[0] = f;
  for (int j = threadIdx.x; j < store_floats; j += kProbeThreads) {
    float* p = &sink[static_cast<size_t>(blockIdx.x) * store_floats + j];
    if (kStore == 0) *p = f;
    else if (kStore == 1) __builtin_nontemporal_store(f, p);
    else store_stream(p, f);
  }
}

using ProbeFn = void (*)(const uint4*, float*, int, unsigned);
ProbeFn pick_probe(bool nt, int store) {
  if (nt) return store == 0 ? probe_read<true, 0> : store == 1 ? probe_read<true, 1> : probe_read<true, 2>;
  return store == 0 ? probe_read<false, 0> : store == 1 ? probe_read<false, 1> : probe_read<false, 2>;
}

}  // namespace
}  // namespace xkv

extern "C" xkv_status xkv_probe_stream_read(const void* buffer, size_t bytes, int32_t non_temporal,
                                            int32_t store_floats_per_workgroup, int32_t store_policy,
                                            float* sink, void* hip_stream) {
  using namespace xkv;
  constexpr size_t per_wg = static_cast<size_t>(kProbeThreads) * kProbeLoads * 16;
  if (buffer == nullptr || (reinterpret_cast<uintptr_t>(buffer) & 15u) || bytes < per_wg)
    return XKV_ERR_INVALID_ARG;
  if (store_floats_per_workgroup < 0 || sink == nullptr || store_policy < 0 || store_policy > 2)
    return XKV_ERR_INVALID_ARG;
  const size_t grid = bytes / per_wg;
  if (grid > 0x7fffffffu) return XKV_ERR_INVALID_ARG;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  hipLaunchKernelGGL(pick_probe(non_temporal != 0, store_policy), dim3(static_cast<unsigned>(grid)),
                     dim3(kProbeThreads), 0, stream, static_cast<const uint4*>(buffer), sink,
                     store_floats_per_workgroup, 0x9e3779b9u);
  return hipGetLastError() == hipSuccess ? XKV_OK : XKV_ERR_DEVICE;
}
