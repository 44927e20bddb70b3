// xkv_cache_importance: the score vector of a layer taken from the decode-time
// cache, for running the allocation (Alg. 1) again during generation: the paper's
// allocation is meant to follow the task (Sec. 2), and Alg. 1 takes one attention
// score distribution vector per layer (Sec. 4.1).  After per-head eviction the KV
// heads of a layer hold different tokens, so the vector is indexed by original
// position: w[p] = the scores of the tokens with pos = p, added over the heads that
// still hold one, in head order in fp32; 0 where no head does.
//
// Workgroup = (range of 8192 positions, region): it keeps its part of w in LDS,
// walks the region's heads in order and, for every head, lets each thread add the
// scores of the slots whose position falls into the range (positions are distinct
// within a stream, so no two threads meet; a barrier separates the heads).  No
// atomics and no workspace: the result is bit-reproducible and zero-filled.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "device_util.h"
#include "xkv_internal.h"

namespace xkv {
namespace {

constexpr int kImpThreads = 1024;
constexpr int kImpRange = 8192;          // positions per workgroup (32 KiB of LDS)
constexpr int kImpRegions = 1024;        // regions per launch (16 KiB of kernel arguments)

struct ImpPair {
  int64_t slot0;   // first slot of the region
  int32_t cap;     // slots per stream
  int32_t n;       // live slots
};

struct ImpParams {
  const float* score;
  const int32_t* pos;
  float* w_out;            // first region of this launch
  int32_t n_pos, n_kv_heads;
  ImpPair pairs[kImpRegions];
};

__global__ __launch_bounds__(kImpThreads) void cache_importance(const ImpParams P) {
  __shared__ float w_sh[kImpRange];
  const int tid = threadIdx.x;
  const ImpPair pd = P.pairs[blockIdx.y];
  const int p0 = blockIdx.x * kImpRange;
  const int p1 = min(P.n_pos, p0 + kImpRange);
  for (int i = tid; i < kImpRange; i += kImpThreads) w_sh[i] = 0.0f;
  __syncthreads();
  for (int h = 0; h < P.n_kv_heads; ++h) {
    const int64_t base = pd.slot0 + static_cast<int64_t>(h) * pd.cap;
    const int32_t* pos = P.pos + base;
    const float* score = P.score + base;
#pragma unroll 4
    for (int j = tid; j < pd.n; j += kImpThreads) {
      const int p = pos[j];
      if (p >= p0 && p < p1) w_sh[p - p0] = w_sh[p - p0] + score[j];
    }
    __syncthreads();
  }
  float* w = P.w_out + static_cast<int64_t>(blockIdx.y) * P.n_pos + p0;
  for (int i = tid; i < p1 - p0; i += kImpThreads) w[i] = w_sh[i];
}

}  // namespace
}  // namespace xkv

extern "C" xkv_status xkv_cache_importance(const xkv_cache* cache, int32_t layer_begin,
                                           int32_t layer_end, int32_t n_pos, float* w_out,
                                           void* hip_stream) {
  using namespace xkv;
  xkv_status st = check_cache(cache);
  if (st != XKV_OK) return st;
  st = check_layers(cache, layer_begin, layer_end);
  if (st != XKV_OK) return st;
  if (w_out == nullptr || n_pos < 1 || (reinterpret_cast<uintptr_t>(w_out) & 3u)) return XKV_ERR_INVALID_ARG;
  const int B = cache->batch;
  const int64_t first = static_cast<int64_t>(layer_begin) * B;
  const int64_t n_pairs = static_cast<int64_t>(layer_end - layer_begin) * B;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  ImpParams P;
  P.score = cache->score;
  P.pos = cache->pos;
  P.n_pos = n_pos;
  P.n_kv_heads = cache->n_kv_heads;
  const unsigned ranges = static_cast<unsigned>(ceil_div(n_pos, kImpRange));
  for (int64_t g0 = 0; g0 < n_pairs; g0 += kImpRegions) {
    const int np = static_cast<int>(std::min<int64_t>(kImpRegions, n_pairs - g0));
    for (int i = 0; i < np; ++i) {
      const int64_t idx = first + g0 + i;
      P.pairs[i].slot0 = cache->region_off[idx];
      P.pairs[i].cap = cache->cap[idx];
      P.pairs[i].n = cache->len[idx];
    }
    P.w_out = w_out + g0 * n_pos;
    hipLaunchKernelGGL(cache_importance, dim3(ranges, static_cast<unsigned>(np)), dim3(kImpThreads), 0, stream, P);
    if (hipGetLastError() != hipSuccess) return XKV_ERR_DEVICE;
  }
  return XKV_OK;
}
