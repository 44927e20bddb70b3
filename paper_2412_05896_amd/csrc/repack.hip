// xkv_repack: moves the live tokens of a ragged cache into another cache of the
// same shape whose streams have other capacities (the ragged layout of the
// per-layer cache sizes that Alg. 1 hands out: once the prefill-phase eviction
// has cut every layer to its budget, the prompt-sized arena can be given back
// and decoding continues in an arena sized by the allocation list).
//
// One launch per 1024 (layer, sequence) regions, the geometry in the kernel
// arguments: nothing is copied from the host and the call can be captured in a
// HIP graph.  Workgroup = 256 consecutive slots of one stream: whole K and V rows
// with 16-byte non-temporal loads, score and pos by the first lanes.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <limits>

#include "device_util.h"
#include "xkv_internal.h"

namespace xkv {
namespace {

constexpr int kThreads = 256;
constexpr int kBlockRows = 256;          // slots per workgroup
constexpr int kRepackRegions = 1024;     // regions per launch (32 KiB of kernel arguments)

struct RepackPair {
  int64_t src_slot0, dst_slot0;          // first slot of the region in either cache
  int32_t src_cap, dst_cap;              // slots per stream
  int32_t n;                             // live slots
  int32_t block0;                        // first workgroup of the region in this launch
};

struct RepackParams {
  const void* src_k;
  const void* src_v;
  const float* src_score;
  const int32_t* src_pos;
  void* dst_k;
  void* dst_v;
  float* dst_score;
  int32_t* dst_pos;
  int32_t n_pairs, n_kv_heads, row_bytes;
  RepackPair pairs[kRepackRegions];
};

__global__ __launch_bounds__(kThreads) void repack_copy(const RepackParams P) {
  const int bid = blockIdx.x;
  int lo = 0, hi = P.n_pairs - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (P.pairs[mid].block0 <= bid) lo = mid; else hi = mid - 1;
  }
  const RepackPair pd = P.pairs[lo];
  const int chunks = (pd.n + kBlockRows - 1) / kBlockRows;
  const int local = bid - pd.block0;
  const int h = local / chunks;
  const int r0 = (local - h * chunks) * kBlockRows;
  const int r1 = min(pd.n, r0 + kBlockRows);
  const int64_t s_slot = pd.src_slot0 + static_cast<int64_t>(h) * pd.src_cap;
  const int64_t d_slot = pd.dst_slot0 + static_cast<int64_t>(h) * pd.dst_cap;
  const int tid = threadIdx.x;
  if (r0 + tid < r1) {
    P.dst_score[d_slot + r0 + tid] = P.src_score[s_slot + r0 + tid];
    P.dst_pos[d_slot + r0 + tid] = P.src_pos[s_slot + r0 + tid];
  }
  // The rows of a stream are contiguous in both caches: the block's K (and V)
  // bytes are one contiguous range, copied 16 bytes per thread and pass, four
  // passes requested before the first is stored.
  const int64_t bytes = static_cast<int64_t>(r1 - r0) * P.row_bytes;
  const char* sk = static_cast<const char*>(P.src_k) + (s_slot + r0) * P.row_bytes;
  const char* sv = static_cast<const char*>(P.src_v) + (s_slot + r0) * P.row_bytes;
  char* dk = static_cast<char*>(P.dst_k) + (d_slot + r0) * P.row_bytes;
  char* dv = static_cast<char*>(P.dst_v) + (d_slot + r0) * P.row_bytes;
  constexpr int kPasses = 8;
  for (int64_t off = static_cast<int64_t>(tid) * 16; off < bytes; off += kPasses * kThreads * 16) {
    uint4 a[kPasses], b[kPasses];
#pragma unroll
    for (int u = 0; u < kPasses; ++u) {
      const int64_t o = off + static_cast<int64_t>(u) * kThreads * 16;
      const int64_t oc = o < bytes ? o : off;           // past the end: a valid piece again, not stored
      a[u] = load_stream16(sk + oc);
      b[u] = load_stream16(sv + oc);
    }
#pragma unroll
    for (int u = 0; u < kPasses; ++u) {
      const int64_t o = off + static_cast<int64_t>(u) * kThreads * 16;
      if (o < bytes) {
        *reinterpret_cast<uint4*>(dk + o) = a[u];
        *reinterpret_cast<uint4*>(dv + o) = b[u];
      }
    }
  }
}

}  // namespace
}  // namespace xkv

extern "C" xkv_status xkv_repack(const xkv_cache* src, xkv_cache* dst, int32_t layer_begin,
                                 int32_t layer_end, void* hip_stream) {
  using namespace xkv;
  xkv_status st = check_cache(src);
  if (st != XKV_OK) return st;
  st = check_cache(dst);
  if (st != XKV_OK) return st;
  st = check_layers(src, layer_begin, layer_end);
  if (st != XKV_OK) return st;
  if (src->n_layers != dst->n_layers || src->batch != dst->batch || src->n_q_heads != dst->n_q_heads ||
      src->n_kv_heads != dst->n_kv_heads || src->head_dim != dst->head_dim || src->dtype != dst->dtype)
    return XKV_ERR_INVALID_ARG;
  const int B = src->batch, hkv = src->n_kv_heads;
  const int row_bytes = src->head_dim * (src->dtype == XKV_F32 ? 4 : 2);
  const int64_t first = static_cast<int64_t>(layer_begin) * B;
  const int64_t n_pairs = static_cast<int64_t>(layer_end - layer_begin) * B;
  // The arenas must not overlap where this call touches them: the copy is not in place.
  auto overlaps = [](const void* a, int64_t an, const void* b, int64_t bn) {
    const char* pa = static_cast<const char*>(a);
    const char* pb = static_cast<const char*>(b);
    return pa < pb + bn && pb < pa + an;
  };
  if (overlaps(src->k, src->arena_slots * row_bytes, dst->k, dst->arena_slots * row_bytes) ||
      overlaps(src->v, src->arena_slots * row_bytes, dst->v, dst->arena_slots * row_bytes) ||
      overlaps(src->score, src->arena_slots * 4, dst->score, dst->arena_slots * 4) ||
      overlaps(src->pos, src->arena_slots * 4, dst->pos, dst->arena_slots * 4))
    return XKV_ERR_INVALID_ARG;
  for (int64_t i = 0; i < n_pairs; ++i)
    if (src->len[first + i] > dst->cap[first + i]) return XKV_ERR_CAPACITY;

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  RepackParams P;
  P.src_k = src->k; P.src_v = src->v; P.src_score = src->score; P.src_pos = src->pos;
  P.dst_k = dst->k; P.dst_v = dst->v; P.dst_score = dst->score; P.dst_pos = dst->pos;
  P.n_kv_heads = hkv;
  P.row_bytes = row_bytes;
  for (int64_t g0 = 0; g0 < n_pairs; g0 += kRepackRegions) {
    const int np = static_cast<int>(std::min<int64_t>(kRepackRegions, n_pairs - g0));
    int64_t blocks = 0;
    for (int i = 0; i < np; ++i) {
      const int64_t idx = first + g0 + i;
      RepackPair& pd = P.pairs[i];
      pd.src_slot0 = src->region_off[idx];
      pd.dst_slot0 = dst->region_off[idx];
      pd.src_cap = src->cap[idx];
      pd.dst_cap = dst->cap[idx];
      pd.n = src->len[idx];
      if (blocks > std::numeric_limits<int32_t>::max()) return XKV_ERR_UNSUPPORTED;
      pd.block0 = static_cast<int32_t>(blocks);
      blocks += ceil_div(pd.n, kBlockRows) * hkv;
    }
    if (blocks > std::numeric_limits<int32_t>::max()) return XKV_ERR_UNSUPPORTED;
    P.n_pairs = np;
    if (blocks > 0) {
      hipLaunchKernelGGL(repack_copy, dim3(static_cast<unsigned>(blocks)), dim3(kThreads), 0, stream, P);
      if (hipGetLastError() != hipSuccess) return XKV_ERR_DEVICE;
    }
  }
  for (int64_t i = 0; i < n_pairs; ++i) dst->len[first + i] = src->len[first + i];
  return XKV_OK;
}
