// Host-side pieces shared by the entry points: descriptor validation,
// workspace sizing, status names and the optional per-kernel event timing.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <functional>
#include <mutex>
#include <vector>

#include "xkv_internal.h"

namespace xkv {

xkv_status check_cache(const xkv_cache* c) {
  if (c == nullptr) return XKV_ERR_INVALID_ARG;
  if (c->n_layers <= 0 || c->batch <= 0 || c->n_q_heads <= 0 || c->n_kv_heads <= 0)
    return XKV_ERR_INVALID_ARG;
  if (c->n_q_heads % c->n_kv_heads != 0) return XKV_ERR_INVALID_ARG;
  if (c->dtype != XKV_F32 && c->dtype != XKV_BF16) return XKV_ERR_INVALID_ARG;
  if (c->k == nullptr || c->v == nullptr || c->score == nullptr || c->pos == nullptr ||
      c->region_off == nullptr || c->cap == nullptr || c->len == nullptr)
    return XKV_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(c->k) & 15u) || (reinterpret_cast<uintptr_t>(c->v) & 15u))
    return XKV_ERR_INVALID_ARG;
  if (c->arena_slots < 0) return XKV_ERR_INVALID_ARG;
  if (c->head_dim != 64 && c->head_dim != 128) return XKV_ERR_UNSUPPORTED;
  const int group = c->n_q_heads / c->n_kv_heads;
  if (group != 1 && group != 2 && group != 4 && group != 8) return XKV_ERR_UNSUPPORTED;
  const int64_t regions = static_cast<int64_t>(c->n_layers) * c->batch;
  for (int64_t i = 0; i < regions; ++i) {
    const int64_t off = c->region_off[i], cap = c->cap[i], len = c->len[i];
    if (off < 0 || cap < 0 || len < 0 || len > cap) return XKV_ERR_INVALID_ARG;
    if (off + cap * c->n_kv_heads > c->arena_slots) return XKV_ERR_INVALID_ARG;
  }
  return XKV_OK;
}

xkv_status check_layers(const xkv_cache* c, int32_t layer_begin, int32_t layer_end) {
  if (layer_begin < 0 || layer_end > c->n_layers || layer_end <= layer_begin)
    return XKV_ERR_INVALID_ARG;
  return XKV_OK;
}

namespace {
// Sum of the `layers` largest per-layer needs: an upper bound for any range of
// that many layers.
size_t top_layers_sum(const xkv_cache* c, int32_t layers,
                      const std::function<size_t(int64_t cap)>& per_region) {
  std::vector<size_t> need(static_cast<size_t>(c->n_layers), 0);
  for (int32_t l = 0; l < c->n_layers; ++l)
    for (int32_t b = 0; b < c->batch; ++b)
      need[l] += per_region(c->cap[static_cast<int64_t>(l) * c->batch + b]);
  std::sort(need.begin(), need.end(), std::greater<size_t>());
  size_t tot = 0;
  for (int32_t l = 0; l < layers && l < c->n_layers; ++l) tot += need[l];
  return tot;
}
}  // namespace

size_t evict_workspace_bytes(const xkv_cache* c, int32_t layers) {
  // Per stream: keys, hole list and mover list (one 32-bit word per slot each,
  // slot counts rounded up to 32) and one move counter.
  const int hkv = c->n_kv_heads;
  // ... and, for calls on more regions than the kernel arguments hold, 24 bytes per region.
  return top_layers_sum(c, layers, [=](int64_t cap) {
    return static_cast<size_t>(hkv) * (static_cast<size_t>(ceil_div(cap, 32) * 32) * 12 + 4) + 24;
  }) + 512;
}

// ---- per-kernel event timing ------------------------------------------------
namespace {
struct Span { hipEvent_t start, stop; int kernel; };
std::mutex g_prof_mu;
bool g_prof_on = false;
std::vector<Span> g_spans;

void drop_spans() {
  for (Span& s : g_spans) {
    (void)hipEventDestroy(s.start);
    (void)hipEventDestroy(s.stop);
  }
  g_spans.clear();
}
}  // namespace

int profile_begin(int kernel_index, void* stream) {
  std::lock_guard<std::mutex> lock(g_prof_mu);
  if (!g_prof_on) return -1;
  Span s;
  s.kernel = kernel_index;
  if (hipEventCreate(&s.start) != hipSuccess) return -1;
  if (hipEventCreate(&s.stop) != hipSuccess) { (void)hipEventDestroy(s.start); return -1; }
  (void)hipEventRecord(s.start, static_cast<hipStream_t>(stream));
  g_spans.push_back(s);
  return static_cast<int>(g_spans.size()) - 1;
}

void profile_end(int token, void* stream) {
  if (token < 0) return;
  std::lock_guard<std::mutex> lock(g_prof_mu);
  if (token < static_cast<int>(g_spans.size()))
    (void)hipEventRecord(g_spans[token].stop, static_cast<hipStream_t>(stream));
}

}  // namespace xkv

extern "C" const char* xkv_status_string(xkv_status s) {
  switch (s) {
    case XKV_OK: return "XKV_OK";
    case XKV_ERR_INVALID_ARG: return "XKV_ERR_INVALID_ARG";
    case XKV_ERR_INFEASIBLE: return "XKV_ERR_INFEASIBLE";
    case XKV_ERR_CAPACITY: return "XKV_ERR_CAPACITY";
    case XKV_ERR_UNSUPPORTED: return "XKV_ERR_UNSUPPORTED";
    case XKV_ERR_DEVICE: return "XKV_ERR_DEVICE";
    default: return "XKV_ERR_UNKNOWN";
  }
}

extern "C" xkv_status xkv_workspace_bytes(const xkv_cache* cache, int32_t max_layers_per_call,
                                          size_t* bytes_out) {
  const xkv_status st = xkv::check_cache(cache);
  if (st != XKV_OK) return st;
  if (bytes_out == nullptr || max_layers_per_call <= 0) return XKV_ERR_INVALID_ARG;
  const int32_t layers = std::min(max_layers_per_call, cache->n_layers);
  *bytes_out = std::max(xkv::attend_workspace_bytes(cache, layers),
                        xkv::evict_workspace_bytes(cache, layers)) + 4096;
  return XKV_OK;
}

extern "C" xkv_status xkv_profile_enable(int32_t on) {
  std::lock_guard<std::mutex> lock(xkv::g_prof_mu);
  if (on) xkv::drop_spans();
  xkv::g_prof_on = on != 0;
  return XKV_OK;
}

extern "C" xkv_status xkv_profile_read(int32_t kernel_index, int64_t* launches_out,
                                       double* total_ms_out) {
  if (launches_out == nullptr || total_ms_out == nullptr) return XKV_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lock(xkv::g_prof_mu);
  int64_t cnt = 0;
  double ms = 0.0;
  for (xkv::Span& s : xkv::g_spans) {
    if (s.kernel != kernel_index) continue;
    if (hipEventSynchronize(s.stop) != hipSuccess) return XKV_ERR_DEVICE;
    float t = 0.0f;
    if (hipEventElapsedTime(&t, s.start, s.stop) != hipSuccess) return XKV_ERR_DEVICE;
    ms += t;
    ++cnt;
  }
  *launches_out = cnt;
  *total_ms_out = ms;
  return XKV_OK;
}
