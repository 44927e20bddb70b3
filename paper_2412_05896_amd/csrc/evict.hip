// xkv_evict_compact: per-(layer, sequence, KV head) top-budget selection and
// in-place compaction (Alg. 2 steps 4-7 of the paper: Pooling, TopK,
// EvictByIndex on K and V).
//
//  evict_select   one workgroup per stream.  Builds the keys (score, or its
//                 pooled window sum; +inf for protected tokens), finds the
//                 k'-th largest key by a 4-pass radix select on the fp32 bit
//                 pattern (scores are non-negative, so unsigned order = float
//                 order), then walks the slots in order to decide what is kept
//                 (equal keys: lower slot first) and to number the holes
//                 (evicted slots < k') and the movers (kept slots >= k').
//                 When every stream of the call moves only a few rows, the
//                 same workgroup moves them; otherwise it leaves the two lists
//                 in the workspace for
//  evict_move     which copies mover i over hole i, several workgroups per
//                 stream.  Sources are all >= k' and destinations all < k', so
//                 the copy is free of hazards.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <limits>

#include "device_util.h"
#include "select_util.h"
#include "xkv_internal.h"

namespace xkv {
namespace {

constexpr int kSelThreads = 512;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kMoveThreads = 256;
constexpr int kFuseMax = 64;     // moves the selecting workgroup does itself
constexpr int kSmallE = 8;       // evictions per stream found by repeated minimum search
constexpr int kWsAlign = 32;     // workspace words per stream are a multiple of this

struct EvictPair {
  int64_t slot0;   // first slot of the region
  int32_t cap;     // slots per stream
  int32_t n;       // live slots
  int32_t k;       // slots to keep, already min(budget, n)
  int32_t ws0;     // first workspace word of the region (per array)
};

struct EvictCommon {
  void* k;
  void* v;
  float* score;
  int32_t* pos;
  int32_t* kept_idx;     // may be null
  uint32_t* ws_keys;
  int32_t* ws_holes;
  int32_t* ws_movers;
  int32_t* ws_count;     // moves per stream of this launch
  int32_t n_pairs;
  int32_t n_kv_heads;
  int32_t pool;
  int32_t n_protect;
  int32_t row_bytes;
  int32_t fused;
  int32_t small;         // every stream evicts at most kSmallE tokens
};

// Geometry of up to kMaxPairs regions inside the kernel arguments, or, for larger
// calls, in device memory (written there from kernel arguments by evict_table_write),
// so that a call is one selection launch whatever its size.
struct EvictParams : EvictCommon {
  EvictPair pairs[kMaxPairs];
};
struct EvictTableParams : EvictCommon {
  const EvictPair* pairs;
};

constexpr int kEvictTableChunk = 1024;
struct EvictTableChunk {
  int32_t first, count;
  EvictPair pairs[kEvictTableChunk];
};
__global__ void evict_table_write(const EvictTableChunk c, EvictPair* pairs) {
  const int i = threadIdx.x;
  if (i < c.count) pairs[c.first + i] = c.pairs[i];
}

__device__ __forceinline__ int ws_stride(int n) { return (n + kWsAlign - 1) / kWsAlign * kWsAlign; }

// Copies the token at slot src over slot dst: K row, V row, score, pos.
__device__ __forceinline__ void move_row(const EvictCommon& P, int64_t stream_slot, int dst, int src,
                                         int lane) {
  const int frags = P.row_bytes >> 4;
  if (lane < frags) {
    char* kb = static_cast<char*>(P.k) + stream_slot * P.row_bytes;
    char* vb = static_cast<char*>(P.v) + stream_slot * P.row_bytes;
    const int64_t so = static_cast<int64_t>(src) * P.row_bytes + lane * 16;
    const int64_t dof = static_cast<int64_t>(dst) * P.row_bytes + lane * 16;
    const uint4 a = *reinterpret_cast<const uint4*>(kb + so);
    const uint4 b = *reinterpret_cast<const uint4*>(vb + so);
    *reinterpret_cast<uint4*>(kb + dof) = a;
    *reinterpret_cast<uint4*>(vb + dof) = b;
  } else if (lane == 32) {
    P.score[stream_slot + dst] = P.score[stream_slot + src];
  } else if (lane == 33) {
    P.pos[stream_slot + dst] = P.pos[stream_slot + src];
  } else if (lane == 34 && P.kept_idx != nullptr) {
    P.kept_idx[stream_slot + dst] = src;
  }
}

template <typename PT>
__global__ __launch_bounds__(kSelThreads) void evict_select(const PT P) {
  __shared__ RadixShared radix_sh;
  __shared__ int scan_sh[kSelWaves];
  __shared__ int cnt_sh[3][kSelWaves];
  __shared__ int hole_l[kFuseMax], mover_l[kFuseMax];
  __shared__ unsigned long long best_sh[kSelWaves];
  __shared__ int ev_sh[kSmallE];
  __shared__ int moves_sh;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int u = blockIdx.x;
  const int p = u / P.n_kv_heads;
  const int h = u - p * P.n_kv_heads;
  const EvictPair pd = P.pairs[p];
  const int n = pd.n;
  const int kk = pd.k;
  const int64_t stream_slot = pd.slot0 + static_cast<int64_t>(h) * pd.cap;
  const float* score = P.score + stream_slot;
  const int32_t* pos = P.pos + stream_slot;
  int32_t* kept = P.kept_idx ? P.kept_idx + stream_slot : nullptr;

  if (kk >= n || kk == 0) {                 // nothing to select
    if (kept != nullptr)
      for (int j = tid; j < kk; j += kSelThreads) kept[j] = j;
    if (tid == 0) P.ws_count[u] = 0;
    return;
  }
  const int64_t ws_off = static_cast<int64_t>(pd.ws0) + static_cast<int64_t>(h) * ws_stride(n);
  uint32_t* keys = P.ws_keys + ws_off;
  int32_t* holes_g = P.ws_holes + ws_off;
  int32_t* movers_g = P.ws_movers + ws_off;

  // ---- keys ----------------------------------------------------------------
  const bool derived = P.pool > 1 || P.n_protect > 0;
  if (derived) {
    int limit = std::numeric_limits<int>::min();      // protected: pos >= limit
    const bool protect = P.n_protect > 0;
    if (protect) {
      int mx = std::numeric_limits<int>::min();
#pragma unroll 4
      for (int j = tid; j < n; j += kSelThreads) mx = max(mx, pos[j]);
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) mx = max(mx, __shfl_xor(mx, off));
      if (lane == 0) scan_sh[wave] = mx;
      __syncthreads();
      mx = scan_sh[0];
#pragma unroll
      for (int w = 1; w < kSelWaves; ++w) mx = max(mx, scan_sh[w]);
      const long long lim = static_cast<long long>(mx) + 1 - P.n_protect;
      limit = lim < std::numeric_limits<int>::min() ? std::numeric_limits<int>::min()
                                                    : static_cast<int>(lim);
      __syncthreads();
    }
    const int half = P.pool >> 1;
#pragma unroll 2
    for (int j = tid; j < n; j += kSelThreads) {
      // window sum, fp32, left to right, zeros outside the stream; the terms are
      // fetched eight at a time so that their loads overlap
      float acc = 0.0f;
      for (int t0 = 0; t0 < P.pool; t0 += 8) {
        float term[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          const int x = j - half + t0 + q;
          const bool in = t0 + q < P.pool && x >= 0 && x < n;
          term[q] = in ? score[x] : 0.0f;
        }
#pragma unroll
        for (int q = 0; q < 8; ++q)
          if (t0 + q < P.pool) acc = (t0 + q == 0) ? term[q] : acc + term[q];
      }
      unsigned key = __float_as_uint(acc);
      if (protect && pos[j] >= limit) key = 0x7f800000u;
      keys[j] = key;
    }
    __syncthreads();
  }
  auto key_at = [&](int j) -> unsigned { return derived ? keys[j] : __float_as_uint(score[j]); };

  // ---- few evictions: the steady state of decoding ----------------------------
  // The evicted tokens are the last ones in (key descending, slot ascending)
  // order, i.e. the smallest under (key ascending, slot descending).  Packing
  // (key, ~slot) into 64 bits turns that into a plain minimum; E rounds, each
  // taking the smallest pack above the previous one, find them one by one.
  if (P.small) {
    const int E = n - kk;
    unsigned long long last = 0;            // every pack is > 0: ~slot has its top bit set
    for (int r = 0; r < E; ++r) {
      unsigned long long best = ~0ull;
#pragma unroll 4
      for (int j = tid; j < n; j += kSelThreads) {
        const unsigned long long pk =
            (static_cast<unsigned long long>(key_at(j)) << 32) | (0xffffffffu - static_cast<unsigned>(j));
        if (pk > last && pk < best) best = pk;
      }
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) {
        const unsigned long long o = __shfl_xor(best, off);
        best = o < best ? o : best;
      }
      if (lane == 0) best_sh[wave] = best;
      __syncthreads();
      best = best_sh[0];
#pragma unroll
      for (int w = 1; w < kSelWaves; ++w) best = best_sh[w] < best ? best_sh[w] : best;
      last = best;
      if (tid == 0) ev_sh[r] = static_cast<int>(0xffffffffu - static_cast<unsigned>(best & 0xffffffffull));
      __syncthreads();
    }
    if (tid == 0) {
      // holes: evicted slots below kk, ascending; movers: the survivors among
      // the E slots [kk, n), ascending.
      for (int a = 1; a < E; ++a) {          // insertion sort of at most kSmallE slots
        const int x = ev_sh[a];
        int b = a - 1;
        while (b >= 0 && ev_sh[b] > x) { ev_sh[b + 1] = ev_sh[b]; --b; }
        ev_sh[b + 1] = x;
      }
      int nh = 0, nm = 0;
      for (int a = 0; a < E; ++a)
        if (ev_sh[a] < kk) hole_l[nh++] = ev_sh[a];
      for (int s = kk; s < n; ++s) {
        bool evicted = false;
        for (int a = 0; a < E; ++a) evicted = evicted || ev_sh[a] == s;
        if (!evicted) mover_l[nm++] = s;
      }
      moves_sh = nh;
      P.ws_count[u] = 0;
    }
    __syncthreads();
    const int moves = moves_sh;
    if (kept != nullptr)
      for (int j = tid; j < kk; j += kSelThreads) {
        bool is_hole = false;
        for (int a = 0; a < moves; ++a) is_hole = is_hole || hole_l[a] == j;
        if (!is_hole) kept[j] = j;
      }
    for (int i = wave; i < moves; i += kSelWaves) move_row(P, stream_slot, hole_l[i], mover_l[i], lane);
    return;
  }

  // ---- radix select: the kk-th largest key -----------------------------------
  unsigned thr, need;                       // keys above thr are kept, `need` of the equal ones too
  radix_select([&](auto&& fn) { for (int j = tid; j < n; j += kSelThreads) fn(key_at(j)); }, kk, radix_sh,
               thr, need);

  // ---- walk the slots in order ---------------------------------------------
  int carry_eq = 0, carry_h = 0, carry_m = 0;
  for (int base = 0; base < n; base += kSelThreads) {
    const int j = base + tid;
    const bool live = j < n;
    const unsigned key = live ? key_at(j) : 0u;
    const bool is_eq = live && key == thr;
    const unsigned long long v_eq = __ballot(is_eq);
    if (lane == 0) cnt_sh[0][wave] = __popcll(v_eq);
    __syncthreads();
    int eq_rank = carry_eq + rank_in_wave(v_eq), eq_tot = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) {
      const int cw = cnt_sh[0][w];
      if (w < wave) eq_rank += cw;
      eq_tot += cw;
    }
    carry_eq += eq_tot;
    const bool keep = live && (key > thr || (is_eq && eq_rank < static_cast<int>(need)));
    const bool is_hole = live && j < kk && !keep;
    const bool is_mover = live && j >= kk && keep;
    const unsigned long long v_h = __ballot(is_hole);
    const unsigned long long v_m = __ballot(is_mover);
    if (lane == 0) {
      cnt_sh[1][wave] = __popcll(v_h);
      cnt_sh[2][wave] = __popcll(v_m);
    }
    __syncthreads();
    int h_rank = carry_h + rank_in_wave(v_h), m_rank = carry_m + rank_in_wave(v_m);
    int h_tot = 0, m_tot = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) {
      const int ch = cnt_sh[1][w], cm = cnt_sh[2][w];
      if (w < wave) { h_rank += ch; m_rank += cm; }
      h_tot += ch;
      m_tot += cm;
    }
    carry_h += h_tot;
    carry_m += m_tot;
    if (is_hole) { if (P.fused) hole_l[h_rank] = j; else holes_g[h_rank] = j; }
    if (is_mover) { if (P.fused) mover_l[m_rank] = j; else movers_g[m_rank] = j; }
    if (kept != nullptr && keep && j < kk) kept[j] = j;
    __syncthreads();                        // cnt_sh is reused by the next tile
  }

  if (!P.fused) {
    if (tid == 0) P.ws_count[u] = carry_h;
    return;
  }
  if (tid == 0) P.ws_count[u] = 0;
  for (int i = wave; i < carry_h; i += kSelWaves) move_row(P, stream_slot, hole_l[i], mover_l[i], lane);
}

template <typename PT>
__global__ __launch_bounds__(kMoveThreads) void evict_move(const PT P) {
  const int u = blockIdx.x;
  const int moves = P.ws_count[u];
  if (moves == 0) return;
  const int p = u / P.n_kv_heads;
  const int h = u - p * P.n_kv_heads;
  const EvictPair pd = P.pairs[p];
  const int64_t stream_slot = pd.slot0 + static_cast<int64_t>(h) * pd.cap;
  const int64_t ws_off = static_cast<int64_t>(pd.ws0) + static_cast<int64_t>(h) * ws_stride(pd.n);
  const int32_t* holes = P.ws_holes + ws_off;
  const int32_t* movers = P.ws_movers + ws_off;
  // A workgroup takes rows_per_pass moves at a time: every thread copies one 16-byte
  // piece of a K row and of a V row, the first thread of each row also score, pos and
  // the kept index.
  const int frags = P.row_bytes >> 4;                 // 8, 16 or 32 pieces per row
  const int rows_per_pass = kMoveThreads / frags;
  const int fr = threadIdx.x % frags, rw = threadIdx.x / frags;
  char* kb = static_cast<char*>(P.k) + stream_slot * P.row_bytes;
  char* vb = static_cast<char*>(P.v) + stream_slot * P.row_bytes;
  for (int i = blockIdx.y * rows_per_pass + rw; i < moves; i += gridDim.y * rows_per_pass) {
    const int dst = holes[i], src = movers[i];
    const int64_t so = static_cast<int64_t>(src) * P.row_bytes + fr * 16;
    const int64_t dof = static_cast<int64_t>(dst) * P.row_bytes + fr * 16;
    const uint4 a = *reinterpret_cast<const uint4*>(kb + so);
    const uint4 b = *reinterpret_cast<const uint4*>(vb + so);
    *reinterpret_cast<uint4*>(kb + dof) = a;
    *reinterpret_cast<uint4*>(vb + dof) = b;
    if (fr == 0) {
      P.score[stream_slot + dst] = P.score[stream_slot + src];
      P.pos[stream_slot + dst] = P.pos[stream_slot + src];
      if (P.kept_idx != nullptr) P.kept_idx[stream_slot + dst] = src;
    }
  }
}

}  // namespace

xkv_status evict_check_args(const xkv_cache* cache, int32_t layer_begin, int32_t layer_end, const int32_t* budgets,
                            int32_t pool_size, int32_t n_protect, int32_t extra_rows, const void* workspace,
                            size_t workspace_bytes) {
  if (budgets == nullptr) return XKV_ERR_INVALID_ARG;
  if (pool_size < 1 || (pool_size & 1) == 0 || n_protect < 0) return XKV_ERR_INVALID_ARG;
  const int B = cache->batch, hkv = cache->n_kv_heads;
  const int64_t first = static_cast<int64_t>(layer_begin) * B;
  const int64_t n_pairs = static_cast<int64_t>(layer_end - layer_begin) * B;
  int64_t words = 0;
  for (int64_t i = 0; i < n_pairs; ++i) {
    if (budgets[i] < 0 || budgets[i] < n_protect) return XKV_ERR_INVALID_ARG;
    words += ceil_div(static_cast<int64_t>(cache->len[first + i]) + extra_rows, kWsAlign) * kWsAlign * hkv;
  }
  if (words > std::numeric_limits<int32_t>::max()) return XKV_ERR_UNSUPPORTED;
  const int64_t units = n_pairs * hkv;
  const uint64_t table_off = (static_cast<uint64_t>(words) * 12 + static_cast<uint64_t>(units) * 4 + 255) / 256 * 256;
  const uint64_t need_bytes = n_pairs > kMaxPairs ? table_off + static_cast<uint64_t>(n_pairs) * sizeof(EvictPair)
                                                  : static_cast<uint64_t>(words) * 12 + static_cast<uint64_t>(units) * 4;
  if (workspace == nullptr || need_bytes > workspace_bytes) return XKV_ERR_CAPACITY;
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return XKV_ERR_INVALID_ARG;
  return XKV_OK;
}

}  // namespace xkv

extern "C" xkv_status xkv_evict_compact(xkv_cache* cache, int32_t layer_begin, int32_t layer_end,
                                        const int32_t* budgets, int32_t pool_size,
                                        int32_t n_protect, int32_t* kept_idx_out, void* workspace,
                                        size_t workspace_bytes, void* hip_stream) {
  using namespace xkv;
  xkv_status st = check_cache(cache);
  if (st != XKV_OK) return st;
  st = check_layers(cache, layer_begin, layer_end);
  if (st != XKV_OK) return st;
  if (budgets == nullptr) return XKV_ERR_INVALID_ARG;
  if (pool_size < 1 || (pool_size & 1) == 0 || n_protect < 0) return XKV_ERR_INVALID_ARG;

  const int B = cache->batch, hkv = cache->n_kv_heads;
  const int64_t first = static_cast<int64_t>(layer_begin) * B;
  const int64_t n_pairs = static_cast<int64_t>(layer_end - layer_begin) * B;
  int64_t words = 0;            // workspace words per array
  int64_t max_moves = 0, max_evict = 0;
  bool any_work = false;
  for (int64_t i = 0; i < n_pairs; ++i) {
    const int64_t bud = budgets[i];
    if (bud < 0 || bud < n_protect) return XKV_ERR_INVALID_ARG;
    const int64_t n = cache->len[first + i];
    const int64_t kk = std::min(bud, n);
    if (kk < n && kk > 0) {
      max_moves = std::max(max_moves, std::min(kk, n - kk));
      max_evict = std::max(max_evict, n - kk);
      any_work = true;
    }
    words += ceil_div(n, kWsAlign) * kWsAlign * hkv;
  }
  const int64_t units = n_pairs * hkv;
  // keys, holes, movers; a move counter per stream; the region table of a large call
  const uint64_t table_off = (static_cast<uint64_t>(words) * 12 + static_cast<uint64_t>(units) * 4 + 255) / 256 * 256;
  const uint64_t need_bytes = n_pairs > kMaxPairs ? table_off + static_cast<uint64_t>(n_pairs) * sizeof(EvictPair)
                                                  : static_cast<uint64_t>(words) * 12 + static_cast<uint64_t>(units) * 4;
  if (workspace == nullptr || need_bytes > workspace_bytes) return XKV_ERR_CAPACITY;
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return XKV_ERR_INVALID_ARG;

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (any_work || kept_idx_out != nullptr) {
    EvictParams P;
    P.k = cache->k; P.v = cache->v; P.score = cache->score; P.pos = cache->pos;
    P.kept_idx = kept_idx_out;
    P.ws_keys = static_cast<uint32_t*>(workspace);
    P.ws_holes = reinterpret_cast<int32_t*>(P.ws_keys + words);
    P.ws_movers = P.ws_holes + words;
    int32_t* counts = P.ws_movers + words;
    P.n_kv_heads = hkv;
    P.pool = pool_size;
    P.n_protect = n_protect;
    P.row_bytes = cache->head_dim * (cache->dtype == XKV_F32 ? 4 : 2);
    P.fused = max_moves <= kFuseMax ? 1 : 0;
    P.small = max_evict <= kSmallE ? 1 : 0;
    const unsigned move_blocks =
        static_cast<unsigned>(std::min<int64_t>(64, std::max<int64_t>(1, ceil_div(max_moves, 64))));

    if (words > std::numeric_limits<int32_t>::max()) return XKV_ERR_UNSUPPORTED;   // 32-bit word offsets
    P.ws_count = counts;
    P.n_pairs = static_cast<int32_t>(n_pairs);
    auto fill_pair = [&](EvictPair& pd, int64_t i, int64_t w) {
      const int64_t idx = first + i;
      pd.slot0 = cache->region_off[idx];
      pd.cap = cache->cap[idx];
      pd.n = cache->len[idx];
      pd.k = static_cast<int32_t>(std::min<int64_t>(budgets[i], pd.n));
      pd.ws0 = static_cast<int32_t>(w);
      return w + ceil_div(pd.n, kWsAlign) * kWsAlign * hkv;
    };
    const dim3 sel_grid(static_cast<unsigned>(units));
    const dim3 move_grid(static_cast<unsigned>(units), move_blocks);
    if (n_pairs <= kMaxPairs) {
      int64_t w = 0;
      for (int64_t i = 0; i < n_pairs; ++i) w = fill_pair(P.pairs[i], i, w);
      const int tok = profile_begin(1, stream);
      hipLaunchKernelGGL(evict_select<EvictParams>, sel_grid, dim3(kSelThreads), 0, stream, P);
      profile_end(tok, stream);
      if (hipGetLastError() != hipSuccess) return XKV_ERR_DEVICE;
      if (!P.fused) {
        hipLaunchKernelGGL(evict_move<EvictParams>, move_grid, dim3(kMoveThreads), 0, stream, P);
        if (hipGetLastError() != hipSuccess) return XKV_ERR_DEVICE;
      }
    } else {
      EvictPair* d_pairs = reinterpret_cast<EvictPair*>(static_cast<char*>(workspace) + table_off);
      int64_t w = 0;
      for (int64_t c0 = 0; c0 < n_pairs; c0 += kEvictTableChunk) {
        EvictTableChunk ch;
        ch.first = static_cast<int32_t>(c0);
        ch.count = static_cast<int32_t>(std::min<int64_t>(kEvictTableChunk, n_pairs - c0));
        for (int i = 0; i < ch.count; ++i) w = fill_pair(ch.pairs[i], c0 + i, w);
        hipLaunchKernelGGL(evict_table_write, dim3(1), dim3(kEvictTableChunk), 0, stream, ch, d_pairs);
      }
      if (hipGetLastError() != hipSuccess) return XKV_ERR_DEVICE;
      EvictTableParams T;
      static_cast<EvictCommon&>(T) = static_cast<const EvictCommon&>(P);
      T.pairs = d_pairs;
      const int tok = profile_begin(1, stream);
      hipLaunchKernelGGL(evict_select<EvictTableParams>, sel_grid, dim3(kSelThreads), 0, stream, T);
      profile_end(tok, stream);
      if (hipGetLastError() != hipSuccess) return XKV_ERR_DEVICE;
      if (!T.fused) {
        hipLaunchKernelGGL(evict_move<EvictTableParams>, move_grid, dim3(kMoveThreads), 0, stream, T);
        if (hipGetLastError() != hipSuccess) return XKV_ERR_DEVICE;
      }
    }
  }
  for (int64_t i = 0; i < n_pairs; ++i) {
    const int64_t n = cache->len[first + i];
    cache->len[first + i] = static_cast<int32_t>(std::min<int64_t>(budgets[i], n));
  }
  return XKV_OK;
}
