// xkv_decode_attend_score: decode attention over the ragged cache with
// per-token attention-mass scoring (Eq. 1 and Eq. 2 of the paper; scoring is the
// Select + Merge step of Eq. 3 with the decode query as observation row).
//
// Two kernels per launch group, no atomics:
//
//  attend_partial   one workgroup per (stream, chunk of 256 slots).  Streams
//                   the chunk's K and V rows once with 16-byte loads, computes
//                   the G logits of every row, the chunk's softmax statistics
//                   (max m_c, sum l_c), the un-normalised probabilities
//                   e_j = 2^(s_j - m_c) and the partial output sum_j e_j V_j,
//                   and writes all of that to the workspace.  The workgroup
//                   that owns the last slot also stores the appended token.
//  attend_finalize  one workgroup per (stream, 4 chunks).  Every workgroup merges
//                   the chunk statistics of its stream into (m, l) and the chunk
//                   weights w_c = 2^(m_c - m) / l, adds p_j = e_j w_c, summed over
//                   the G query heads, to score[j] for its own slots, and
//                   computes its share of the channels of out = sum_c w_c o_c.
//
// The ragged geometry travels in the kernel arguments (at most kMaxPairs
// (layer, sequence) regions per launch), so nothing is copied to the device
// and the launches can be captured in a HIP graph.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <limits>
#include <vector>

#include "device_util.h"
#include "xkv_internal.h"

namespace xkv {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

struct PairDesc {
  int64_t slot0;    // first slot of the region
  int32_t cap;      // slots per stream
  int32_t n;        // live slots, the appended token included
  int32_t block0;   // first streaming-kernel workgroup of the region in this launch
  int32_t fblock0;  // first finalize-kernel workgroup of the region in this launch
};

struct AttendParams {
  const void* q;
  const void* k_new;
  const void* v_new;
  void* k;
  void* v;
  float* score;
  int32_t* pos;
  float* out;
  float* ws;              // first record of this launch
  float scale_log2e;      // softmax scale times log2(e): logits live in the base-2 domain
  int32_t n_pairs;
  int32_t pair_base;      // index of pairs[0] relative to (layer_begin, sequence 0)
  int32_t n_kv_heads;
  int32_t append;
  PairDesc pairs[kMaxPairs];
  int32_t pos_new[kMaxPairs];  // original position of the token appended to each region
};

// Chunks of one stream that one workgroup of the finalize kernel covers.
constexpr int kFinalChunks = 4;

// Finds the region, KV head and chunk of workgroup `bid` (same numbering in
// both kernels): the last pair whose first workgroup is <= bid.  A stream with
// no live slot still owns one workgroup.
struct Work { int pair_local, h, c, nchunks; };
__device__ __forceinline__ Work locate(const AttendParams& P, int bid) {
  int lo = 0, hi = P.n_pairs - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (P.pairs[mid].block0 <= bid) lo = mid; else hi = mid - 1;
  }
  Work w;
  w.pair_local = lo;
  w.nchunks = (P.pairs[lo].n + kChunk - 1) / kChunk;
  const int per_head = w.nchunks > 0 ? w.nchunks : 1;
  const int local = bid - P.pairs[lo].block0;
  w.h = local / per_head;
  w.c = local - w.h * per_head;
  return w;
}


// Loads kNB consecutive wave-wide fragments of a stream (rows first_row,
// first_row + RPW, ...) into registers, without branches: rows at or past n are
// clamped to row n-1 (in bounds; their logits are masked later and their
// probabilities are zero), and with append_here the lanes of row n-1 read the
// token being appended from `newrow` instead of the not yet written slot.
template <int ROWB, int RPW, int kNB>
__device__ __forceinline__ void load_rows(uint4 (&reg)[kNB], const char* base, const char* newrow,
                                          int first_row, int n, bool full, bool append_here,
                                          int cl) {
  if (full) {
#pragma unroll
    for (int i = 0; i < kNB; ++i) {
      const int64_t off = static_cast<int64_t>(first_row + i * RPW) * ROWB + cl * 16;
      reg[i] = load_stream16(base + off);
    }
  } else {
#pragma unroll
    for (int i = 0; i < kNB; ++i) {
      const int r = first_row + i * RPW;
      const int rc = r < n ? r : n - 1;
      const char* src = base + static_cast<int64_t>(rc) * ROWB + cl * 16;
      if (append_here && r == n - 1) src = newrow + cl * 16;
      reg[i] = load_stream16(src);
    }
  }
}

// The append itself: the lanes that hold row n-1 (read from the new token's
// row by load_rows) store it into the stream.
template <int ROWB, int RPW, int kNB>
__device__ __forceinline__ void store_appended(const uint4 (&reg)[kNB], char* base, int first_row,
                                               int n, int cl) {
#pragma unroll
  for (int i = 0; i < kNB; ++i) {
    const int r = first_row + i * RPW;
    if (r == n - 1)
      *reinterpret_cast<uint4*>(base + static_cast<int64_t>(r) * ROWB + cl * 16) = reg[i];
  }
}

// ---------------------------------------------------------------------------
template <typename T, int D, int G>
__global__ __launch_bounds__(kThreads) void attend_partial(const AttendParams P) {
  constexpr int EPL = T::kPerLane;          // elements per lane per load
  constexpr int LPR = D / EPL;              // lanes that cover one row
  constexpr int RPW = 64 / LPR;             // rows per wave-wide load
  constexpr int NT = 64 / RPW;              // loads per wave for its 64 rows
  constexpr int ROWB = D * T::kBytes;       // bytes per row
  constexpr int REC = G * (kChunk + D + 2);
  constexpr int kTB = NT < 16 ? NT : 16;    // wave-wide loads in flight per batch
  constexpr bool V_EARLY = NT <= 16 && G <= 2;

  __shared__ float s_sh[G][kChunk];         // logits, then probabilities
  __shared__ float red_sh[2][G][kWaves];
  __shared__ float o_sh[kWaves][G][D];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int sub = lane / LPR;               // row within a wave-wide load
  const int cl = lane % LPR;                // 16-byte column of the row
  const int bid = blockIdx.x;

  const Work wk = locate(P, bid);
  const int lo = wk.pair_local;
  const PairDesc pd = P.pairs[lo];
  const int n = pd.n;
  if (n == 0) return;                       // an empty stream: the finalize kernel zeroes its output
  const int h = wk.h, c = wk.c;
  const int pair = P.pair_base + lo;
  const int64_t stream_slot = pd.slot0 + static_cast<int64_t>(h) * pd.cap;
  char* kbase = static_cast<char*>(P.k) + stream_slot * ROWB;
  char* vbase = static_cast<char*>(P.v) + stream_slot * ROWB;
  const int row0 = c * kChunk + wave * 64;
  const bool append_here = P.append && (n - 1) / kChunk == c;
  const char* knew = nullptr;
  const char* vnew = nullptr;
  if (append_here) {
    const int64_t r = (static_cast<int64_t>(pair) * P.n_kv_heads + h) * ROWB;
    knew = static_cast<const char*>(P.k_new) + r;
    vnew = static_cast<const char*>(P.v_new) + r;
  }

  // Queries of the group, widened to fp32, this lane's columns only.
  float qf[G][EPL];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    const int64_t hq = (static_cast<int64_t>(pair) * P.n_kv_heads + h) * G + g;
    const uint4 raw = *reinterpret_cast<const uint4*>(static_cast<const char*>(P.q) + hq * ROWB + cl * 16);
    Unpack<T>::run(raw, qf[g]);
  }

  // K rows of this wave, kTB wave-wide loads at a time, all issued before the
  // first is used; when registers allow, the V loads go out right behind them
  // so that they are in flight during the softmax statistics.
  const bool full = (c + 1) * kChunk <= n && !append_here;
  constexpr int NV = V_EARLY ? NT : 1;
  uint4 vreg[NV];
#pragma unroll
  for (int b0 = 0; b0 < NT; b0 += kTB) {
    uint4 kreg[kTB];
    load_rows<ROWB, RPW, kTB>(kreg, kbase, knew, row0 + b0 * RPW + sub, n, full, append_here, cl);
    if constexpr (V_EARLY)
      if (b0 == 0) load_rows<ROWB, RPW, NV>(vreg, vbase, vnew, row0 + sub, n, full, append_here, cl);
    // Logits: scale * q_g . K_j in base-2 units, one per (row, g).
#pragma unroll
    for (int i = 0; i < kTB; ++i) {
      float kf[EPL];
      Unpack<T>::run(kreg[i], kf);
      const int lr = wave * 64 + (b0 + i) * RPW + sub;   // row within the chunk
      const bool valid = c * kChunk + lr < n;
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float a = 0.0f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) a = fmaf(kf[e], qf[g][e], a);
        a = group_sum<LPR>(a);
        if (cl == 0) s_sh[g][lr] = valid ? a * P.scale_log2e : -INFINITY;
      }
    }
    if (append_here) store_appended<ROWB, RPW, kTB>(kreg, kbase, row0 + b0 * RPW + sub, n, cl);
  }
  if constexpr (V_EARLY)
    if (append_here) store_appended<ROWB, RPW, NV>(vreg, vbase, row0 + sub, n, cl);
  __syncthreads();

  // Chunk statistics.  Thread t owns row t of the chunk.
  float s_own[G], m_c[G], l_c[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    s_own[g] = s_sh[g][tid];
    const float wm = wave_max(s_own[g]);
    if (lane == 0) red_sh[0][g][wave] = wm;
  }
  __syncthreads();
  float* rec = P.ws + static_cast<int64_t>(bid) * REC;
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float m = red_sh[0][g][0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) m = fmaxf(m, red_sh[0][g][w]);
    m_c[g] = m;
    const float e = fast_exp2(s_own[g] - m);      // 0 for rows past the end
    s_sh[g][tid] = e;
    store_stream(&rec[g * kChunk + tid], e);
    const float ws = wave_sum(e);
    if (lane == 0) red_sh[1][g][wave] = ws;
  }
  __syncthreads();
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float l = red_sh[1][g][0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) l += red_sh[1][g][w];
    l_c[g] = l;
  }
  if (tid < G) {
    // tid selects the head: pick with a loop the compiler can unroll.
#pragma unroll
    for (int g = 0; g < G; ++g)
      if (g == tid) {
        store_stream(&rec[G * (kChunk + D) + 2 * g], m_c[g]);
        store_stream(&rec[G * (kChunk + D) + 2 * g + 1], l_c[g]);
      }
  }

  // Partial output: sum over this wave's rows of e_j V_j.
  float acc[G][EPL];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[g][e] = 0.0f;
#pragma unroll
  for (int b0 = 0; b0 < NT; b0 += kTB) {
    uint4 vlate[kTB];
    if constexpr (!V_EARLY) {
      load_rows<ROWB, RPW, kTB>(vlate, vbase, vnew, row0 + b0 * RPW + sub, n, full, append_here, cl);
      if (append_here) store_appended<ROWB, RPW, kTB>(vlate, vbase, row0 + b0 * RPW + sub, n, cl);
    }
#pragma unroll
    for (int i = 0; i < kTB; ++i) {
      float vf[EPL];
      if constexpr (V_EARLY) Unpack<T>::run(vreg[b0 + i], vf); else Unpack<T>::run(vlate[i], vf);
      const int lr = wave * 64 + (b0 + i) * RPW + sub;
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float p = s_sh[g][lr];
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(p, vf[e], acc[g][e]);
      }
    }
  }
  // Rows of a wave-wide load sit LPR lanes apart: fold them together.
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      float x = acc[g][e];
#pragma unroll
      for (int off = LPR; off < 64; off <<= 1) x += __shfl_xor(x, off);
      if (sub == 0) o_sh[wave][g][cl * EPL + e] = x;
    }
  __syncthreads();
  for (int idx = tid; idx < G * D; idx += kThreads) {
    const int g = idx / D, ch = idx - g * D;
    float o = o_sh[0][g][ch];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) o += o_sh[w][g][ch];
    store_stream(&rec[G * kChunk + idx], o);
  }
}

// ---------------------------------------------------------------------------
template <int D, int G>
__global__ __launch_bounds__(kThreads) void attend_finalize(const AttendParams P) {
  constexpr int REC = G * (kChunk + D + 2);
  constexpr int GD = G * D;
  extern __shared__ float dyn_sh[];         // [G][nchunks] chunk weights, then [G][nchunks] chunk sums
  __shared__ float red_sh[kWaves];
  __shared__ float o_red[kThreads];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int bid = blockIdx.x;

  // Region: last pair whose first finalize workgroup is <= bid.
  int lo = 0, hi = P.n_pairs - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (P.pairs[mid].fblock0 <= bid) lo = mid; else hi = mid - 1;
  }
  const PairDesc pd = P.pairs[lo];
  const int n = pd.n;
  const int nchunks = (n + kChunk - 1) / kChunk;
  const int nblk = nchunks > 0 ? (nchunks + kFinalChunks - 1) / kFinalChunks : 1;
  const int local = bid - pd.fblock0;
  const int h = local / nblk;
  const int blk = local - h * nblk;
  const int pair = P.pair_base + lo;
  float* out = P.out + (static_cast<int64_t>(pair) * P.n_kv_heads + h) * GD;
  if (n == 0) {
    for (int idx = tid; idx < GD; idx += kThreads) out[idx] = 0.0f;
    return;
  }
  const float* rec0 =
      P.ws + (static_cast<int64_t>(pd.block0) + static_cast<int64_t>(h) * nchunks) * REC;
  const int64_t stream_slot = pd.slot0 + static_cast<int64_t>(h) * pd.cap;
  float* score = P.score + stream_slot;
  float* w_sh = dyn_sh;
  float* l_sh = dyn_sh + G * nchunks;

  // Start the loads that do not depend on the statistics: the un-normalised
  // probabilities and the old scores of this workgroup's slots.
  float e_r[kFinalChunks][G], old_r[kFinalChunks];
#pragma unroll
  for (int i = 0; i < kFinalChunks; ++i) {
    const int c = blk * kFinalChunks + i;
    const int j = c * kChunk + tid;
    old_r[i] = 0.0f;
#pragma unroll
    for (int g = 0; g < G; ++g) e_r[i][g] = 0.0f;
    if (c < nchunks && j < n) {
#pragma unroll
      for (int g = 0; g < G; ++g) e_r[i][g] = rec0[static_cast<int64_t>(c) * REC + g * kChunk + tid];
      if (!(P.append && j == n - 1)) old_r[i] = score[j];   // the appended token starts from zero
    }
  }

  // Stream statistics from the chunk statistics.  Every workgroup of the stream
  // repeats this small reduction in the same order, so all agree bit for bit.
  for (int c = tid; c < nchunks; c += kThreads) {
    const float* ml = rec0 + static_cast<int64_t>(c) * REC + G * (kChunk + D);
#pragma unroll
    for (int g = 0; g < G; ++g) {
      w_sh[g * nchunks + c] = ml[2 * g];
      l_sh[g * nchunks + c] = ml[2 * g + 1];
    }
  }
  __syncthreads();
  for (int g = 0; g < G; ++g) {
    float m = -INFINITY;
    for (int c = tid; c < nchunks; c += kThreads) m = fmaxf(m, w_sh[g * nchunks + c]);
    m = wave_max(m);
    if (lane == 0) red_sh[wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(red_sh[0], red_sh[1]), fmaxf(red_sh[2], red_sh[3]));
    __syncthreads();
    float l = 0.0f;
    for (int c = tid; c < nchunks; c += kThreads) {
      const float wgt = fast_exp2(w_sh[g * nchunks + c] - m);
      w_sh[g * nchunks + c] = wgt;
      l += wgt * l_sh[g * nchunks + c];
    }
    l = wave_sum(l);
    if (lane == 0) red_sh[wave] = l;
    __syncthreads();
    l = (red_sh[0] + red_sh[1]) + (red_sh[2] + red_sh[3]);
    const float inv = 1.0f / l;
    for (int c = tid; c < nchunks; c += kThreads) w_sh[g * nchunks + c] *= inv;
    __syncthreads();
  }

  // score_j += sum_g e_gj w_gc
#pragma unroll
  for (int i = 0; i < kFinalChunks; ++i) {
    const int c = blk * kFinalChunks + i;
    const int j = c * kChunk + tid;
    if (c < nchunks && j < n) {
      float add = 0.0f;
#pragma unroll
      for (int g = 0; g < G; ++g) add = fmaf(e_r[i][g], w_sh[g * nchunks + c], add);
      score[j] = old_r[i] + add;
    }
  }
  if (P.append && blk == 0 && tid == 0) P.pos[stream_slot + n - 1] = P.pos_new[lo];

  // out = sum_c w_c o_c.  The G*D channels of the stream are split evenly over
  // its workgroups.  Within a workgroup the threads form (channel, slice)
  // pairs; a slice sums every S-th chunk, then the slices are added in order.
  const int cpb = (GD + nblk - 1) / nblk;
  const int ch_first = blk * cpb;
  const int nch = min(cpb, GD - ch_first);
  for (int tb = 0; tb < nch; tb += kThreads) {
    const int tn = min(kThreads, nch - tb);
    const int S = kThreads / tn;
    const int ch_l = tid % tn, slice = tid / tn;
    float o = 0.0f;
    if (slice < S) {
      const int idx = ch_first + tb + ch_l;
      const int g = idx / D;
      const float* col = rec0 + G * kChunk + idx;
#pragma unroll 4
      for (int c = slice; c < nchunks; c += S)
        o = fmaf(w_sh[g * nchunks + c], col[static_cast<int64_t>(c) * REC], o);
    }
    __syncthreads();
    o_red[tid] = o;
    __syncthreads();
    if (tid < tn) {
      float tot = o_red[tid];
      for (int sl = 1; sl < S; ++sl) tot += o_red[sl * tn + tid];
      out[ch_first + tb + tid] = tot;
    }
  }
}

// ---------------------------------------------------------------------------
using PartialFn = void (*)(const AttendParams);
using FinalizeFn = void (*)(const AttendParams);

template <typename T, int D>
bool pick_group(int group, PartialFn* pf, FinalizeFn* ff) {
  switch (group) {
    case 1: *pf = attend_partial<T, D, 1>; *ff = attend_finalize<D, 1>; return true;
    case 2: *pf = attend_partial<T, D, 2>; *ff = attend_finalize<D, 2>; return true;
    case 4: *pf = attend_partial<T, D, 4>; *ff = attend_finalize<D, 4>; return true;
    case 8: *pf = attend_partial<T, D, 8>; *ff = attend_finalize<D, 8>; return true;
    default: return false;
  }
}

bool pick_kernels(int dtype, int head_dim, int group, PartialFn* pf, FinalizeFn* ff) {
  if (dtype == XKV_F32 && head_dim == 64) return pick_group<F32, 64>(group, pf, ff);
  if (dtype == XKV_F32 && head_dim == 128) return pick_group<F32, 128>(group, pf, ff);
  if (dtype == XKV_BF16 && head_dim == 64) return pick_group<BF16, 64>(group, pf, ff);
  if (dtype == XKV_BF16 && head_dim == 128) return pick_group<BF16, 128>(group, pf, ff);
  return false;
}

}  // namespace
}  // namespace xkv

extern "C" xkv_status xkv_decode_attend_score(xkv_cache* cache, int32_t layer_begin,
                                              int32_t layer_end, const void* q, const void* k_new,
                                              const void* v_new, const int32_t* pos_new,
                                              float softmax_scale, float* out, void* workspace,
                                              size_t workspace_bytes, void* hip_stream) {
  using namespace xkv;
  xkv_status st = check_cache(cache);
  if (st != XKV_OK) return st;
  st = check_layers(cache, layer_begin, layer_end);
  if (st != XKV_OK) return st;
  if (q == nullptr || out == nullptr) return XKV_ERR_INVALID_ARG;
  if ((k_new == nullptr) != (v_new == nullptr)) return XKV_ERR_INVALID_ARG;
  const bool append = k_new != nullptr;
  if (append && pos_new == nullptr) return XKV_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(q) & 15u) || (reinterpret_cast<uintptr_t>(k_new) & 15u) ||
      (reinterpret_cast<uintptr_t>(v_new) & 15u))
    return XKV_ERR_INVALID_ARG;
  if (!(softmax_scale >= 0.0f) || std::isinf(softmax_scale)) return XKV_ERR_INVALID_ARG;

  const int B = cache->batch, hkv = cache->n_kv_heads, D = cache->head_dim;
  const int G = cache->n_q_heads / hkv;
  PartialFn partial = nullptr;
  FinalizeFn finalize = nullptr;
  if (!pick_kernels(cache->dtype, D, G, &partial, &finalize)) return XKV_ERR_UNSUPPORTED;

  const int64_t first = static_cast<int64_t>(layer_begin) * B;
  const int64_t n_pairs = static_cast<int64_t>(layer_end - layer_begin) * B;
  int64_t total_blocks = 0;
  int64_t max_chunks = 0;
  const int fin_chunks = kFinalChunks;
  for (int64_t i = 0; i < n_pairs; ++i) {
    const int64_t n = static_cast<int64_t>(cache->len[first + i]) + (append ? 1 : 0);
    if (n > cache->cap[first + i]) return XKV_ERR_CAPACITY;
    const int64_t chunks = ceil_div(n, kChunk);
    max_chunks = std::max(max_chunks, chunks);
    total_blocks += std::max<int64_t>(chunks, 1) * hkv;
  }
  const int64_t rec = attend_record_floats(G, D);
  if (workspace == nullptr) return XKV_ERR_INVALID_ARG;
  if (static_cast<uint64_t>(total_blocks) * rec * sizeof(float) > workspace_bytes)
    return XKV_ERR_CAPACITY;
  if (reinterpret_cast<uintptr_t>(workspace) & 3u) return XKV_ERR_INVALID_ARG;
  const size_t fin_lds = static_cast<size_t>(std::max<int64_t>(max_chunks, 1)) * G * 2 * sizeof(float);
  if (fin_lds > 48 * 1024) return XKV_ERR_UNSUPPORTED;

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const float scale = softmax_scale > 0.0f ? softmax_scale : 1.0f / std::sqrt(static_cast<float>(D));
  AttendParams P;
  P.q = q; P.k_new = k_new; P.v_new = v_new;
  P.k = cache->k; P.v = cache->v; P.score = cache->score; P.pos = cache->pos; P.out = out;
  P.scale_log2e = scale * 1.44269504088896340736f;
  P.n_kv_heads = hkv;
  P.append = append ? 1 : 0;

  int64_t blocks_done = 0;
  for (int64_t g0 = 0; g0 < n_pairs; g0 += kMaxPairs) {
    const int np = static_cast<int>(std::min<int64_t>(kMaxPairs, n_pairs - g0));
    int64_t blocks = 0, fblocks = 0;
    for (int i = 0; i < np; ++i) {
      const int64_t idx = first + g0 + i;
      PairDesc& pd = P.pairs[i];
      pd.slot0 = cache->region_off[idx];
      pd.cap = cache->cap[idx];
      pd.n = cache->len[idx] + (append ? 1 : 0);
      pd.block0 = static_cast<int32_t>(blocks);
      pd.fblock0 = static_cast<int32_t>(fblocks);
      P.pos_new[i] = append ? pos_new[(g0 + i) % B] : 0;
      const int64_t chunks = ceil_div(pd.n, kChunk);
      blocks += std::max<int64_t>(chunks, 1) * hkv;
      fblocks += std::max<int64_t>(ceil_div(chunks, fin_chunks), 1) * hkv;
    }
    if (blocks > std::numeric_limits<int32_t>::max()) return XKV_ERR_UNSUPPORTED;
    P.n_pairs = np;
    P.pair_base = static_cast<int32_t>(g0);
    P.ws = static_cast<float*>(workspace) + blocks_done * rec;
    const int tok = profile_begin(0, stream);
    hipLaunchKernelGGL(partial, dim3(static_cast<unsigned>(blocks)), dim3(kThreads), 0, stream, P);
    profile_end(tok, stream);
    if (hipGetLastError() != hipSuccess) return XKV_ERR_DEVICE;
    hipLaunchKernelGGL(finalize, dim3(static_cast<unsigned>(fblocks)), dim3(kThreads), fin_lds,
                       stream, P);
    if (hipGetLastError() != hipSuccess) return XKV_ERR_DEVICE;
    blocks_done += blocks;
  }
  if (append)
    for (int64_t i = 0; i < n_pairs; ++i) cache->len[first + i] += 1;
  return XKV_OK;
}
