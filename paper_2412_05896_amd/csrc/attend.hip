// xkv_decode_attend_score: decode attention over the ragged cache with
// per-token attention-mass scoring (Eq. 1 and Eq. 2 of the paper; scoring is the
// Select + Merge step of Eq. 3 with the decode query as observation row).
//
// A stream (layer, sequence, KV head) is cut into strips of `strip_rows` slots.
// Two or three kernels per call, no atomics, results bit-reproducible:
//
//  streaming kernel  one workgroup per (stream, strip).  Reads the strip's K and
//                    V rows once with 16-byte non-temporal loads and writes, per
//                    query head of the group: the logit of every slot, and the
//                    strip's softmax statistics (max m_s, sum l_s) and partial
//                    output o_s = sum_j 2^(s_j - m_s) V_j.  The workgroup that
//                    owns the last slot also stores the appended token.
//                    Three variants:
//                      attend_strip   (G <= 2) every wave runs its own online
//                                     softmax over interleaved groups of rows,
//                                     with the next group's loads in flight
//                                     while the current one is used; the four
//                                     waves merge once at the end; logits are
//                                     collected in LDS and written in one burst.
//                      attend_gqa     (G >= 4, bf16, 128 channels) logits and
//                                     output on the matrix cores (bf16 MFMA,
//                                     fp32 result); each wave runs its own
//                                     online softmax over tiles of 32 rows; a
//                                     tile's logits leave as one aligned block
//                                     of 16-bit distances below the tile's
//                                     reference (see the record layout below).
//                      attend_chunk   (other G >= 4 cases) strips of 256 slots
//                                     handled by the whole workgroup in one
//                                     pass; bf16 logits from MFMA.
//  attend_finalize   (attend_strip, attend_chunk) one workgroup per (stream, up
//                    to 4096 slots).  Merges the strip statistics of its stream
//                    into (m, l), adds p_j = 2^(s_j - m) / l, summed over the G
//                    query heads, to score[j] for its own slots, and computes
//                    its share of the channels of out = sum_s 2^(m_s - m) o_s / l.
//  attend_gqa_merge, attend_gqa_scores   (attend_gqa) the same work as two
//                    kernels: one workgroup per stream folds the strip records
//                    into (m, 1/l) and the output rows; then a streaming kernel
//                    over (stream, 1024 slots) adds the probabilities to the
//                    scores, reading 2 G bytes per slot.
//
// The ragged geometry travels in the kernel arguments: up to kMaxPairs (layer,
// sequence) regions directly, more through tables that small launches write into
// the workspace from their own arguments.  Nothing is copied from the host, the
// launches can be captured in a HIP graph, and a call is one streaming launch and
// one or two finishing launches whatever its size.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <limits>
#include <numeric>
#include <type_traits>
#include <vector>

#include "device_util.h"
#include "xkv_internal.h"

namespace xkv {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
constexpr int kMaxHeld = 64;            // strips one workgroup of the fused kernel can hold
// Longest strip of attend_gqa.  Every strip costs a record (partial outputs and
// statistics, G (D + 2) floats) that is stored inside the K/V stream and read again by the
// merge kernel: measured per decode step of the batched 16k and the 128k GQA workloads,
// 512 / 1024 / 2048 / 4096 slots: 3.83 / 3.78 / 3.75 / 3.75 ms and 4.90 / 4.77 / 4.66 / 4.61 ms.
constexpr int kGqaStripRows = 4096;
constexpr int kGqaScoreRows = 1024;      // slots per workgroup of attend_gqa_scores

struct PairDesc {
  int64_t slot0;    // first slot of the region
  int32_t cap;      // slots per stream
  int32_t n;        // live slots, the appended token included
  int32_t strip0;   // first strip record of the region in the launch's workspace (canonical order)
  int32_t full0;    // first streaming workgroup (fused kernel: queue position) among the full strips;
                    // in the finalize launch: first finalize workgroup of the region
};

// What every launch carries besides the geometry tables.
struct AttendCommon {
  const void* q;
  const void* k_new;
  const void* v_new;
  void* k;
  void* v;
  float* score;
  int32_t* pos;
  float* out;
  float* ws;              // first strip record of this launch
  float* stats;           // matrix-core path: (m, 1 / l) per (stream of the call, query head), written by
                          // attend_gqa_merge and read by attend_gqa_scores
  unsigned* barrier;      // fused kernel: {arrival count, timeout flag, queue head, unused}, zero at launch
  float scale_log2e;      // softmax scale times log2(e): logits live in the base-2 domain
  int32_t n_pairs;
  int32_t pair_base;      // index of pairs[0] relative to (layer_begin, sequence 0)
  int32_t n_kv_heads;
  int32_t append;
  int32_t strip_rows;     // slots per strip, a multiple of kChunk
  int32_t full_blocks;    // streaming workgroups that own a full strip; the rest own tail strips
  int32_t n_tail_pairs;   // regions whose streams end in a partial strip
  int32_t rec_floats;     // floats per strip record in the workspace
  int32_t lds_rows;       // fused kernel: rows of logits a workgroup can hold
  int32_t fin_strips;     // finalize kernel: strips per workgroup
  int32_t fin_rows;       // attend_gqa_scores: slots per workgroup (a power of two, any relation to strip_rows)
  uint32_t spin_limit;    // fused kernel: polls of the grid-wide wait before a workgroup gives up
};

// Geometry of up to kMaxPairs regions inside the kernel arguments: nothing is
// copied to the device for such a call.
struct AttendParams : AttendCommon {
  PairDesc pairs[kMaxPairs];
  int32_t pos_new[kMaxPairs];    // original position of the token appended to each region
  uint8_t tail_order[kMaxPairs]; // regions with a partial last strip, longest tail first
};

// Geometry of a call with more regions: the same tables in device memory (in the
// caller's workspace, written there by table_write launches), so that the whole
// call is still one streaming launch and one finalize launch.
struct AttendTableParams : AttendCommon {
  const PairDesc* pairs;
  const int32_t* pos_new;
  const int32_t* tail_order;
  const int32_t* fin0;           // first finalize workgroup of each region
};

// The finalize kernel that also evicts (xkv_decode_step): the attention geometry plus,
// per region, the number of tokens to keep.
struct StepParams : AttendParams {
  int32_t keep[kMaxPairs];   // min(budget, n) of every region
  int32_t* kept_idx;         // may be null
  int32_t row_bytes;
  int32_t pool, n_protect;   // as for xkv_evict_compact
};
struct StepTableParams : AttendTableParams {
  const int32_t* keep;       // the same, in device memory (it takes the place of fin0, which these kernels do not use)
  int32_t* kept_idx;
  int32_t row_bytes;
  int32_t pool, n_protect;
};

// First finalize workgroup of region i: with the tables in the arguments the host
// rewrites full0 between the two launches.
__device__ __forceinline__ int fin_first(const AttendParams& P, int i) { return P.pairs[i].full0; }
__device__ __forceinline__ int fin_first(const AttendTableParams& P, int i) { return P.fin0[i]; }

// Floats per strip record: per query head, strip_rows logits, D partial outputs,
// (m, l); padded so that every record starts on a 128-byte line.
__host__ __device__ inline int64_t record_floats(int group, int head_dim, int strip_rows) {
  return (static_cast<int64_t>(group) * (strip_rows + head_dim + 2) + 31) / 32 * 32;
}

// Strip record of the matrix-core path (attend_gqa).  A probability leaves the
// streaming kernel as a 16-bit fixed-point distance d = (m_tile - s) * 2^10 of its
// base-2 logit s below a reference m_tile that is stored once per tile of 32 slots
// and query head (the wave's running maximum when it reached the tile), so that
// p = 2^(m_tile - d / 2^10 - m) / l later: half the bytes of an fp32 logit, a
// relative error of at most ln 2 * 2^-11 = 3.4e-4 on every probability whatever
// its size, and distances beyond 64 (probabilities below 2^-64 of the tile's
// reference) saturate.  In floats: d16[strip_rows][G] (two per float), then
// m_tile[strip_rows / 32][G], then o[G][D] and (m, l)[G]; padded to a 128-byte line.
constexpr int kGqaTile = 32;
constexpr float kLogitFixScale = 1024.0f;
// attend_gqa holds its distances back in LDS (this many bytes per workgroup) and writes them in chip-wide
// bursts: all waves of the chip flush when the wall clock (s_memrealtime, 100 MHz) enters a new window of
// this many ticks, or when their buffer is full.  Stores that trickle into a read stream cost read bandwidth
// far beyond their volume; arriving together they cost about half of that (read-only probe with 4 KiB stored
// per 128 KiB read: 5.9 TB/s written at once, 6.1 held back per workgroup, 6.4 in windows of 40-80 us, 7.2
// without).  The window is as long as the buffer allows: a wave fills 32 tiles (G = 4) in about 130 us, 16
// tiles (G = 8) in about 65 us.
constexpr int kGqaHeldBytesG4 = 32 * 1024, kGqaHeldBytesG8 = 48 * 1024;
constexpr unsigned long long kStoreWindowTicksG4 = 12000, kStoreWindowTicksG8 = 6000;
__host__ __device__ inline int64_t gqa_tilem_offset(int group, int strip_rows) {
  return static_cast<int64_t>(strip_rows) * group / 2;
}
__host__ __device__ inline int64_t gqa_out_offset(int group, int strip_rows) {
  return gqa_tilem_offset(group, strip_rows) + static_cast<int64_t>(strip_rows / kGqaTile) * group;
}
__host__ __device__ inline int64_t gqa_record_floats(int group, int head_dim, int strip_rows) {
  return (gqa_out_offset(group, strip_rows) + static_cast<int64_t>(group) * (head_dim + 2) + 31) / 32 * 32;
}

// Strip record of attend_strip over bf16 caches: the logits leave as 16-bit
// fixed-point distances d = (m_s - s) * 2^10 below the strip's own maximum m_s
// (which the record holds anyway), two per float, [head][slot]; then o[G][D] and
// (m, l)[G].  Same precision argument as above; fp32 caches keep fp32 logits.
__host__ __device__ inline int64_t half_record_floats(int group, int head_dim, int strip_rows) {
  return (static_cast<int64_t>(group) * (strip_rows / 2 + head_dim + 2) + 31) / 32 * 32;
}

struct StripWork { int pair_local, h, s; };

// Streaming kernels: full strips first (all the same size), then the partial
// last strips of the streams, longest first, so that short work fills the end
// of the launch.
template <typename PT>
__device__ __forceinline__ StripWork locate_stream_block(const PT& P, int bid) {
  StripWork w;
  if (bid < P.full_blocks) {
    int lo = 0, hi = P.n_pairs - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (P.pairs[mid].full0 <= bid) lo = mid; else hi = mid - 1;
    }
    const int nfull = P.pairs[lo].n / P.strip_rows;
    const int local = bid - P.pairs[lo].full0;
    w.pair_local = lo;
    w.h = local / nfull;
    w.s = local - w.h * nfull;
  } else {
    const int t = bid - P.full_blocks;
    w.pair_local = P.tail_order[t / P.n_kv_heads];
    w.h = t % P.n_kv_heads;
    w.s = P.pairs[w.pair_local].n / P.strip_rows;
  }
  return w;
}

// Loads kNB consecutive wave-wide fragments of a stream (rows first_row,
// first_row + RPW, ...) into registers, without branches: rows at or past n are
// clamped to row n-1 (in bounds; their logits are masked later and their
// probabilities are zero), and with append_here every lane that ends up on row
// n-1, clamped ones included, reads the token being appended from `newrow`
// instead of the not yet written slot: whatever that slot holds (the arenas are
// the caller's; a dead slot may hold any bit pattern, NaN included) never
// reaches a register, so 0 * V stays 0.
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
      if (append_here && rc == n - 1) src = newrow + cl * 16;
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

// Addresses shared by the streaming kernels.
template <typename T, int D, int G>
struct StreamCtx {
  static constexpr int EPL = T::kPerLane;    // elements per lane per load
  static constexpr int LPR = D / EPL;        // lanes that cover one row
  static constexpr int RPW = 64 / LPR;       // rows per wave-wide load
  static constexpr int ROWB = D * T::kBytes; // bytes per row
  int n, h, s, pair;
  char* kbase;
  char* vbase;
  const char* knew;
  const char* vnew;
  bool append_here;
  float* rec;                                // this strip's record

  // Stream (region pair_local, head h_) of the launch; append_here says whether
  // the caller's row range may hold the appended token.
  template <typename PT>
  __device__ __forceinline__ void init_stream(const PT& P, int pair_local, int h_, bool may_append) {
    const PairDesc pd = P.pairs[pair_local];
    n = pd.n; h = h_; s = 0;
    pair = P.pair_base + pair_local;
    const int64_t stream_slot = pd.slot0 + static_cast<int64_t>(h) * pd.cap;
    kbase = static_cast<char*>(P.k) + stream_slot * ROWB;
    vbase = static_cast<char*>(P.v) + stream_slot * ROWB;
    append_here = P.append && may_append;
    knew = vnew = nullptr;
    if (append_here) {
      const int64_t r = (static_cast<int64_t>(pair) * P.n_kv_heads + h) * ROWB;
      knew = static_cast<const char*>(P.k_new) + r;
      vnew = static_cast<const char*>(P.v_new) + r;
    }
    rec = nullptr;
  }
  template <typename PT>
  __device__ __forceinline__ void init(const PT& P, const StripWork& wk) {
    const PairDesc pd = P.pairs[wk.pair_local];
    const int nstrips = (pd.n + P.strip_rows - 1) / P.strip_rows;
    init_stream(P, wk.pair_local, wk.h, wk.s == nstrips - 1);   // row n-1 lies in the last strip
    s = wk.s;
    rec = P.ws + (static_cast<int64_t>(pd.strip0) + static_cast<int64_t>(h) * nstrips + s) * P.rec_floats;
  }
  // Queries of the group, widened to fp32, this lane's columns only.
  template <typename PT>
  __device__ __forceinline__ void load_q(const PT& P, int cl, float (&qf)[G][EPL]) const {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const int64_t hq = (static_cast<int64_t>(pair) * P.n_kv_heads + h) * G + g;
      const uint4 raw =
          *reinterpret_cast<const uint4*>(static_cast<const char*>(P.q) + hq * ROWB + cl * 16);
      Unpack<T>::run(raw, qf[g]);
    }
  }
};

// ---------------------------------------------------------------------------
// One pass of a workgroup over rows [r_begin, r_end) of one stream.  A round is
// TPI wave-wide loads of K and of V per wave (TPI * RPW rows), the four waves
// taking consecutive row groups.  Each wave keeps its own running (m, l, o) and
// rescales them when the maximum moves; two register buffers alternate so that
// the loads of round r+1 are in flight while round r is computed.  The logits go
// to LDS (lg[g * lg_stride + row - r_begin]); the four waves merge at the end
// and the segment's partial output o[G][D] and statistics ml[G][2] are written
// with `put`.  Ends with a barrier, after which mrg_sh may be reused.
template <typename T, int D, int G, int TPI, typename PT, typename Put>
__device__ __forceinline__ void segment_pass(const PT& P, const StreamCtx<T, D, G>& cx,
                                             int r_begin, int r_end, float* lg, int lg_stride,
                                             float (*mrg_sh)[G][D + 2], float* rec_o, float* rec_ml,
                                             Put put, float* m_out_sh = nullptr) {
  using Ctx = StreamCtx<T, D, G>;
  constexpr int EPL = Ctx::EPL, LPR = Ctx::LPR, RPW = Ctx::RPW, ROWB = Ctx::ROWB;
  constexpr int RPI = TPI * RPW;            // rows per wave per round
  constexpr int RPR = RPI * kWaves;         // rows per workgroup per round

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int sub = lane / LPR;               // row within a wave-wide load
  const int cl = lane % LPR;                // 16-byte column of the row
  const int n = cx.n;
  const int rows = r_end - r_begin;
  const int rounds = (rows + RPR - 1) / RPR;
  const bool append_here = cx.append_here && r_end == n;   // this segment holds row n-1
  const int n_plain = n - (append_here ? 1 : 0);           // rows below this come straight from the cache

  float qf[G][EPL];
  cx.load_q(P, cl, qf);

  float m_run[G], l_run[G], acc[G][EPL];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m_run[g] = -INFINITY;
    l_run[g] = 0.0f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[g][e] = 0.0f;
  }

  struct Buf { uint4 k[TPI]; uint4 v[TPI]; };
  auto issue = [&](Buf& b, int round) {
    const int first = r_begin + round * RPR + wave * RPI;
    const bool full = first + RPI <= n_plain;
    load_rows<ROWB, RPW, TPI>(b.k, cx.kbase, cx.knew, first + sub, n, full, append_here, cl);
    load_rows<ROWB, RPW, TPI>(b.v, cx.vbase, cx.vnew, first + sub, n, full, append_here, cl);
  };
  auto compute = [&](Buf& b, int round) {
    const int first = r_begin + round * RPR + wave * RPI + sub;
    float sv[TPI][G];
#pragma unroll
    for (int i = 0; i < TPI; ++i) {
      float kf[EPL];
      Unpack<T>::run(b.k[i], kf);
      const int row = first + i * RPW;
      const bool valid = row < r_end;
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float a = 0.0f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) a = fmaf(kf[e], qf[g][e], a);
        a = group_sum<LPR>(a);
        sv[i][g] = valid ? a * P.scale_log2e : -INFINITY;
        if (cl == 0 && valid) lg[g * lg_stride + (row - r_begin)] = sv[i][g];
      }
    }
    float pv[TPI][G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float gm = sv[0][g];
#pragma unroll
      for (int i = 1; i < TPI; ++i) gm = fmaxf(gm, sv[i][g]);
#pragma unroll
      for (int off = LPR; off < 64; off <<= 1) gm = fmaxf(gm, __shfl_xor(gm, off));
      const float m_new = fmaxf(m_run[g], gm);
      const float m_safe = m_new == -INFINITY ? 0.0f : m_new;   // a wave may see no live row at all
      const float rescale = fast_exp2(m_run[g] - m_safe);
      m_run[g] = m_new;
      float l = l_run[g] * rescale;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[g][e] *= rescale;
#pragma unroll
      for (int i = 0; i < TPI; ++i) {
        pv[i][g] = fast_exp2(sv[i][g] - m_safe);
        l += pv[i][g];
      }
      l_run[g] = l;
    }
#pragma unroll
    for (int i = 0; i < TPI; ++i) {
      float vf[EPL];
      Unpack<T>::run(b.v[i], vf);
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(pv[i][g], vf[e], acc[g][e]);
    }
    if (append_here) {
      store_appended<ROWB, RPW, TPI>(b.k, cx.kbase, first, n, cl);
      store_appended<ROWB, RPW, TPI>(b.v, cx.vbase, first, n, cl);
    }
  };

  Buf A, B;
  issue(A, 0);
  for (int r = 0; r < rounds; r += 2) {
    if (r + 1 < rounds) issue(B, r + 1);
    compute(A, r);
    if (r + 1 < rounds) {
      if (r + 2 < rounds) issue(A, r + 2);
      compute(B, r + 1);
    }
  }

  // Fold the row groups of the wave together (each lane so far summed only the
  // rows of its own group), then merge the four waves.
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float l = l_run[g];
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) l += __shfl_xor(l, off);
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      float x = acc[g][e];
#pragma unroll
      for (int off = LPR; off < 64; off <<= 1) x += __shfl_xor(x, off);
      if (sub == 0) mrg_sh[wave][g][cl * EPL + e] = x;
    }
    if (lane == 0) {
      mrg_sh[wave][g][D] = m_run[g];
      mrg_sh[wave][g][D + 1] = l;
    }
  }
  __syncthreads();
  for (int idx = tid; idx < G * (D + 1); idx += kThreads) {
    const int g = idx / (D + 1), ch = idx - g * (D + 1);     // ch == D: the sum l
    float m = mrg_sh[0][g][D];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) m = fmaxf(m, mrg_sh[w][g][D]);
    const int col = ch < D ? ch : D + 1;
    float tot = 0.0f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) tot += mrg_sh[w][g][col] * fast_exp2(mrg_sh[w][g][D] - m);
    if (ch < D) {
      put(&rec_o[g * D + ch], tot);
    } else {
      put(&rec_ml[2 * g], m);
      put(&rec_ml[2 * g + 1], tot);
      if (m_out_sh != nullptr) m_out_sh[g] = m;
    }
  }
  __syncthreads();
}

// ---------------------------------------------------------------------------
// Strip kernel for small query groups: one workgroup per (stream, strip); the
// strip's logits are collected in LDS and written in one burst.
template <typename T, int D, int G, int TPI, typename PT = AttendParams>
__global__ __launch_bounds__(kThreads) void attend_strip(const PT P) {
  constexpr bool kHalf = std::is_same<T, BF16>::value;   // 16-bit distances instead of fp32 logits
  extern __shared__ float lg_sh[];          // [G][strip_rows] logits of the strip
  __shared__ float mrg_sh[kWaves][G][D + 2];
  __shared__ float m_sh[G];                 // the strip's maxima

  StreamCtx<T, D, G> cx;
  cx.init(P, locate_stream_block(P, blockIdx.x));
  const int strip_rows = P.strip_rows;
  const int r_begin = cx.s * strip_rows;
  const int r_end = min(cx.n, r_begin + strip_rows);
  const int rows = r_end - r_begin;
  float* rec = cx.rec;
  const int lg_floats = kHalf ? strip_rows / 2 : strip_rows;   // floats of logit data per head in the record
  segment_pass<T, D, G, TPI>(P, cx, r_begin, r_end, lg_sh, strip_rows, mrg_sh,
                             rec + G * lg_floats, rec + G * (lg_floats + D),
                             [](float* p, float v) { store_stream(p, v); }, m_sh);
  if constexpr (kHalf) {
    // two slots per 32-bit word; an odd last slot is paired with a saturated distance
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float m = m_sh[g];
      for (int j = threadIdx.x; 2 * j < rows; j += kThreads) {
        const float s0 = lg_sh[g * strip_rows + 2 * j];
        const float s1 = 2 * j + 1 < rows ? lg_sh[g * strip_rows + 2 * j + 1] : -INFINITY;
        const unsigned d0 = __float2uint_rn(fminf((m - s0) * kLogitFixScale, 65535.0f));
        const unsigned d1 = __float2uint_rn(fminf((m - s1) * kLogitFixScale, 65535.0f));
        store_stream(&rec[g * lg_floats + j], __uint_as_float(d0 | (d1 << 16)));
      }
    }
  } else {
#pragma unroll
    for (int g = 0; g < G; ++g)
      for (int j = threadIdx.x; j < rows; j += kThreads)
        store_stream(&rec[g * strip_rows + j], lg_sh[g * strip_rows + j]);
  }
}

// ---------------------------------------------------------------------------
// Fused kernel: the whole call in one cooperative launch, nothing but strip-sized
// records written while K and V stream in.  The strips of the launch (numbered
// as for the streaming kernels: full strips first, then the partial ones,
// longest first) form a queue; every workgroup takes strips from it for as long
// as its LDS has room for another strip's logits, runs the pass over each and
// publishes the strip's (o, m, l) record.  After a grid-wide barrier each
// workgroup merges the records of the streams its strips belong to, turns the
// logits it holds into probabilities and adds them to the scores; the holder of a
// stream's first strip writes the stream's output.  The K/V read is thus free of
// concurrent per-token write traffic, which on this GPU costs read bandwidth far
// beyond its volume.
//
// Grid-wide barrier for a cooperative launch (all workgroups resident).  The
// counter starts at zero; every workgroup adds one and waits until all have.
// No cache maintenance is tied to it: what crosses it (the strip records) is
// written and read with agent-scope accesses that bypass the per-XCD caches, and
// the barrier before the count makes sure those writes have been acknowledged.
// The wait is bounded: should the count not fill within spin_limit polls (it
// always does, unless the launch was not resident), the workgroup gives up and
// raises the flag next to the counter, so the kernel always ends.  Returns, to
// every thread, whether the flag was up when this workgroup left the wait: the
// strip records may then be incomplete, and the caller must not use them.
__device__ __forceinline__ bool grid_barrier(unsigned* counter, unsigned n_wgs, unsigned spin_limit,
                                             int* flag_sh) {
  __syncthreads();
  if (threadIdx.x == 0) {
    __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    unsigned spins = 0;
    while (__hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < n_wgs) {
      if (spins++ >= spin_limit) {
        __hip_atomic_store(counter + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        break;
      }
      __builtin_amdgcn_s_sleep(4);
    }
    *flag_sh = static_cast<int>(__hip_atomic_load(counter + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
  }
  __syncthreads();
  return *flag_sh != 0;
}

// control words of a fused launch: {barrier count, barrier timeout flag, queue head, unused}
__global__ void fused_prepare(unsigned* control) {
  if (threadIdx.x < 4) control[threadIdx.x] = 0u;
}

__device__ __forceinline__ float load_agent(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <typename T, int D, int G, int TPI>
__global__ __launch_bounds__(kThreads) void attend_fused(const AttendParams P) {
  constexpr int SEG = G * (D + 2);          // floats per strip record: o[G][D], (m, l)[G]
  extern __shared__ float lg_sh[];          // [G][lds_rows] logits of the strips held
  __shared__ float mrg_sh[kWaves][G][D + 2];
  __shared__ float red_sh[2][G][kWaves];
  __shared__ float st_sh[G][2];
  __shared__ int held_sh[kMaxHeld];         // queue positions of the strips held
  __shared__ int next_sh;
  __shared__ int gave_up_sh;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int strip_rows = P.strip_rows;
  const int lds_rows = P.lds_rows;
  const int n_units = P.full_blocks + P.n_tail_pairs * P.n_kv_heads;
  unsigned* queue = P.barrier + 2;

  // ---- phase 1: take strips while there is room; logits to LDS, one record each ----
  int n_held = 0;
  while (n_held < kMaxHeld && (n_held + 1) * strip_rows <= lds_rows) {
    if (tid == 0)
      next_sh = static_cast<int>(__hip_atomic_fetch_add(queue, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    __syncthreads();
    const int unit = next_sh;
    __syncthreads();
    if (unit >= n_units) break;
    if (tid == 0) held_sh[n_held] = unit;
    StreamCtx<T, D, G> cx;
    cx.init(P, locate_stream_block(P, unit));
    const int r_begin = cx.s * strip_rows;
    const int r_end = min(cx.n, r_begin + strip_rows);
    segment_pass<T, D, G, TPI>(P, cx, r_begin, r_end, lg_sh + n_held * strip_rows, lds_rows, mrg_sh,
                               cx.rec, cx.rec + G * D, [](float* p, float v) {
                                 __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                               });
    ++n_held;
  }
  if (grid_barrier(P.barrier, gridDim.x, P.spin_limit, &gave_up_sh)) {
    // Some workgroup gave up waiting: records may be missing.  Nothing is merged;
    // the output rows of the streams this workgroup holds strips of become NaN and
    // their scores stay as they were.  The host reads the flag with
    // xkv_fused_status.
    for (int k = 0; k < n_held; ++k) {
      const StripWork wk = locate_stream_block(P, held_sh[k]);
      float* out = P.out + (static_cast<int64_t>(P.pair_base + wk.pair_local) * P.n_kv_heads + wk.h) * G * D;
      for (int idx = tid; idx < G * D; idx += kThreads) out[idx] = __builtin_nanf("");
    }
    return;
  }

  // ---- phase 2: normalise, add to the scores, write the outputs -----------------
  for (int k = 0; k < n_held; ++k) {
    const StripWork wk = locate_stream_block(P, held_sh[k]);
    const PairDesc pd = P.pairs[wk.pair_local];
    const int n = pd.n;
    const int nstrips = (n + strip_rows - 1) / strip_rows;
    const float* rec0 = P.ws + (static_cast<int64_t>(pd.strip0) + static_cast<int64_t>(wk.h) * nstrips) * SEG;
    // Stream statistics from the strip statistics, 256 strips at a time.
    float m_run[G], l_run[G];
#pragma unroll
    for (int g = 0; g < G; ++g) { m_run[g] = -INFINITY; l_run[g] = 0.0f; }
    for (int base = 0; base < nstrips; base += kThreads) {
      const int c = base + tid;
      float mc[G], lc[G];
#pragma unroll
      for (int g = 0; g < G; ++g) {
        mc[g] = -INFINITY;
        lc[g] = 0.0f;
        if (c < nstrips) {
          mc[g] = load_agent(rec0 + static_cast<int64_t>(c) * SEG + G * D + 2 * g);
          lc[g] = load_agent(rec0 + static_cast<int64_t>(c) * SEG + G * D + 2 * g + 1);
        }
      }
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float wm = wave_max(mc[g]);
        if (lane == 0) red_sh[0][g][wave] = wm;
      }
      __syncthreads();
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float m_new = m_run[g];
#pragma unroll
        for (int w = 0; w < kWaves; ++w) m_new = fmaxf(m_new, red_sh[0][g][w]);
        const float contrib = lc[g] * fast_exp2(mc[g] - m_new);     // m_new is finite: some strip has a live row
        const float wsum = wave_sum(contrib);
        if (lane == 0) red_sh[1][g][wave] = wsum;
        l_run[g] *= fast_exp2(m_run[g] - m_new);
        m_run[g] = m_new;
      }
      __syncthreads();
#pragma unroll
      for (int g = 0; g < G; ++g) {
#pragma unroll
        for (int w = 0; w < kWaves; ++w) l_run[g] += red_sh[1][g][w];
      }
      __syncthreads();
    }
    if (tid == 0) {
#pragma unroll
      for (int g = 0; g < G; ++g) { st_sh[g][0] = m_run[g]; st_sh[g][1] = 1.0f / l_run[g]; }
    }
    __syncthreads();

    const int r_begin = wk.s * strip_rows;
    const int r_end = min(n, r_begin + strip_rows);
    const int64_t stream_slot = pd.slot0 + static_cast<int64_t>(wk.h) * pd.cap;
    float* score = P.score + stream_slot;
    const float* lg = lg_sh + k * strip_rows;
    // Batches of eight rows per thread: all eight score loads go out before the first is used.
    for (int j0 = tid; j0 < r_end - r_begin; j0 += 8 * kThreads) {
      float old[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int row = r_begin + j0 + u * kThreads;
        old[u] = (row < r_end && !(P.append && row == n - 1)) ? score[row] : 0.0f;   // the appended token starts from zero
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int jj = j0 + u * kThreads;
        if (r_begin + jj < r_end) {
          float add = 0.0f;
#pragma unroll
          for (int g = 0; g < G; ++g) add = fmaf(fast_exp2(lg[g * lds_rows + jj] - st_sh[g][0]), st_sh[g][1], add);
          score[r_begin + jj] = old[u] + add;
        }
      }
    }
    if (P.append && r_end == n && tid == 0) P.pos[stream_slot + n - 1] = P.pos_new[wk.pair_local];
    if (wk.s == 0) {
      const int pair = P.pair_base + wk.pair_local;
      float* out = P.out + (static_cast<int64_t>(pair) * P.n_kv_heads + wk.h) * G * D;
      for (int idx = tid; idx < G * D; idx += kThreads) {
        const int g = idx / D;
        float o = 0.0f;
#pragma unroll 4
        for (int c = 0; c < nstrips; ++c) {
          const float* r = rec0 + static_cast<int64_t>(c) * SEG;
          o = fmaf(load_agent(r + idx), fast_exp2(load_agent(r + G * D + 2 * g) - st_sh[g][0]), o);
        }
        out[idx] = o * st_sh[g][1];
      }
    }
    __syncthreads();
  }
  // Streams without a live slot: zero output rows.
  if (blockIdx.x == 0)
    for (int p = 0; p < P.n_pairs; ++p)
      if (P.pairs[p].n == 0) {
        float* out = P.out + static_cast<int64_t>(P.pair_base + p) * P.n_kv_heads * G * D;
        for (int idx = tid; idx < P.n_kv_heads * G * D; idx += kThreads) out[idx] = 0.0f;
      }
}

// ---------------------------------------------------------------------------
// Chunk kernel for larger query groups: strips are kChunk slots, the workgroup
// makes one pass (thread t owns slot t for the statistics).
template <typename T, int D, int G, typename PT = AttendParams>
__global__ __launch_bounds__(kThreads) void attend_chunk(const PT P) {
  using Ctx = StreamCtx<T, D, G>;
  constexpr int EPL = Ctx::EPL, LPR = Ctx::LPR, RPW = Ctx::RPW, ROWB = Ctx::ROWB;
  constexpr int NT = 64 / RPW;              // loads per wave for its 64 rows
  constexpr int kTB = NT < 16 ? NT : 16;    // wave-wide loads in flight per batch

  __shared__ float s_sh[G][kChunk];         // logits, then probabilities
  __shared__ float red_sh[2][G][kWaves];
  __shared__ float o_sh[kWaves][G][D];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int sub = lane / LPR;
  const int cl = lane % LPR;

  Ctx cx;
  cx.init(P, locate_stream_block(P, blockIdx.x));
  const int n = cx.n, c = cx.s;
  const int row0 = c * kChunk + wave * 64;
  const bool append_here = cx.append_here;
  const bool full = (c + 1) * kChunk <= n && !append_here;

  // V rows: issued together with the K rows so that they arrive during the
  // logit and statistics phases.
  uint4 vreg[NT];
  if constexpr (std::is_same<T, BF16>::value) {
    // Logits on the matrix cores: S[g][t] = sum_c Q[g][c] K[t][c] as D = A * B with
    // A = the query group (rows g < G, zero rows up to 16) and B = 16 K rows.  In
    // both operands lane (j, x) = (lane / 16, lane % 16) holds 8 consecutive
    // channels 32 s + 8 j .. of row x for contraction slice s, so a K operand is a
    // 16-byte load straight from the cache row: no staging.  The result has
    // S[4 j + i][t = lane % 16] in register i of lane (j, t).
    constexpr int NS = D / 32;              // contraction slices of 32 channels
    const int x16 = lane & 15, j4 = lane >> 4;
    bf16x8 qa[NS];
#pragma unroll
    for (int sl = 0; sl < NS; ++sl) {
      uint4 raw = make_uint4(0, 0, 0, 0);
      if (x16 < G) {
        const int64_t hq = (static_cast<int64_t>(cx.pair) * P.n_kv_heads + cx.h) * G + x16;
        raw = *reinterpret_cast<const uint4*>(static_cast<const char*>(P.q) + hq * ROWB + sl * 64 + j4 * 16);
      }
      qa[sl] = __builtin_bit_cast(bf16x8, raw);
    }
    load_rows<ROWB, RPW, NT>(vreg, cx.vbase, cx.vnew, row0 + sub, n, full, append_here, cl);
    // The wave's 64 rows are 4 groups of 16; two groups of K operands are in flight at a time.
#pragma unroll
    for (int g0 = 0; g0 < 4; g0 += 2) {
      uint4 kb[2][NS];
#pragma unroll
      for (int gi = 0; gi < 2; ++gi) {
        const int r = row0 + (g0 + gi) * 16 + x16;
        const int rc = r < n ? r : n - 1;
        const char* src = cx.kbase + static_cast<int64_t>(rc) * ROWB + j4 * 16;
        if (append_here && rc == n - 1) src = cx.knew + j4 * 16;
#pragma unroll
        for (int sl = 0; sl < NS; ++sl) kb[gi][sl] = load_stream16(src + sl * 64);
      }
#pragma unroll
      for (int gi = 0; gi < 2; ++gi) {
        floatx4 acc4 = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int sl = 0; sl < NS; ++sl)
          acc4 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qa[sl], __builtin_bit_cast(bf16x8, kb[gi][sl]), acc4, 0, 0, 0);
        const int lr = wave * 64 + (g0 + gi) * 16 + x16;
        const int r = c * kChunk + lr;
        const bool valid = r < n;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int g = 4 * j4 + i;
          if (g < G) s_sh[g][lr] = valid ? acc4[i] * P.scale_log2e : -INFINITY;
        }
        if (append_here && r == n - 1) {    // the append itself, K part
#pragma unroll
          for (int sl = 0; sl < NS; ++sl)
            *reinterpret_cast<uint4*>(cx.kbase + static_cast<int64_t>(r) * ROWB + sl * 64 + j4 * 16) = kb[gi][sl];
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  } else {
    float qf[G][EPL];
    cx.load_q(P, cl, qf);
#pragma unroll
    for (int b0 = 0; b0 < NT; b0 += kTB) {
      uint4 kreg[kTB];
      load_rows<ROWB, RPW, kTB>(kreg, cx.kbase, cx.knew, row0 + b0 * RPW + sub, n, full, append_here, cl);
      if (b0 + kTB >= NT)
        load_rows<ROWB, RPW, NT>(vreg, cx.vbase, cx.vnew, row0 + sub, n, full, append_here, cl);
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
      if (append_here) store_appended<ROWB, RPW, kTB>(kreg, cx.kbase, row0 + b0 * RPW + sub, n, cl);
    }
  }
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
  float* rec = cx.rec;
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float m = red_sh[0][g][0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) m = fmaxf(m, red_sh[0][g][w]);
    m_c[g] = m;
    const float e = fast_exp2(s_own[g] - m);      // 0 for rows past the end
    s_sh[g][tid] = e;
    store_stream(&rec[g * kChunk + tid], s_own[g]);
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
#pragma unroll
    for (int g = 0; g < G; ++g)
      if (g == tid) {
        store_stream(&rec[G * (kChunk + D) + 2 * g], m_c[g]);
        store_stream(&rec[G * (kChunk + D) + 2 * g + 1], l_c[g]);
      }
  }

  // Partial output: sum over this wave's rows of e_j V_j, at most four query
  // heads at a time (the V registers are reused), which keeps the accumulators
  // small enough for several waves per SIMD.
  constexpr int GP = G > 4 ? 4 : G;
  if (append_here) store_appended<ROWB, RPW, NT>(vreg, cx.vbase, row0 + sub, n, cl);
#pragma unroll
  for (int gp = 0; gp < G; gp += GP) {
    float acc[GP][EPL];
#pragma unroll
    for (int g = 0; g < GP; ++g)
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[g][e] = 0.0f;
#pragma unroll
    for (int i = 0; i < NT; ++i) {
      float vf[EPL];
      Unpack<T>::run(vreg[i], vf);
      const int lr = wave * 64 + i * RPW + sub;
#pragma unroll
      for (int g = 0; g < GP; ++g) {
        const float p = s_sh[gp + g][lr];
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(p, vf[e], acc[g][e]);
      }
      // Keeps the compiler from gathering the probability reads of all rows first
      // (it would interchange the loops and hold them all in registers).
      asm volatile("" ::: "memory");
    }
    // Rows of a wave-wide load sit LPR lanes apart: fold them together.
#pragma unroll
    for (int g = 0; g < GP; ++g) {
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        float x = acc[g][e];
#pragma unroll
        for (int off = LPR; off < 64; off <<= 1) x += __shfl_xor(x, off);
        if (sub == 0) o_sh[wave][gp + g][cl * EPL + e] = x;
      }
    }
    __builtin_amdgcn_sched_barrier(0);
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
// Streaming kernel for query groups of 4 and 8 over bf16 rows of 128 channels:
// both contractions run on the matrix cores (16x16x32 bf16 MFMA, fp32 result),
// the VALUs only do the softmax.  One workgroup per (stream, strip); its waves
// take the strip's tiles of 32 rows in turn and each keeps its own running
// (m, l, o); the four waves merge at the end.
//
// Lane (j, x) = (lane / 16, lane % 16).  An MFMA operand holds, per lane, 8
// consecutive contraction indices 8 j .. 8 j + 7 of row (A) or column (B) x, and
// the result has element (4 j + i, x) in register i.
//   logits   S^T = K Q^T per 16 rows: A = K rows, B = the query group (columns
//            g >= G are zero).  Lane (j, g) receives the logits of head g for
//            rows 4 j .. 4 j + 3.  An A operand read straight from the cache would
//            take 64 bytes of each of 16 rows per instruction; reading whole rows
//            and turning the tile in LDS measured 10 % faster on short streams.
//   output   O += P V per 32 rows: the probabilities a lane holds after two
//            logit MFMAs (rows 4 j + i and 16 + 4 j + i) are exactly one A operand,
//            so P never changes lanes.  The matching B operand needs, per lane, 8
//            rows of one channel: the lane loads 16 bytes (channels 8 x .. 8 x + 7)
//            of each of its 8 rows and transposes the 8 x 8 block in registers
//            with byte permutes; MFMA c then produces channels 8 x + c.
// A probability enters the MFMA as the sum of two bf16 numbers (the rounded
// value and the rounded remainder), which keeps its relative error below 2^-16.
template <int G, typename PT = AttendParams>
__global__ __launch_bounds__(kThreads, G == 4 ? 2 : 1) void attend_gqa(const PT P) {
  constexpr int D = 128, ROWB = 256, NS = D / 32, kTile = 32;
  typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));
  __shared__ float ml_sh[kWaves][G][2];
  constexpr int kBufTiles = (G == 4 ? kGqaHeldBytesG4 : kGqaHeldBytesG8) / (kWaves * kTile * G * 2);   // tiles a wave can hold back
  __shared__ __attribute__((aligned(16))) unsigned short d_sh[kWaves][kBufTiles][kTile * G];   // logit distances, [row][head]
  __shared__ float tm_sh[kGqaStripRows / kTile][G];                         // reference of every tile of the strip
  static_assert(kTile == kGqaTile, "");
  constexpr int kPitch = ROWB + 16;         // staged K rows, padded against bank conflicts
  // A wave stages the tile's K rows 16 at a time (one logit MFMA group): half the LDS of a whole tile,
  // which the held distances take.
  __shared__ __attribute__((aligned(16))) char kt_sh[kWaves][(kTile / 2) * kPitch];
  // The waves' partial outputs at the end take the place of their K staging areas, which are free by then.
  static_assert(G * D * sizeof(float) <= (kTile / 2) * kPitch, "a wave's outputs fit its staging area");
  auto o_sh = [&](int w, int g, int ch) -> float& {
    return reinterpret_cast<float*>(kt_sh[w])[g * D + ch];
  };

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int x = lane & 15, j = lane >> 4;

  // The kernel is persistent: workgroup b takes the launch's strips b, 2 grid - 1 - b, 2 grid + b, ...
  // (the strips are sorted by length, so every workgroup gets about the same number of rows), and a
  // wave's held tiles may belong to several strips: each remembers where it goes.  At G = 4 the
  // registers are held to two waves per SIMD (two workgroups per compute unit: 3.29 -> 3.24 ms per
  // launch of the batched 16k workload); at G = 8 one workgroup per compute unit measured faster
  // (4.13 against 4.19 ms on the 128k workload), and the host launches one per unit.
  constexpr unsigned long long kWindowTicks = G == 4 ? kStoreWindowTicksG4 : kStoreWindowTicksG8;
  __shared__ char* dst_sh[kWaves][kBufTiles];
  int held = 0;
  unsigned long long last_win = wall_clock64() / kWindowTicks;
  constexpr int kLanesPerTile = kTile * G / 8, kTilesPerInst = 64 / kLanesPerTile;
  auto flush = [&]() {
    const int sub = lane / kLanesPerTile, piece = lane % kLanesPerTile;
    for (int k0 = 0; k0 < held; k0 += kTilesPerInst) {
      const int kk2 = k0 + sub;
      if (kk2 < held) {
        const uint4 dv = *reinterpret_cast<const uint4*>(&d_sh[wave][kk2][8 * piece]);
        store_stream16(dst_sh[wave][kk2] + 16 * piece, dv);
      }
    }
    held = 0;
  };
  const int n_units = P.full_blocks + P.n_tail_pairs * P.n_kv_heads;
  const int grid = gridDim.x;
  for (int round = 0;; ++round) {
  const int unit = round * grid + ((round & 1) ? grid - 1 - static_cast<int>(blockIdx.x) : static_cast<int>(blockIdx.x));
  if (unit >= n_units) break;
  StreamCtx<BF16, D, G> cx;
  cx.init(P, locate_stream_block(P, unit));
  const int n = cx.n;
  const int strip_rows = P.strip_rows;
  const int r_begin = cx.s * strip_rows;
  const int r_end = min(n, r_begin + strip_rows);
  const int tiles = (r_end - r_begin + kTile - 1) / kTile;
  const bool append_here = cx.append_here;
  const int n_plain = n - (append_here ? 1 : 0);   // rows below this come straight from the cache
  float* rec = cx.rec;

  bf16x8 qb[NS];
#pragma unroll
  for (int sl = 0; sl < NS; ++sl) {
    uint4 raw = make_uint4(0, 0, 0, 0);
    if (x < G) {
      const int64_t hq = (static_cast<int64_t>(cx.pair) * P.n_kv_heads + cx.h) * G + x;
      raw = *reinterpret_cast<const uint4*>(static_cast<const char*>(P.q) + hq * ROWB + sl * 64 + j * 16);
    }
    qb[sl] = __builtin_bit_cast(bf16x8, raw);
  }

  floatx4 acc[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) acc[c] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
  float m_run = -INFINITY;                  // head x, all rows of this wave so far
  float l_run = 0.0f;                       // head x, this lane's rows only

  auto dword = [](const uint4& u, int k) { return k == 0 ? u.x : k == 1 ? u.y : k == 2 ? u.z : u.w; };
  // Row of V load i of this lane within a tile.
  auto vrow = [&](int i) { return (i < 4 ? 0 : 12) + 4 * j + i; };
  // Rows at or past n are clamped to row n-1 (their logits are masked); the
  // lanes of an appended row n-1 read the new token instead of the empty slot.
  // One tile of K or V: load i of lane (j, x) is the 16 bytes at column x of row
  // vrow(i), so that every instruction reads whole 256-byte rows.
  auto issue = [&](uint4 (&rb)[8], int t, const char* base, const char* newrow) {
    const int row0 = r_begin + t * kTile;
    if (row0 + kTile <= n_plain) {
      const char* src = base + static_cast<int64_t>(row0 + 4 * j) * ROWB + x * 16;
#pragma unroll
      for (int i = 0; i < 8; ++i) rb[i] = load_stream16(src + ((i < 4 ? 0 : 12) + i) * ROWB);
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int r = row0 + vrow(i);
        const int rc = r < n ? r : n - 1;
        const char* src = base + static_cast<int64_t>(rc) * ROWB + x * 16;
        if (append_here && rc == n - 1) src = newrow + x * 16;
        rb[i] = load_stream16(src);
      }
    }
  };
  auto issue_k = [&](uint4 (&rb)[8], int t) { issue(rb, t, cx.kbase, cx.knew); };
  auto issue_v = [&](uint4 (&rb)[8], int t) { issue(rb, t, cx.vbase, cx.vnew); };

  // The wave's tiles are wave, wave + 4, ...  K and V have one register buffer
  // each; the K rows of the next tile are requested as soon as the current ones
  // sit in LDS, the V rows after the output MFMAs, so each request has most of a
  // tile's work (and the other resident waves) to hide behind.
  uint4 kb[8], vb[8];
  char* kt = kt_sh[wave];
  if (wave < tiles) {
    issue_k(kb, wave);
    issue_v(vb, wave);
  }
  for (int t = wave; t < tiles; t += kWaves) {
    const int row0 = r_begin + t * kTile;
    const bool more = t + kWaves < tiles;
    const bool last_tile = append_here && row0 + kTile >= n;   // holds the appended row n-1
    // The K tile passes through the wave's LDS staging area, 16 rows at a time, to reach the MFMA
    // operand layout (row x of the 16-row group, 16 bytes at column 4 sl + j).  Loads 0..3 of a
    // lane are rows 4 j + i of the first group, loads 4..7 the same rows of the second.
    if (last_tile) {                          // the append itself, K part
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (row0 + vrow(i) == n - 1)
          *reinterpret_cast<uint4*>(cx.kbase + static_cast<int64_t>(n - 1) * ROWB + x * 16) = kb[i];
    }
    float sv[8];
#pragma unroll
    for (int grp = 0; grp < 2; ++grp) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        *reinterpret_cast<uint4*>(kt + (4 * j + i) * kPitch + x * 16) = kb[4 * grp + i];
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      if (grp == 1) {
        __builtin_amdgcn_sched_barrier(0);
        if (more) issue_k(kb, t + kWaves);
        __builtin_amdgcn_sched_barrier(0);
      }
      floatx4 a = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
      for (int sl = 0; sl < NS; ++sl) {
        const uint4 ka = *reinterpret_cast<const uint4*>(kt + x * kPitch + sl * 64 + j * 16);
        a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka), qb[sl], a, 0, 0, 0);
      }
      const int r = row0 + grp * 16 + 4 * j;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        sv[grp * 4 + i] = r + i < r_end ? a[i] * P.scale_log2e : -INFINITY;
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }

    // Online softmax for head x: the tile's first row is live, so the maximum is finite.
    float tm = fmaxf(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])),
                     fmaxf(fmaxf(sv[4], sv[5]), fmaxf(sv[6], sv[7])));
    tm = fmaxf(tm, __shfl_xor(tm, 16));
    tm = fmaxf(tm, __shfl_xor(tm, 32));
    const float m_new = fmaxf(m_run, tm);
    const float alpha = fast_exp2(m_run - m_new);
    const bool moved = m_new > m_run;
    m_run = m_new;
    float pv[8];
    float ls = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      pv[i] = fast_exp2(sv[i] - m_new);
      ls += pv[i];
    }
    l_run = fmaf(l_run, alpha, ls);
    if (x < G) {
      // What the score update needs of this tile: every logit's distance below the
      // running maximum, 16-bit fixed point (masked rows saturate; they are never read).
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float dist = fminf((m_new - sv[i]) * kLogitFixScale, 65535.0f);
        d_sh[wave][held][((i < 4 ? 0 : 12) + 4 * j + i) * G + x] = static_cast<unsigned short>(__float2uint_rn(dist));
      }
      if (j == 0) tm_sh[t][x] = m_new;
    }
    if (__builtin_amdgcn_ballot_w64(moved) != 0) {
      // Accumulator register i of lane (j, .) belongs to head 4 j + i.
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float a_i = __shfl(alpha, 4 * j + i);
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[c][i] *= a_i;
      }
    }
    bf16x8 p_hi, p_lo;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      p_hi[i] = static_cast<__bf16>(pv[i]);
      p_lo[i] = static_cast<__bf16>(pv[i] - static_cast<float>(p_hi[i]));
    }
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const unsigned sel = (c & 1) ? 0x07060302u : 0x05040100u;
      uintx4 vt;
#pragma unroll
      for (int rp = 0; rp < 4; ++rp)
        vt[rp] = __builtin_amdgcn_perm(dword(vb[2 * rp + 1], c >> 1), dword(vb[2 * rp], c >> 1), sel);
      const bf16x8 vop = __builtin_bit_cast(bf16x8, vt);
      acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(p_hi, vop, acc[c], 0, 0, 0);
      acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(p_lo, vop, acc[c], 0, 0, 0);
    }
    if (last_tile) {                          // the append itself, V part
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (row0 + vrow(i) == n - 1)
          *reinterpret_cast<uint4*>(cx.vbase + static_cast<int64_t>(n - 1) * ROWB + x * 16) = vb[i];
    }
    __builtin_amdgcn_sched_barrier(0);
    if (more) issue_v(vb, t + kWaves);
    __builtin_amdgcn_sched_barrier(0);
    // The tile's distances stay in the wave's LDS buffer; the held tiles are written when the wall clock
    // (the same on every compute unit) enters a new window or when the buffer is full: the chip's stores
    // then come in bursts instead of a trickle inside the read stream.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    if (lane == 0) dst_sh[wave][held] = reinterpret_cast<char*>(rec) + static_cast<int64_t>(t) * kTile * G * 2;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    ++held;
    {
      const unsigned long long win = wall_clock64() / kWindowTicks;
      if (win != last_win || held == kBufTiles) {
        flush();
        last_win = win;
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_sched_barrier(0);
  }

  // Merge the four waves.
  float l = l_run;
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);
  if (j == 0 && x < G) {
    ml_sh[wave][x][0] = m_run;
    ml_sh[wave][x][1] = l;
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int g = 4 * j + i;
    if (g < G) {
#pragma unroll
      for (int c = 0; c < 8; ++c) o_sh(wave, g, 8 * x + c) = acc[c][i];
    }
  }
  __syncthreads();
  float* rec_tm = rec + gqa_tilem_offset(G, strip_rows);
  float* rec_o = rec + gqa_out_offset(G, strip_rows);
  float* rec_ml = rec_o + G * D;
  for (int idx = tid; idx < tiles * G; idx += kThreads) store_stream(&rec_tm[idx], tm_sh[idx / G][idx % G]);
  for (int idx = tid; idx < G * (D + 1); idx += kThreads) {
    const int g = idx / (D + 1), ch = idx - g * (D + 1);     // ch == D: the sum l
    float m = ml_sh[0][g][0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) m = fmaxf(m, ml_sh[w][g][0]);
    float tot = 0.0f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const float part = ch < D ? o_sh(w, g, ch) : ml_sh[w][g][1];
      tot += part * fast_exp2(ml_sh[w][g][0] - m);
    }
    if (ch < D) {
      store_stream(&rec_o[g * D + ch], tot);
    } else {
      store_stream(&rec_ml[2 * g], m);
      store_stream(&rec_ml[2 * g + 1], tot);
    }
  }
  __syncthreads();                            // the staging areas and tm_sh are free for the next strip
  }
  flush();
}

// ---------------------------------------------------------------------------
// Second and third kernel of the matrix-core path.
//
// attend_gqa_merge: one workgroup per stream.  Folds the strip statistics into the
// stream's (m, l) per query head, writes (m, 1 / l) for attend_gqa_scores and the
// stream's output rows out = sum_s 2^(m_s - m) o_s / l.  Thread t owns channels
// t, t + 256, ... of the G * D outputs and walks the strips in order, several
// loads in flight.
template <int G, typename PT = AttendParams>
__global__ __launch_bounds__(kThreads) void attend_gqa_merge(const PT P) {
  constexpr int D = 128, GD = G * D, CPT = GD / kThreads;
  extern __shared__ float w_sh[];           // [G][nstrips] strip weights 2^(m_s - m) / l
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int lo = blockIdx.x / P.n_kv_heads;
  const int h = blockIdx.x - lo * P.n_kv_heads;
  const PairDesc pd = P.pairs[lo];
  const int n = pd.n;
  const int strip_rows = P.strip_rows;
  const int64_t stream_idx = static_cast<int64_t>(P.pair_base + lo) * P.n_kv_heads + h;
  float* out = P.out + stream_idx * GD;
  if (n == 0) {
    for (int idx = tid; idx < GD; idx += kThreads) out[idx] = 0.0f;
    return;
  }
  const int nstrips = (n + strip_rows - 1) / strip_rows;
  const int64_t REC = P.rec_floats;
  const float* rec0 = P.ws + (static_cast<int64_t>(pd.strip0) + static_cast<int64_t>(h) * nstrips) * REC +
                      gqa_out_offset(G, strip_rows);
  for (int g = wave; g < G; g += kWaves) {
    const float* ml = rec0 + GD + 2 * g;
    float m = -INFINITY;
    for (int c = lane; c < nstrips; c += 64) m = fmaxf(m, ml[static_cast<int64_t>(c) * REC]);
    m = wave_max(m);
    float l = 0.0f;
    for (int c = lane; c < nstrips; c += 64) {
      const float wgt = fast_exp2(ml[static_cast<int64_t>(c) * REC] - m);
      w_sh[g * nstrips + c] = wgt;
      l = fmaf(wgt, ml[static_cast<int64_t>(c) * REC + 1], l);
    }
    l = wave_sum(l);
    const float inv = 1.0f / l;
    for (int c = lane; c < nstrips; c += 64) w_sh[g * nstrips + c] *= inv;
    if (lane == 0) {
      P.stats[(stream_idx * G + g) * 2] = m;
      P.stats[(stream_idx * G + g) * 2 + 1] = inv;
    }
  }
  __syncthreads();
  float o[CPT];
#pragma unroll
  for (int k = 0; k < CPT; ++k) o[k] = 0.0f;
#pragma unroll 4
  for (int c = 0; c < nstrips; ++c) {
    const float* col = rec0 + static_cast<int64_t>(c) * REC + tid;
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      const int g = (k * kThreads + tid) / D;
      o[k] = fmaf(w_sh[g * nstrips + c], col[k * kThreads], o[k]);
    }
  }
#pragma unroll
  for (int k = 0; k < CPT; ++k) out[k * kThreads + tid] = o[k];
}

// attend_gqa_scores: one workgroup per (stream, fin_rows slots).  A thread takes
// four slots at a time, a workgroup-width apart so that every load instruction
// covers whole lines: the slot's G distances (2 G bytes), its tile's references and
// its score, all requested before the first is used; then
// score_j += sum_g 2^(m_tile - d / 2^10 - m_g) / l_g, the appended token starting
// from zero.
template <int G, typename PT = AttendParams>
__global__ __launch_bounds__(kThreads) void attend_gqa_scores(const PT P) {
  constexpr int kBatch = 4;
  typedef unsigned int uintxg __attribute__((ext_vector_type(G / 2)));   // G distances
  typedef float floatxg __attribute__((ext_vector_type(G)));
  const int tid = threadIdx.x;
  const int bid = blockIdx.x;
  const int strip_rows = P.strip_rows;
  const int FR = P.fin_rows;
  const int64_t REC = P.rec_floats;

  int lo = 0, hi = P.n_pairs - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (fin_first(P, mid) <= bid) lo = mid; else hi = mid - 1;
  }
  const PairDesc pd = P.pairs[lo];
  const int n = pd.n;
  if (n == 0) return;
  const int nstrips = (n + strip_rows - 1) / strip_rows;
  const int nfin = (n + FR - 1) / FR;
  const int local = bid - fin_first(P, lo);
  const int h = local / nfin;
  const int f_own = local - h * nfin;
  const int64_t stream_idx = static_cast<int64_t>(P.pair_base + lo) * P.n_kv_heads + h;
  const float* rec0 = P.ws + (static_cast<int64_t>(pd.strip0) + static_cast<int64_t>(h) * nstrips) * REC;
  const floatxg* st = reinterpret_cast<const floatxg*>(P.stats + stream_idx * G * 2);
  float m_g[G], inv_g[G];
  {
    floatxg a = st[0], b = st[1];           // (m, 1/l) pairs of heads 0 .. G/2-1 and G/2 .. G-1
#pragma unroll
    for (int g = 0; g < G / 2; ++g) {
      m_g[g] = a[2 * g]; inv_g[g] = a[2 * g + 1];
      m_g[G / 2 + g] = b[2 * g]; inv_g[G / 2 + g] = b[2 * g + 1];
    }
  }
  const int64_t stream_slot = pd.slot0 + static_cast<int64_t>(h) * pd.cap;
  float* score = P.score + stream_slot;
  const int shift = __ffs(strip_rows) - 1;  // strip lengths are powers of two
  const int r_begin = f_own * FR;
  const int rows = min(n, r_begin + FR) - r_begin;
  const int64_t tm_off = gqa_tilem_offset(G, strip_rows);
  for (int j0 = tid; j0 < rows; j0 += kBatch * kThreads) {
    uintxg dv[kBatch];
    floatxg tm[kBatch];
    float old[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int j = min(j0 + u * kThreads, rows - 1);         // past the end: a live row again, not stored
      const int row = r_begin + j;
      const int js = row & (strip_rows - 1);
      const float* rec = rec0 + static_cast<int64_t>(row >> shift) * REC;
      dv[u] = __builtin_nontemporal_load(reinterpret_cast<const uintxg*>(rec) + js);
      tm[u] = *(reinterpret_cast<const floatxg*>(rec + tm_off) + (js >> 5));
      old[u] = (P.append && row == n - 1) ? 0.0f : score[row];
    }
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int j = j0 + u * kThreads;
      if (j < rows) {
        float add = 0.0f;
#pragma unroll
        for (int g = 0; g < G; ++g) {
          const unsigned word = dv[u][g >> 1];
          const float dist = static_cast<float>((g & 1) ? (word >> 16) : (word & 0xffffu));
          add = fmaf(fast_exp2(fmaf(dist, -1.0f / kLogitFixScale, tm[u][g] - m_g[g])), inv_g[g], add);
        }
        // Scores left dirty in L2 would be written back under the next launch's K/V
        // stream: they are written through instead.
        store_stream(&score[r_begin + j], old[u] + add);
      }
    }
  }
  if (P.append && f_own == 0 && tid == 0) P.pos[stream_slot + n - 1] = P.pos_new[lo];
}

// ---------------------------------------------------------------------------
// Second kernel of the attend_strip / attend_chunk paths (records with fp32 logits
// [head][slot]).
// kHalf: the records hold 16-bit distances below the strip's maximum (attend_strip
// over bf16 caches) instead of fp32 logits.
template <int D, int G, bool kHalf = false, typename PT = AttendParams>
__global__ __launch_bounds__(kThreads) void attend_finalize(const PT P) {
  constexpr int GD = G * D;
  extern __shared__ float w_sh[];           // [G][nstrips] strip weights 2^(m_s - m) / l
  __shared__ float m_sh[G], inv_sh[G];
  __shared__ float o_red[kThreads];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int bid = blockIdx.x;
  const int strip_rows = P.strip_rows;
  const int F = P.fin_strips;
  const int64_t REC = kHalf ? half_record_floats(G, D, strip_rows) : record_floats(G, D, strip_rows);
  const int lg_floats = kHalf ? strip_rows / 2 : strip_rows;   // floats of logit data per head in a record

  // Region: last pair whose first finalize workgroup is <= bid.  An empty stream
  // owns one strip and one workgroup.
  int lo = 0, hi = P.n_pairs - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (fin_first(P, mid) <= bid) lo = mid; else hi = mid - 1;
  }
  const PairDesc pd = P.pairs[lo];
  const int n = pd.n;
  const int nstrips_live = (n + strip_rows - 1) / strip_rows;
  const int nstrips = nstrips_live > 0 ? nstrips_live : 1;
  const int nfin = (nstrips + F - 1) / F;
  const int local = bid - fin_first(P, lo);
  const int h = local / nfin;
  const int f_own = local - h * nfin;
  const int pair = P.pair_base + lo;
  float* out = P.out + (static_cast<int64_t>(pair) * P.n_kv_heads + h) * GD;
  if (n == 0) {
    for (int idx = tid; idx < GD; idx += kThreads) out[idx] = 0.0f;
    return;
  }
  const float* rec0 = P.ws + (static_cast<int64_t>(pd.strip0) + static_cast<int64_t>(h) * nstrips) * REC;
  const int64_t stream_slot = pd.slot0 + static_cast<int64_t>(h) * pd.cap;
  float* score = P.score + stream_slot;
  const int shift = __ffs(strip_rows) - 1;  // strip lengths are powers of two
  const int s_begin = f_own * F;
  const int r_begin = s_begin << shift;
  const int rows = min(n, (s_begin + F) << shift) - r_begin;
  const float* lg0 = rec0 + static_cast<int64_t>(s_begin) * REC;

  // With 16-bit records a thread's share of the workgroup's slots (at most
  // kMaxStripRows / 2 pairs over 256 threads) fits in registers: their distance
  // words and old scores are requested now, before the statistics below need
  // their own round trip to memory.
  constexpr int kPre = kHalf ? kMaxStripRows / (2 * kThreads) : 1;
  unsigned wpre[kPre][G];
  float old0[kPre], old1[kPre];
  if constexpr (kHalf) {
#pragma unroll
    for (int it = 0; it < kPre; ++it) {
      const int j = 2 * (tid + it * kThreads);
      const int jc = j < rows ? j : 0;            // past the end: slot 0 again, not used
      const int js = jc & (strip_rows - 1);
      const float* lg = lg0 + static_cast<int64_t>(jc >> shift) * REC + (js >> 1);
#pragma unroll
      for (int g = 0; g < G; ++g) wpre[it][g] = __float_as_uint(lg[g * lg_floats]);
      const int row = r_begin + jc;
      const bool two = jc + 1 < rows;
      old0[it] = (P.append && row == n - 1) ? 0.0f : score[row];            // the appended token starts from zero
      old1[it] = (!two || (P.append && row + 1 == n - 1)) ? 0.0f : score[row + 1];
    }
  }

  // Stream statistics from the strip statistics, one wave per query head.  Every
  // workgroup of the stream repeats this small reduction in the same order, so
  // all agree bit for bit.
  for (int g = wave; g < G; g += kWaves) {
    const float* ml = rec0 + G * (lg_floats + D) + 2 * g;
    float m = -INFINITY;
    for (int c = lane; c < nstrips; c += 64) m = fmaxf(m, ml[static_cast<int64_t>(c) * REC]);
    m = wave_max(m);
    float l = 0.0f;
    for (int c = lane; c < nstrips; c += 64) {
      const float wgt = fast_exp2(ml[static_cast<int64_t>(c) * REC] - m);
      w_sh[g * nstrips + c] = wgt;
      l = fmaf(wgt, ml[static_cast<int64_t>(c) * REC + 1], l);
    }
    l = wave_sum(l);
    const float inv = 1.0f / l;
    for (int c = lane; c < nstrips; c += 64) w_sh[g * nstrips + c] *= inv;
    if (lane == 0) { m_sh[g] = m; inv_sh[g] = inv; }
  }
  __syncthreads();

  // score_j += sum_g p_gj for the slots of this workgroup's strips.
  if constexpr (kHalf) {
    // p = 2^(-d / 2^10) * [2^(m_s - m) / l], the bracket being the strip's weight w_sh.
    // A thread takes pairs of neighbouring slots: one word of distances per head.
#pragma unroll
    for (int it = 0; it < kPre; ++it) {
      const int j = 2 * (tid + it * kThreads);
      if (j < rows) {
        const int c = s_begin + (j >> shift);
        float add0 = 0.0f, add1 = 0.0f;
#pragma unroll
        for (int g = 0; g < G; ++g) {
          const unsigned word = wpre[it][g];
          const float wgt = w_sh[g * nstrips + c];
          add0 = fmaf(fast_exp2(static_cast<float>(word & 0xffffu) * (-1.0f / kLogitFixScale)), wgt, add0);
          add1 = fmaf(fast_exp2(static_cast<float>(word >> 16) * (-1.0f / kLogitFixScale)), wgt, add1);
        }
        const int row = r_begin + j;
        score[row] = old0[it] + add0;
        if (j + 1 < rows) score[row + 1] = old1[it] + add1;
      }
    }
  } else {
    float m_g[G], inv_g[G];
#pragma unroll
    for (int g = 0; g < G; ++g) { m_g[g] = m_sh[g]; inv_g[g] = inv_sh[g]; }
#pragma unroll 8
    for (int j = tid; j < rows; j += kThreads) {
      const int js = j & (strip_rows - 1);
      const float* lg = lg0 + static_cast<int64_t>(j >> shift) * REC + js;
      float add = 0.0f;
#pragma unroll
      for (int g = 0; g < G; ++g) add = fmaf(fast_exp2(lg[g * strip_rows] - m_g[g]), inv_g[g], add);
      const int row = r_begin + j;
      const float old = (P.append && row == n - 1) ? 0.0f : score[row];
      score[row] = old + add;
    }
  }
  if (P.append && f_own == 0 && tid == 0) P.pos[stream_slot + n - 1] = P.pos_new[lo];

  // out = sum_s w_s o_s.  The G*D channels of the stream are split evenly over
  // its workgroups.  Within a workgroup the threads form (channel, slice)
  // pairs; a slice sums every S-th strip, then the slices are added in order.
  const int cpb = (GD + nfin - 1) / nfin;
  const int ch_first = f_own * cpb;
  const int nch = min(cpb, GD - ch_first);
  for (int tb = 0; tb < nch; tb += kThreads) {
    const int tn = min(kThreads, nch - tb);
    const int S = kThreads / tn;
    const int ch_l = tid % tn, slice = tid / tn;
    float o = 0.0f;
    if (slice < S) {
      const int idx = ch_first + tb + ch_l;
      const int g = idx / D;
      const float* col = rec0 + G * lg_floats + idx;
#pragma unroll 4
      for (int c = slice; c < nstrips; c += S)
        o = fmaf(w_sh[g * nstrips + c], col[static_cast<int64_t>(c) * REC], o);
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

constexpr int kStepEvict = 8;

template <int kStepThreads>
struct StepEvictShared {
  unsigned long long best[kStepThreads / 64];
  int ev[kStepEvict], hole[kStepEvict], mover[kStepEvict];
  int moves;
};

// The eviction of one stream by its workgroup, after the pass that wrote the
// stream's updated scores: `mine` is the smallest (score, -slot) pack the calling
// thread saw in that pass (or in a pass of its own over key_at, for derived keys).
// Round 0 takes the workgroup's minimum of those; every further eviction takes a
// pass over key_at(slot), the key of a slot from the scores in memory.  Then the holes (evicted
// slots below kk) receive the surviving tokens of slots [kk, n), both ascending.
template <int kStepThreads, typename PT, typename KeyAt>
__device__ __forceinline__ void step_evict(const PT& P, unsigned long long mine, int n, int kk,
                                           int64_t stream_slot, StepEvictShared<kStepThreads>& sh, KeyAt key_at) {
  constexpr int kStepWaves = kStepThreads / 64;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  // ---- eviction: the E = n - kk smallest (score, -slot), one per round ----------------
  int32_t* kept = P.kept_idx ? P.kept_idx + stream_slot : nullptr;
  const int E = (kk >= n || kk == 0) ? 0 : n - kk;        // nothing to select when all or none stay
  unsigned long long last = 0;              // every pack is > 0: ~slot has its top bit set
  for (int r = 0; r < E; ++r) {
    unsigned long long best = mine;         // round 0: from the pass above
    if (r > 0) {
      __syncthreads();                      // the scores written above are visible to the whole workgroup
      best = ~0ull;
#pragma unroll 4
      for (int j = tid; j < n; j += kStepThreads) {
        const unsigned long long pk =
            (static_cast<unsigned long long>(key_at(j)) << 32) | (0xffffffffu - static_cast<unsigned>(j));
        if (pk > last && pk < best) best = pk;
      }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      const unsigned long long o = __shfl_xor(best, off);
      best = o < best ? o : best;
    }
    if (lane == 0) sh.best[wave] = best;
    __syncthreads();
    best = sh.best[0];
#pragma unroll
    for (int w = 1; w < kStepWaves; ++w) best = sh.best[w] < best ? sh.best[w] : best;
    last = best;
    if (tid == 0) sh.ev[r] = static_cast<int>(0xffffffffu - static_cast<unsigned>(best & 0xffffffffull));
    __syncthreads();
  }
  if (tid == 0) {
    // holes: evicted slots below kk, ascending; movers: the survivors among the slots [kk, n), ascending.
    for (int a = 1; a < E; ++a) {
      const int x = sh.ev[a];
      int b = a - 1;
      while (b >= 0 && sh.ev[b] > x) { sh.ev[b + 1] = sh.ev[b]; --b; }
      sh.ev[b + 1] = x;
    }
    int nh = 0, nm = 0;
    for (int a = 0; a < E; ++a)
      if (sh.ev[a] < kk) sh.hole[nh++] = sh.ev[a];
    for (int s = kk; s < n && E > 0; ++s) {
      bool evicted = false;
      for (int a = 0; a < E; ++a) evicted = evicted || sh.ev[a] == s;
      if (!evicted) sh.mover[nm++] = s;
    }
    sh.moves = nh;
  }
  __syncthreads();                          // also: the new scores and the appended pos are visible to the movers
  const int moves = sh.moves;
  if (kept != nullptr)
    for (int j = tid; j < kk; j += kStepThreads) {
      bool is_hole = false;
      for (int a = 0; a < moves; ++a) is_hole = is_hole || sh.hole[a] == j;
      if (!is_hole) kept[j] = j;
    }
  for (int i = wave; i < moves; i += kStepWaves) {
    const int dst = sh.hole[i], src = sh.mover[i];
    const int frags = P.row_bytes >> 4;     // 16-byte pieces per row: 8, 16 or 32
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
    } else if (lane == 34 && kept != nullptr) {
      kept[dst] = src;
    }
  }

}

// ---------------------------------------------------------------------------
// attend_finalize and the steady-state eviction in one kernel (xkv_decode_step):
// one workgroup per stream.  It does what attend_finalize does for the whole
// stream (statistics, score update, output) with the same arithmetic in the same
// order, and while it writes the updated scores it keeps track of the smallest
// (score, -slot) it has seen: that is the first token to evict (equal scores go
// to the higher slot, as in the selection kernel), found without a second pass.
// Further evictions (at most kStepEvict per stream) each take one more pass over
// the scores just written, which the L2 still holds.  Then the kept tokens of
// the slots at or beyond the budget move into the holes.  The host takes this
// kernel only when every stream of the call evicts at most kStepEvict tokens.
// With pooling or protected tokens the keys are derived from the scores just
// written (a pass of its own over them, out of the L2).
//
// Three workgroup sizes: 256 threads when the call has enough streams to fill the
// chip with such workgroups (the kernel is a chain of dependent steps, and the
// more streams are resident at once the sooner the call is through) or its
// streams are short, 512 when such a call has streams beyond 8192 slots (a
// workgroup's time grows with its stream), 1024 for calls of few long streams.
template <int D, int G, bool kHalf, int kStepThreads, typename PT = StepParams>
__global__ __launch_bounds__(kStepThreads) void attend_finalize_evict(const PT P) {
  constexpr int GD = G * D;
  constexpr int kStepWaves = kStepThreads / 64;
  constexpr int kBatch = 8;                 // slot pairs (16-bit records) or slots per thread in flight
  extern __shared__ float w_sh[];           // [G][nstrips] strip weights 2^(m_s - m) / l
  __shared__ float m_sh[G], inv_sh[G];
  __shared__ float o_red[kStepThreads];
  __shared__ StepEvictShared<kStepThreads> ev;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int strip_rows = P.strip_rows;
  const int64_t REC = kHalf ? half_record_floats(G, D, strip_rows) : record_floats(G, D, strip_rows);
  const int lg_floats = kHalf ? strip_rows / 2 : strip_rows;
  const int lo = blockIdx.x / P.n_kv_heads;
  const int h = blockIdx.x - lo * P.n_kv_heads;
  const PairDesc pd = P.pairs[lo];
  const int n = pd.n;
  const int kk = P.keep[lo];
  const int pair = P.pair_base + lo;
  float* out = P.out + (static_cast<int64_t>(pair) * P.n_kv_heads + h) * GD;
  if (n == 0) {
    for (int idx = tid; idx < GD; idx += kStepThreads) out[idx] = 0.0f;
    return;
  }
  const int nstrips = (n + strip_rows - 1) / strip_rows;
  const float* rec0 = P.ws + (static_cast<int64_t>(pd.strip0) + static_cast<int64_t>(h) * nstrips) * REC;
  const int64_t stream_slot = pd.slot0 + static_cast<int64_t>(h) * pd.cap;
  float* score = P.score + stream_slot;
  const int shift = __ffs(strip_rows) - 1;  // strip lengths are powers of two
  constexpr int kStride = kHalf ? 2 : 1;    // slots per thread and turn
  // Turn `it` of the pass: this thread's first slot, and what it needs of it (the distance word
  // of a slot pair, or nothing yet for fp32 logits) and the old scores.
  auto first_slot = [&](int it) { return kStride * (tid + it * kStepThreads); };
  const int turns = (n + kStride * kStepThreads - 1) / (kStride * kStepThreads);
  unsigned wv[kBatch][G];
  float old0[kBatch], old1[kBatch];
  auto request = [&](int it0) {
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int j = first_slot(it0 + u);
      const int jc = j < n ? j : 0;                          // past the end: slot 0 again, not used
      if constexpr (kHalf) {
        const float* lg = rec0 + static_cast<int64_t>(jc >> shift) * REC + ((jc & (strip_rows - 1)) >> 1);
#pragma unroll
        for (int g = 0; g < G; ++g) wv[u][g] = __float_as_uint(lg[g * lg_floats]);
        old1[u] = (jc + 1 >= n || (P.append && jc + 1 == n - 1)) ? 0.0f : score[jc + 1];
      }
      old0[u] = (P.append && jc == n - 1) ? 0.0f : score[jc];          // the appended token starts from zero
    }
  };
  request(0);                               // in flight while the statistics below take their own round trip

  // Stream statistics from the strip statistics, one wave per query head at a time.
  for (int g = wave; g < G; g += kStepWaves) {
    const float* ml = rec0 + G * (lg_floats + D) + 2 * g;
    float m = -INFINITY;
    for (int c = lane; c < nstrips; c += 64) m = fmaxf(m, ml[static_cast<int64_t>(c) * REC]);
    m = wave_max(m);
    float l = 0.0f;
    for (int c = lane; c < nstrips; c += 64) {
      const float wgt = fast_exp2(ml[static_cast<int64_t>(c) * REC] - m);
      w_sh[g * nstrips + c] = wgt;
      l = fmaf(wgt, ml[static_cast<int64_t>(c) * REC + 1], l);
    }
    l = wave_sum(l);
    const float inv = 1.0f / l;
    for (int c = lane; c < nstrips; c += 64) w_sh[g * nstrips + c] *= inv;
    if (lane == 0) { m_sh[g] = m; inv_sh[g] = inv; }
  }
  if (P.append && tid == 0) P.pos[stream_slot + n - 1] = P.pos_new[lo];
  __syncthreads();

  // score_j += sum_g p_gj; the smallest (score, -slot) of this thread's slots on the way.
  unsigned long long mine = ~0ull;
  auto see = [&](float sc, int j) {
    const unsigned long long pk =
        (static_cast<unsigned long long>(__float_as_uint(sc)) << 32) | (0xffffffffu - static_cast<unsigned>(j));
    mine = pk < mine ? pk : mine;
  };
  float m_g[G], inv_g[G];
#pragma unroll
  for (int g = 0; g < G; ++g) { m_g[g] = m_sh[g]; inv_g[g] = inv_sh[g]; }
  for (int it0 = 0; it0 < turns; it0 += kBatch) {
    if (it0 > 0) request(it0);
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int j = first_slot(it0 + u);
      if (j < n) {
        if constexpr (kHalf) {
          const int c = j >> shift;
          float add0 = 0.0f, add1 = 0.0f;
#pragma unroll
          for (int g = 0; g < G; ++g) {
            const unsigned word = wv[u][g];
            const float wgt = w_sh[g * nstrips + c];
            add0 = fmaf(fast_exp2(static_cast<float>(word & 0xffffu) * (-1.0f / kLogitFixScale)), wgt, add0);
            add1 = fmaf(fast_exp2(static_cast<float>(word >> 16) * (-1.0f / kLogitFixScale)), wgt, add1);
          }
          const float s0 = old0[u] + add0;
          score[j] = s0;
          see(s0, j);
          if (j + 1 < n) {
            const float s1 = old1[u] + add1;
            score[j + 1] = s1;
            see(s1, j + 1);
          }
        } else {
          const float* lg = rec0 + static_cast<int64_t>(j >> shift) * REC + (j & (strip_rows - 1));
          float add = 0.0f;
#pragma unroll
          for (int g = 0; g < G; ++g) add = fmaf(fast_exp2(lg[g * strip_rows] - m_g[g]), inv_g[g], add);
          const float s0 = old0[u] + add;
          score[j] = s0;
          see(s0, j);
        }
      }
    }
  }

  // Keys of the eviction: the score itself, or (pooling, protected tokens) derived from the
  // scores just written, as in the selection kernel: the fp32 window sum, left to right, zeros
  // outside the stream; +inf for the n_protect highest positions.
  const bool derived = P.pool > 1 || P.n_protect > 0;
  const int32_t* pos = P.pos + stream_slot;
  int limit = std::numeric_limits<int>::min();             // protected: pos >= limit
  const int E_all = (kk >= n || kk == 0) ? 0 : n - kk;
  if (derived && E_all > 0) {
    __syncthreads();                        // the new scores and the appended pos are visible
    if (P.n_protect > 0) {
      int mx = std::numeric_limits<int>::min();
#pragma unroll 4
      for (int j = tid; j < n; j += kStepThreads) mx = max(mx, pos[j]);
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) mx = max(mx, __shfl_xor(mx, off));
      if (lane == 0) reinterpret_cast<int*>(ev.best)[wave] = mx;
      __syncthreads();
      mx = reinterpret_cast<int*>(ev.best)[0];
#pragma unroll
      for (int w = 1; w < kStepWaves; ++w) mx = max(mx, reinterpret_cast<int*>(ev.best)[w]);
      const long long lim = static_cast<long long>(mx) + 1 - P.n_protect;
      limit = lim < std::numeric_limits<int>::min() ? std::numeric_limits<int>::min() : static_cast<int>(lim);
      __syncthreads();
    }
  }
  const int half = P.pool >> 1;
  auto key_at = [&](int j) -> unsigned {
    if (!derived) return __float_as_uint(score[j]);
    float acc = 0.0f;
    for (int t0 = 0; t0 < P.pool; t0 += 8) {              // the terms are fetched eight at a time so that their loads overlap
      float term[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const int x = j - half + t0 + q;
        term[q] = (t0 + q < P.pool && x >= 0 && x < n) ? score[x] : 0.0f;
      }
#pragma unroll
      for (int q = 0; q < 8; ++q)
        if (t0 + q < P.pool) acc = (t0 + q == 0) ? term[q] : acc + term[q];
    }
    unsigned key = __float_as_uint(acc);
    if (P.n_protect > 0 && pos[j] >= limit) key = 0x7f800000u;
    return key;
  };
  if (derived && E_all > 0) {
    mine = ~0ull;
    if (P.pool <= 64) {
      // Tiles of kPer slots per thread: the tile's scores and the window's overhang on both sides pass
      // through LDS (two buffers: the next tile is requested while this one is summed), so that a score
      // is read from memory once instead of pool times.
      constexpr int kPer = 4, kTileSlots = kPer * kStepThreads;
      __shared__ float tile_sh[2][kTileSlots + 64];
      const int span = kTileSlots + P.pool - 1;            // tile plus overhang
      const int tiles = (n + kTileSlots - 1) / kTileSlots;
      float pre[kPer + 1];
      int pj[kPer];
      auto fetch = [&](int t) {
#pragma unroll
        for (int k = 0; k <= kPer; ++k) {
          const int i = tid + k * kStepThreads;
          const int x = t * kTileSlots - half + i;
          pre[k] = (i < span && x >= 0 && x < n) ? score[x] : 0.0f;
        }
#pragma unroll
        for (int k = 0; k < kPer; ++k) {
          const int j = t * kTileSlots + tid + k * kStepThreads;
          pj[k] = (P.n_protect > 0 && j < n) ? pos[j] : std::numeric_limits<int>::min();
        }
      };
      fetch(0);
      for (int t = 0; t < tiles; ++t) {
        float* tile = tile_sh[t & 1];
#pragma unroll
        for (int k = 0; k <= kPer; ++k)
          if (tid + k * kStepThreads < span) tile[tid + k * kStepThreads] = pre[k];
        int pj_now[kPer];
#pragma unroll
        for (int k = 0; k < kPer; ++k) pj_now[k] = pj[k];
        __syncthreads();                      // tile t is in LDS; the other buffer's readers (tile t-1) are past it
        if (t + 1 < tiles) fetch(t + 1);
#pragma unroll
        for (int k = 0; k < kPer; ++k) {
          const int jl = tid + k * kStepThreads;
          const int j = t * kTileSlots + jl;
          if (j < n) {
            float acc = tile[jl];             // window sum, fp32, left to right
            for (int q = 1; q < P.pool; ++q) acc = acc + tile[jl + q];
            unsigned key = __float_as_uint(acc);
            if (P.n_protect > 0 && pj_now[k] >= limit) key = 0x7f800000u;
            const unsigned long long pk =
                (static_cast<unsigned long long>(key) << 32) | (0xffffffffu - static_cast<unsigned>(j));
            mine = pk < mine ? pk : mine;
          }
        }
      }
    } else {
#pragma unroll 2
      for (int j = tid; j < n; j += kStepThreads) {
        const unsigned long long pk =
            (static_cast<unsigned long long>(key_at(j)) << 32) | (0xffffffffu - static_cast<unsigned>(j));
        mine = pk < mine ? pk : mine;
      }
    }
  }
  step_evict<kStepThreads>(P, mine, n, kk, stream_slot, ev, key_at);

  // out = sum_s w_s o_s: threads form (channel, slice) pairs; a slice sums every
  // S-th strip, then the slices are added in order.
  for (int tb = 0; tb < GD; tb += kStepThreads) {
    const int tn = min(kStepThreads, GD - tb);
    const int S = kStepThreads / tn;
    const int ch_l = tid % tn, slice = tid / tn;
    float o = 0.0f;
    if (slice < S) {
      const int idx = tb + ch_l;
      const int g = idx / D;
      const float* col = rec0 + G * lg_floats + idx;
#pragma unroll 4
      for (int c = slice; c < nstrips; c += S)
        o = fmaf(w_sh[g * nstrips + c], col[static_cast<int64_t>(c) * REC], o);
    }
    __syncthreads();
    o_red[tid] = o;
    __syncthreads();
    if (tid < tn) {
      float tot = o_red[tid];
      for (int sl = 1; sl < S; ++sl) tot += o_red[sl * tn + tid];
      out[tb + tid] = tot;
    }
  }
}

// ---------------------------------------------------------------------------
// Writes one chunk of the geometry tables of a large call into device memory: the
// entries travel in the kernel arguments, so no host-to-device copy is involved
// and the call stays capturable in a graph.  (Kernel arguments of this size, 36 KB,
// are accepted by the HIP runtime here; 64 KB were tried.)
constexpr int kTableChunk = 1024;
struct TableChunk {
  int32_t first, count;
  PairDesc pairs[kTableChunk];
  int32_t pos_new[kTableChunk];
  int32_t tail_order[kTableChunk];
  int32_t fin0[kTableChunk];
};

__global__ void table_write(const TableChunk c, PairDesc* pairs, int32_t* pos_new, int32_t* tail_order,
                            int32_t* fin0) {
  const int i = threadIdx.x;
  if (i >= c.count) return;
  pairs[c.first + i] = c.pairs[i];
  pos_new[c.first + i] = c.pos_new[i];
  tail_order[c.first + i] = c.tail_order[i];
  fin0[c.first + i] = c.fin0[i];
}

using KernelFn = void (*)(const AttendParams);
using TableKernelFn = void (*)(const AttendTableParams);
struct Kernels {
  KernelFn stream = nullptr;
  KernelFn finalize = nullptr;
  KernelFn fused = nullptr;
  TableKernelFn stream_tab = nullptr;      // the same kernels with the geometry tables in device memory
  TableKernelFn finalize_tab = nullptr;
  KernelFn merge = nullptr;                // matrix-core path: attend_gqa_merge, then `finalize` = attend_gqa_scores
  TableKernelFn merge_tab = nullptr;
  // Score update plus the steady-state eviction (xkv_decode_step): workgroups of 256, 512 and 1024 threads.
  void (*step[3])(const StepParams) = {nullptr, nullptr, nullptr};
  void (*step_tab[3])(const StepTableParams) = {nullptr, nullptr, nullptr};
  int max_strip_rows = kChunk;  // longest strip the streaming kernel is given (a power of two)
  bool lds_logits = false;      // the streaming kernel collects the strip's logits in dynamic LDS
  bool half_records = false;    // attend_strip over bf16: records with 16-bit distances
};

template <typename T, int D>
bool pick_group(int group, Kernels* k) {
  switch (group) {
    case 1:
      k->half_records = std::is_same<T, BF16>::value;
      k->stream = attend_strip<T, D, 1, 8>; k->finalize = attend_finalize<D, 1, std::is_same<T, BF16>::value>;
      k->stream_tab = attend_strip<T, D, 1, 8, AttendTableParams>;
      k->finalize_tab = attend_finalize<D, 1, std::is_same<T, BF16>::value, AttendTableParams>;
      k->max_strip_rows = kMaxStripRows; k->lds_logits = true;
      k->fused = attend_fused<T, D, 1, 8>;
      k->step[0] = attend_finalize_evict<D, 1, std::is_same<T, BF16>::value, 256>;
      k->step_tab[0] = attend_finalize_evict<D, 1, std::is_same<T, BF16>::value, 256, StepTableParams>;
      k->step[1] = attend_finalize_evict<D, 1, std::is_same<T, BF16>::value, 512>;
      k->step_tab[1] = attend_finalize_evict<D, 1, std::is_same<T, BF16>::value, 512, StepTableParams>;
      k->step[2] = attend_finalize_evict<D, 1, std::is_same<T, BF16>::value, 1024>;
      k->step_tab[2] = attend_finalize_evict<D, 1, std::is_same<T, BF16>::value, 1024, StepTableParams>;
      return true;
    case 2:
      k->half_records = std::is_same<T, BF16>::value;
      k->stream = attend_strip<T, D, 2, 8>; k->finalize = attend_finalize<D, 2, std::is_same<T, BF16>::value>;
      k->stream_tab = attend_strip<T, D, 2, 8, AttendTableParams>;
      k->finalize_tab = attend_finalize<D, 2, std::is_same<T, BF16>::value, AttendTableParams>;
      k->max_strip_rows = kMaxStripRows; k->lds_logits = true;
      k->fused = attend_fused<T, D, 2, 8>;
      k->step[0] = attend_finalize_evict<D, 2, std::is_same<T, BF16>::value, 256>;
      k->step_tab[0] = attend_finalize_evict<D, 2, std::is_same<T, BF16>::value, 256, StepTableParams>;
      k->step[1] = attend_finalize_evict<D, 2, std::is_same<T, BF16>::value, 512>;
      k->step_tab[1] = attend_finalize_evict<D, 2, std::is_same<T, BF16>::value, 512, StepTableParams>;
      k->step[2] = attend_finalize_evict<D, 2, std::is_same<T, BF16>::value, 1024>;
      k->step_tab[2] = attend_finalize_evict<D, 2, std::is_same<T, BF16>::value, 1024, StepTableParams>;
      return true;
    case 4:
      k->stream = attend_chunk<T, D, 4>; k->finalize = attend_finalize<D, 4>;
      k->stream_tab = attend_chunk<T, D, 4, AttendTableParams>;
      k->finalize_tab = attend_finalize<D, 4, false, AttendTableParams>;
      k->fused = attend_fused<T, D, 4, 4>;
      k->step[0] = attend_finalize_evict<D, 4, false, 256>;
      k->step_tab[0] = attend_finalize_evict<D, 4, false, 256, StepTableParams>;
      k->step[1] = attend_finalize_evict<D, 4, false, 512>;
      k->step_tab[1] = attend_finalize_evict<D, 4, false, 512, StepTableParams>;
      k->step[2] = attend_finalize_evict<D, 4, false, 1024>;
      k->step_tab[2] = attend_finalize_evict<D, 4, false, 1024, StepTableParams>;
      if constexpr (std::is_same<T, BF16>::value && D == 128) {
        // (the matrix-core path keeps its three kernels: one workgroup per stream for the score update measured
        // no faster than the score kernel's even split plus the selection kernel, 173 against 176 us per step)
        for (int i = 0; i < 3; ++i) { k->step[i] = nullptr; k->step_tab[i] = nullptr; }
        k->stream = attend_gqa<4>; k->merge = attend_gqa_merge<4>; k->finalize = attend_gqa_scores<4>;
        k->stream_tab = attend_gqa<4, AttendTableParams>;
        k->merge_tab = attend_gqa_merge<4, AttendTableParams>;
        k->finalize_tab = attend_gqa_scores<4, AttendTableParams>;
        k->max_strip_rows = kGqaStripRows;
      }
      return true;
    case 8:
      k->stream = attend_chunk<T, D, 8>; k->finalize = attend_finalize<D, 8>;
      k->stream_tab = attend_chunk<T, D, 8, AttendTableParams>;
      k->finalize_tab = attend_finalize<D, 8, false, AttendTableParams>;
      k->fused = attend_fused<T, D, 8, 2>;
      k->step[0] = attend_finalize_evict<D, 8, false, 256>;
      k->step_tab[0] = attend_finalize_evict<D, 8, false, 256, StepTableParams>;
      k->step[1] = attend_finalize_evict<D, 8, false, 512>;
      k->step_tab[1] = attend_finalize_evict<D, 8, false, 512, StepTableParams>;
      k->step[2] = attend_finalize_evict<D, 8, false, 1024>;
      k->step_tab[2] = attend_finalize_evict<D, 8, false, 1024, StepTableParams>;
      if constexpr (std::is_same<T, BF16>::value && D == 128) {
        // (the matrix-core path keeps its three kernels: one workgroup per stream for the score update measured
        // no faster than the score kernel's even split plus the selection kernel, 173 against 176 us per step)
        for (int i = 0; i < 3; ++i) { k->step[i] = nullptr; k->step_tab[i] = nullptr; }
        k->stream = attend_gqa<8>; k->merge = attend_gqa_merge<8>; k->finalize = attend_gqa_scores<8>;
        k->stream_tab = attend_gqa<8, AttendTableParams>;
        k->merge_tab = attend_gqa_merge<8, AttendTableParams>;
        k->finalize_tab = attend_gqa_scores<8, AttendTableParams>;
        k->max_strip_rows = kGqaStripRows;
      }
      return true;
    default: return false;
  }
}

bool pick_kernels(int dtype, int head_dim, int group, Kernels* k) {
  if (dtype == XKV_F32 && head_dim == 64) return pick_group<F32, 64>(group, k);
  if (dtype == XKV_F32 && head_dim == 128) return pick_group<F32, 128>(group, k);
  if (dtype == XKV_BF16 && head_dim == 64) return pick_group<BF16, 64>(group, k);
  if (dtype == XKV_BF16 && head_dim == 128) return pick_group<BF16, 128>(group, k);
  return false;
}

// Strip length of a call: long strips amortise the per-strip record and let a
// workgroup pipeline its loads, but a call must still spread over the whole
// chip, so the strips shrink until there are enough of them.
int choose_strip_rows(int max_rows, int64_t streams, int64_t total_rows) {
  int rows = max_rows;
  // Enough workgroups for several per compute unit; measured on the 4k-context workload
  // (1024 streams of 1640 slots on average) with 768 / 1024 / 1536 / 2048 / 4096: 156.8 / 155.1 /
  // 158.8 / 159.5 / 159.8 us per step; the 32k-context workload does not care (553 us for all but 4096).
  const int64_t want = 1024;
  while (rows > kChunk && total_rows / rows + streams / 2 < want) rows >>= 1;
  return rows;
}

// ---- fused path, host side ---------------------------------------------------
constexpr size_t kFusedLdsBudget = 72 * 1024;   // logits per workgroup; two workgroups share a compute unit

int g_attend_path = 0;                          // 0 auto, 1 two kernels, 2 fused or error
constexpr uint32_t kDefaultSpinLimit = 1u << 24; // polls of about 64 cycles each: several hundred ms
uint32_t g_fused_spin_limit = kDefaultSpinLimit;
// Control words of the most recent fused call, for xkv_fused_status.
struct LastFused { const unsigned* control = nullptr; size_t launches = 0; hipStream_t stream = nullptr; };
LastFused g_last_fused;
// What "auto" picks.  On the 32k benchmark workload the fused launch is 5 % slower
// than the two kernels (its grid barrier and second phase cost more than the logit
// stores it saves), and its larger query groups run on the VALUs; it stays selectable.
constexpr bool kAutoPrefersFused = false;

int compute_units() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) cus = 0;
  }
  return cus;
}

// Workgroups of `fn` that are resident at once with `lds` bytes of dynamic LDS
// each (0 if unknown); raises the kernel's LDS limit when needed.  Cached per kernel.
int resident_workgroups(KernelFn fn, size_t lds) {
  struct Entry { KernelFn fn; size_t lds; int n; };
  static std::vector<Entry> cache;
  for (const Entry& e : cache)
    if (e.fn == fn && e.lds == lds) return e.n;
  const int cus = compute_units();
  const void* f = reinterpret_cast<const void*>(fn);
  int n = 0, per_cu = 0;
  if (cus > 0 &&
      (lds <= 48 * 1024 ||
       hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)) == hipSuccess) &&
      hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, f, kThreads, lds) == hipSuccess)
    n = per_cu * cus;
  (void)hipGetLastError();
  cache.push_back({fn, lds, n});
  return n;
}

// Launches the fused kernel over the call's regions, in groups of consecutive
// regions that fit one launch (kMaxPairs regions, and no more strips than the
// resident workgroups can hold logits for).  Returns XKV_ERR_UNSUPPORTED, before
// anything is enqueued, if the call does not fit this path.
xkv_status launch_fused(const xkv_cache* cache, int64_t first, int64_t n_pairs, bool append,
                        const int32_t* pos_new, AttendParams& P, KernelFn fn, int G, int D,
                        int64_t total_rows, void* workspace, size_t workspace_bytes,
                        hipStream_t stream) {
  const int B = cache->batch, hkv = cache->n_kv_heads;
  const int64_t seg = static_cast<int64_t>(G) * (D + 2);
  const int lds_rows = static_cast<int>(kFusedLdsBudget / (sizeof(float) * G) / kChunk * kChunk);
  const size_t lds = static_cast<size_t>(lds_rows) * G * sizeof(float);
  const int n_wgs = resident_workgroups(fn, lds);
  if (n_wgs <= 0) return XKV_ERR_UNSUPPORTED;
  // Strip length: about nine strips fit a workgroup; shorter when the call is
  // small, so that every workgroup still finds work in the queue.
  int strip_rows = std::max(kChunk, 2048 / G);
  while (strip_rows > kChunk && total_rows / strip_rows < 2 * static_cast<int64_t>(n_wgs)) strip_rows >>= 1;
  const int64_t hold = std::min<int64_t>(kMaxHeld, lds_rows / strip_rows);
  const int64_t capacity = hold * n_wgs;      // strips one launch can take

  struct Group { int64_t g0; int np; int64_t strips; int64_t units; };
  std::vector<Group> groups;
  int64_t total_strips = 0;
  Group cur{0, 0, 0, 0};
  for (int64_t i = 0; i < n_pairs; ++i) {
    const int64_t n = cache->len[first + i] + (append ? 1 : 0);
    const int64_t units = ceil_div(n, strip_rows) * hkv;              // strips with live rows
    const int64_t strips = std::max<int64_t>(ceil_div(n, strip_rows), 1) * hkv;
    if (units > capacity) return XKV_ERR_UNSUPPORTED;
    if (cur.np == kMaxPairs || cur.units + units > capacity) {
      groups.push_back(cur);
      cur = Group{i, 0, 0, 0};
    }
    cur.np += 1;
    cur.units += units;
    cur.strips += strips;
    total_strips += strips;
  }
  if (cur.np > 0) groups.push_back(cur);
  if (total_strips > std::numeric_limits<int32_t>::max()) return XKV_ERR_UNSUPPORTED;
  // Records first, then four control words per launch.
  const uint64_t need = static_cast<uint64_t>(total_strips) * seg * sizeof(float) + groups.size() * 16;
  if (need > workspace_bytes) return XKV_ERR_UNSUPPORTED;
  unsigned* control0 = reinterpret_cast<unsigned*>(static_cast<float*>(workspace) + total_strips * seg);

  P.strip_rows = strip_rows;
  P.rec_floats = static_cast<int32_t>(seg);
  P.lds_rows = lds_rows;
  P.fin_strips = 1;
  P.fin_rows = 0;
  P.spin_limit = g_fused_spin_limit;
  g_last_fused = LastFused{control0, 0, stream};
  int64_t strips_done = 0;
  for (size_t gi = 0; gi < groups.size(); ++gi) {
    const Group& gr = groups[gi];
    int64_t strips = 0, full = 0;
    int tails = 0;
    int tail_len[kMaxPairs];
    for (int i = 0; i < gr.np; ++i) {
      const int64_t idx = first + gr.g0 + i;
      PairDesc& pd = P.pairs[i];
      pd.slot0 = cache->region_off[idx];
      pd.cap = cache->cap[idx];
      pd.n = cache->len[idx] + (append ? 1 : 0);
      pd.strip0 = static_cast<int32_t>(strips);
      pd.full0 = static_cast<int32_t>(full);
      P.pos_new[i] = append ? pos_new[(gr.g0 + i) % B] : 0;
      strips += std::max<int64_t>(ceil_div(pd.n, strip_rows), 1) * hkv;
      full += static_cast<int64_t>(pd.n / strip_rows) * hkv;
      tail_len[i] = pd.n % strip_rows;
      if (tail_len[i] > 0) P.tail_order[tails++] = static_cast<uint8_t>(i);
    }
    std::stable_sort(P.tail_order, P.tail_order + tails,
                     [&](uint8_t a, uint8_t b) { return tail_len[a] > tail_len[b]; });
    P.n_pairs = gr.np;
    P.pair_base = static_cast<int32_t>(gr.g0);
    P.full_blocks = static_cast<int32_t>(full);
    P.n_tail_pairs = tails;
    P.ws = static_cast<float*>(workspace) + strips_done * seg;
    P.barrier = control0 + 4 * gi;
    const int64_t units = full + static_cast<int64_t>(tails) * hkv;
    const int64_t grid = std::max<int64_t>(1, std::min<int64_t>(n_wgs, units));
    hipLaunchKernelGGL(fused_prepare, dim3(1), dim3(64), 0, stream, P.barrier);
    if (hipGetLastError() != hipSuccess) return gi == 0 ? XKV_ERR_UNSUPPORTED : XKV_ERR_DEVICE;
    void* args[] = {&P};
    const int tok = profile_begin(0, stream);
    const hipError_t err =
        hipLaunchCooperativeKernel(reinterpret_cast<const void*>(fn), dim3(static_cast<unsigned>(grid)),
                                   dim3(kThreads), args, lds, stream);
    profile_end(tok, stream);
    if (err != hipSuccess) {
      (void)hipGetLastError();
      return gi == 0 ? XKV_ERR_UNSUPPORTED : XKV_ERR_DEVICE;
    }
    strips_done += gr.strips;
    g_last_fused.launches = gi + 1;
  }
  return XKV_OK;
}

}  // namespace

void note_waiting_launch(const unsigned* control, void* stream) {
  g_last_fused = LastFused{control, control != nullptr ? size_t{1} : size_t{0}, static_cast<hipStream_t>(stream)};
}

uint32_t fused_spin_limit() { return g_fused_spin_limit; }

size_t attend_workspace_bytes(const xkv_cache* c, int32_t layers) {
  // Upper bound over every strip length a call may choose: logits for cap slots
  // plus one padded strip, and one (o, m, l) block per kChunk slots.
  const int group = c->n_q_heads / c->n_kv_heads;
  const int hkv = c->n_kv_heads;
  const int d = c->head_dim;
  std::vector<size_t> need(static_cast<size_t>(c->n_layers), 0);
  for (int32_t l = 0; l < c->n_layers; ++l)
    for (int32_t b = 0; b < c->batch; ++b) {
      const int64_t cap = c->cap[static_cast<int64_t>(l) * c->batch + b];
      const int64_t floats = (cap + kMaxStripRows) * group +
                             std::max<int64_t>(ceil_div(cap, kChunk), 1) * ((d + 2) * group + 32);
      need[l] += static_cast<size_t>(floats) * hkv * sizeof(float);
    }
  std::sort(need.begin(), need.end(), std::greater<size_t>());
  size_t tot = 0;
  for (int32_t l = 0; l < layers && l < c->n_layers; ++l) tot += need[l];
  // geometry tables of a call with more than kMaxPairs regions, and the (m, 1/l) pairs
  // that the matrix-core path hands from its merge kernel to its score kernel
  const size_t regions = static_cast<size_t>(std::min(layers, c->n_layers)) * c->batch;
  tot += regions * (sizeof(PairDesc) + 12) + regions * hkv * group * 2 * sizeof(float) + 2048;
  return tot;
}

}  // namespace xkv

extern "C" xkv_status xkv_configure(int32_t key, int64_t value) {
  if (key == XKV_CFG_ATTEND_PATH && value >= 0 && value <= 2) {
    xkv::g_attend_path = static_cast<int>(value);
    return XKV_OK;
  }
  if (key == XKV_CFG_FUSED_SPIN_LIMIT && value >= -1 && value <= (int64_t{1} << 30)) {
    xkv::g_fused_spin_limit = value < 0 ? xkv::kDefaultSpinLimit : static_cast<uint32_t>(value);
    return XKV_OK;
  }
  return XKV_ERR_INVALID_ARG;
}

extern "C" xkv_status xkv_fused_status(int32_t* gave_up_out) {
  using namespace xkv;
  if (gave_up_out == nullptr) return XKV_ERR_INVALID_ARG;
  *gave_up_out = 0;
  if (g_last_fused.control == nullptr || g_last_fused.launches == 0) return XKV_OK;
  if (hipStreamSynchronize(g_last_fused.stream) != hipSuccess) return XKV_ERR_DEVICE;
  std::vector<unsigned> words(4 * g_last_fused.launches);
  if (hipMemcpy(words.data(), g_last_fused.control, words.size() * sizeof(unsigned), hipMemcpyDeviceToHost) !=
      hipSuccess)
    return XKV_ERR_DEVICE;
  for (size_t i = 0; i < g_last_fused.launches; ++i)
    if (words[4 * i + 1] != 0) *gave_up_out = 1;
  return XKV_OK;
}

// An eviction that may ride on the finalize kernel (xkv_decode_step): the budgets of the call's regions and
// where the kept indices go; `done` says afterwards whether it did.
struct StepEvict {
  const int32_t* budgets;
  int32_t* kept_idx;
  int32_t pool, n_protect;
  bool done;
};

// The call behind the entry points.  allow_fused: whether the cooperative launch
// may be chosen (it needs occupancy queries; the entry point that must not
// allocate keeps to the two kernels).
static xkv_status decode_attend(xkv_cache* cache, int32_t layer_begin, int32_t layer_end, const void* q,
                                const void* k_new, const void* v_new, const int32_t* pos_new,
                                float softmax_scale, float* out, void* workspace, size_t workspace_bytes,
                                void* hip_stream, bool allow_fused, StepEvict* ev = nullptr) {
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
  Kernels kern;
  if (!pick_kernels(cache->dtype, D, G, &kern)) return XKV_ERR_UNSUPPORTED;

  const int64_t first = static_cast<int64_t>(layer_begin) * B;
  const int64_t n_pairs = static_cast<int64_t>(layer_end - layer_begin) * B;
  int64_t total_rows = 0, max_n = 0;
  for (int64_t i = 0; i < n_pairs; ++i) {
    const int64_t n = static_cast<int64_t>(cache->len[first + i]) + (append ? 1 : 0);
    if (n > cache->cap[first + i]) return XKV_ERR_CAPACITY;
    total_rows += n * hkv;
    max_n = std::max(max_n, n);
  }
  if (workspace == nullptr) return XKV_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return XKV_ERR_INVALID_ARG;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const float scale = softmax_scale > 0.0f ? softmax_scale : 1.0f / std::sqrt(static_cast<float>(D));
  AttendParams P;
  P.q = q; P.k_new = k_new; P.v_new = v_new;
  P.k = cache->k; P.v = cache->v; P.score = cache->score; P.pos = cache->pos; P.out = out;
  P.scale_log2e = scale * 1.44269504088896340736f;
  P.n_kv_heads = hkv;
  P.append = append ? 1 : 0;

  // One cooperative launch per group of regions when everything fits on the chip at once.
  if (allow_fused && (g_attend_path == 2 || (g_attend_path == 0 && kAutoPrefersFused)) && kern.fused != nullptr) {
    const xkv_status fs = launch_fused(cache, first, n_pairs, append, pos_new, P, kern.fused, G, D,
                                       total_rows, workspace, workspace_bytes, stream);
    if (fs == XKV_OK) {
      if (append)
        for (int64_t i = 0; i < n_pairs; ++i) cache->len[first + i] += 1;
      return XKV_OK;
    }
    if (fs != XKV_ERR_UNSUPPORTED || g_attend_path == 2) return fs;
  }

  const int strip_rows = choose_strip_rows(kern.max_strip_rows, n_pairs * hkv, total_rows);
  const bool gqa = kern.merge != nullptr;
  const int64_t rec = gqa ? gqa_record_floats(G, D, strip_rows)
                          : kern.half_records ? half_record_floats(G, D, strip_rows) : record_floats(G, D, strip_rows);
  int64_t total_strips = 0;
  for (int64_t i = 0; i < n_pairs; ++i) {
    const int64_t n = static_cast<int64_t>(cache->len[first + i]) + (append ? 1 : 0);
    total_strips += std::max<int64_t>(ceil_div(n, strip_rows), 1) * hkv;
  }
  // Workspace: the strip records, then (matrix-core path) the streams' (m, 1/l) pairs,
  // then the geometry tables of a call with more regions than the kernel arguments hold.
  const size_t rec_bytes = (static_cast<size_t>(total_strips) * rec * sizeof(float) + 255) / 256 * 256;
  const size_t stats_bytes = gqa ? (static_cast<size_t>(n_pairs) * hkv * G * 2 * sizeof(float) + 255) / 256 * 256 : 0;
  if (rec_bytes + stats_bytes > workspace_bytes) return XKV_ERR_CAPACITY;
  const int64_t max_strips = std::max<int64_t>(ceil_div(max_n, strip_rows), 1);
  const size_t fin_lds = static_cast<size_t>(max_strips) * G * sizeof(float);
  // A finalize workgroup covers up to kMaxStripRows slots, fewer when the streams are
  // short or the call is small and would otherwise leave compute units without one.
  // (short streams: 1024, which balances better; measured on the two GQA workloads)
  const int fin_rows = total_rows / std::max<int64_t>(n_pairs * hkv, 1) < 8192 ? 1024 : kMaxStripRows;
  int fin_strips = std::max(1, fin_rows / strip_rows);
  while (fin_strips > 1 && total_strips / fin_strips < 1024) fin_strips >>= 1;
  if (fin_lds > 48 * 1024) return XKV_ERR_UNSUPPORTED;
  const size_t stream_lds = kern.lds_logits ? static_cast<size_t>(G) * strip_rows * sizeof(float) : 0;

  // The eviction rides on the kernel that updates the scores when every stream evicts few enough tokens.
  bool fuse_evict = ev != nullptr && kern.step[0] != nullptr;
  for (int64_t i = 0; fuse_evict && i < n_pairs; ++i) {
    const int64_t n = static_cast<int64_t>(cache->len[first + i]) + (append ? 1 : 0);
    const int64_t kk = std::min<int64_t>(ev->budgets[i], n);
    // (derived keys cost a pass over the pooled scores per eviction after the first: one eviction only)
    fuse_evict = kk == 0 || n - kk <= ((ev->pool > 1 || ev->n_protect > 0) ? 1 : kStepEvict);
  }
  // Small workgroups once there are two per compute unit of them, or when the streams are short anyway.
  const int step_shape = max_n <= 4096 ? 0 : n_pairs * hkv >= 512 ? (max_n > 8192 ? 1 : 0) : 2;

  P.strip_rows = strip_rows;
  P.rec_floats = static_cast<int32_t>(rec);
  P.lds_rows = 0;
  P.fin_strips = fin_strips;
  P.fin_rows = kGqaScoreRows;
  P.barrier = nullptr;
  P.spin_limit = 0;
  P.stats = reinterpret_cast<float*>(static_cast<char*>(workspace) + rec_bytes);

  if (n_pairs > kMaxPairs) {
    // More regions than the kernel arguments hold: the tables go to device memory
    // (behind the strip records in the workspace) and the call is still one
    // streaming launch and one finalize launch.
    if (n_pairs > std::numeric_limits<int32_t>::max() / 2) return XKV_ERR_UNSUPPORTED;
    const size_t np = static_cast<size_t>(n_pairs);
    std::vector<PairDesc> hp(np);
    std::vector<int32_t> hpos(np), horder(np, 0), hfin(np), tail_len(np);
    int64_t strips = 0, full = 0, fin_blocks = 0, tails = 0;
    for (size_t i = 0; i < np; ++i) {
      const int64_t idx = first + static_cast<int64_t>(i);
      PairDesc& pd = hp[i];
      pd.slot0 = cache->region_off[idx];
      pd.cap = cache->cap[idx];
      pd.n = cache->len[idx] + (append ? 1 : 0);
      if (strips > std::numeric_limits<int32_t>::max() || full > std::numeric_limits<int32_t>::max() ||
          fin_blocks > std::numeric_limits<int32_t>::max())
        return XKV_ERR_UNSUPPORTED;
      pd.strip0 = static_cast<int32_t>(strips);
      pd.full0 = static_cast<int32_t>(full);
      // (a call that evicts in its score kernel has no finalize workgroups to number: the column carries
      // the regions' keep counts instead)
      hfin[i] = fuse_evict ? static_cast<int32_t>(std::min<int64_t>(ev->budgets[i], pd.n))
                           : static_cast<int32_t>(fin_blocks);
      hpos[i] = append ? pos_new[i % B] : 0;
      const int64_t nstrips = std::max<int64_t>(ceil_div(pd.n, strip_rows), 1);
      strips += nstrips * hkv;
      full += static_cast<int64_t>(pd.n / strip_rows) * hkv;
      fin_blocks += (gqa ? std::max<int64_t>(ceil_div(pd.n, kGqaScoreRows), 1) : ceil_div(nstrips, fin_strips)) * hkv;
      tail_len[i] = pd.n % strip_rows;
      if (tail_len[i] > 0) horder[tails++] = static_cast<int32_t>(i);
    }
    std::stable_sort(horder.begin(), horder.begin() + tails,
                     [&](int32_t a, int32_t b) { return tail_len[a] > tail_len[b]; });
    const int64_t blocks = full + tails * hkv;
    if (strips > std::numeric_limits<int32_t>::max() || blocks > std::numeric_limits<int32_t>::max() ||
        fin_blocks > std::numeric_limits<int32_t>::max())
      return XKV_ERR_UNSUPPORTED;
    const size_t table_bytes = np * (sizeof(PairDesc) + 12);
    if (rec_bytes + stats_bytes + table_bytes > workspace_bytes) return XKV_ERR_CAPACITY;
    char* tb = static_cast<char*>(workspace) + rec_bytes + stats_bytes;
    PairDesc* d_pairs = reinterpret_cast<PairDesc*>(tb);
    int32_t* d_pos = reinterpret_cast<int32_t*>(tb + np * sizeof(PairDesc));
    int32_t* d_order = d_pos + np;
    int32_t* d_fin = d_order + np;
    for (size_t c0 = 0; c0 < np; c0 += kTableChunk) {
      TableChunk ch;
      ch.first = static_cast<int32_t>(c0);
      ch.count = static_cast<int32_t>(std::min<size_t>(kTableChunk, np - c0));
      for (int i = 0; i < ch.count; ++i) {
        ch.pairs[i] = hp[c0 + i];
        ch.pos_new[i] = hpos[c0 + i];
        ch.tail_order[i] = horder[c0 + i];
        ch.fin0[i] = hfin[c0 + i];
      }
      hipLaunchKernelGGL(table_write, dim3(1), dim3(kTableChunk), 0, stream, ch, d_pairs, d_pos, d_order, d_fin);
    }
    if (hipGetLastError() != hipSuccess) return XKV_ERR_DEVICE;
    AttendTableParams T;
    static_cast<AttendCommon&>(T) = static_cast<const AttendCommon&>(P);
    T.pairs = d_pairs;
    T.pos_new = d_pos;
    T.tail_order = d_order;
    T.fin0 = d_fin;
    T.n_pairs = static_cast<int32_t>(n_pairs);
    T.pair_base = 0;
    T.full_blocks = static_cast<int32_t>(full);
    T.n_tail_pairs = static_cast<int32_t>(tails);
    T.ws = static_cast<float*>(workspace);
    if (blocks > 0) {
      const int tok = profile_begin(0, stream);
      hipLaunchKernelGGL(kern.stream_tab, dim3(static_cast<unsigned>(gqa ? std::min<int64_t>(blocks, (G == 4 ? 2 : 1) * std::max(compute_units(), 1)) : blocks)), dim3(kThreads), stream_lds,
                         stream, T);
      profile_end(tok, stream);
      if (hipGetLastError() != hipSuccess) return XKV_ERR_DEVICE;
    }
    if (fuse_evict) {
      StepTableParams S;
      static_cast<AttendTableParams&>(S) = T;
      S.keep = d_fin;
      S.kept_idx = ev->kept_idx;
      S.row_bytes = D * (cache->dtype == XKV_F32 ? 4 : 2);
      S.pool = ev->pool;
      S.n_protect = ev->n_protect;
      const int tok = profile_begin(3, stream);
      hipLaunchKernelGGL(kern.step_tab[step_shape], dim3(static_cast<unsigned>(n_pairs * hkv)),
                         dim3(256 << step_shape), fin_lds, stream, S);
      profile_end(tok, stream);
    } else if (gqa) {
      hipLaunchKernelGGL(kern.merge_tab, dim3(static_cast<unsigned>(n_pairs * hkv)), dim3(kThreads), fin_lds, stream, T);
      hipLaunchKernelGGL(kern.finalize_tab, dim3(static_cast<unsigned>(fin_blocks)), dim3(kThreads), 0, stream, T);
    } else {
      hipLaunchKernelGGL(kern.finalize_tab, dim3(static_cast<unsigned>(fin_blocks)), dim3(kThreads), fin_lds,
                         stream, T);
    }
    if (hipGetLastError() != hipSuccess) return XKV_ERR_DEVICE;
    for (int64_t i = 0; append && i < n_pairs; ++i) cache->len[first + i] += 1;
    if (fuse_evict) {
      for (int64_t i = 0; i < n_pairs; ++i)
        cache->len[first + i] = static_cast<int32_t>(std::min<int64_t>(ev->budgets[i], cache->len[first + i]));
      ev->done = true;
    }
    return XKV_OK;
  }

  int64_t strips_done = 0;
  for (int64_t g0 = 0; g0 < n_pairs; g0 += kMaxPairs) {
    const int np = static_cast<int>(std::min<int64_t>(kMaxPairs, n_pairs - g0));
    int64_t strips = 0, full = 0;
    int tails = 0;
    int tail_len[kMaxPairs];
    for (int i = 0; i < np; ++i) {
      const int64_t idx = first + g0 + i;
      PairDesc& pd = P.pairs[i];
      pd.slot0 = cache->region_off[idx];
      pd.cap = cache->cap[idx];
      pd.n = cache->len[idx] + (append ? 1 : 0);
      pd.strip0 = static_cast<int32_t>(strips);
      pd.full0 = static_cast<int32_t>(full);
      P.pos_new[i] = append ? pos_new[(g0 + i) % B] : 0;
      strips += std::max<int64_t>(ceil_div(pd.n, strip_rows), 1) * hkv;
      full += static_cast<int64_t>(pd.n / strip_rows) * hkv;
      tail_len[i] = pd.n % strip_rows;
      if (tail_len[i] > 0) P.tail_order[tails++] = static_cast<uint8_t>(i);
    }
    if (strips > std::numeric_limits<int32_t>::max()) return XKV_ERR_UNSUPPORTED;
    std::stable_sort(P.tail_order, P.tail_order + tails,
                     [&](uint8_t a, uint8_t b) { return tail_len[a] > tail_len[b]; });
    P.n_pairs = np;
    P.pair_base = static_cast<int32_t>(g0);
    P.full_blocks = static_cast<int32_t>(full);
    P.n_tail_pairs = tails;
    P.ws = static_cast<float*>(workspace) + strips_done * rec;
    const int64_t blocks = full + static_cast<int64_t>(tails) * hkv;
    if (blocks > 0) {
      const int tok = profile_begin(0, stream);
      hipLaunchKernelGGL(kern.stream, dim3(static_cast<unsigned>(gqa ? std::min<int64_t>(blocks, (G == 4 ? 2 : 1) * std::max(compute_units(), 1)) : blocks)), dim3(kThreads),
                         stream_lds, stream, P);
      profile_end(tok, stream);
      if (hipGetLastError() != hipSuccess) return XKV_ERR_DEVICE;
    }
    int64_t fin_blocks = 0;
    for (int i = 0; i < np; ++i) {
      PairDesc& pd = P.pairs[i];
      pd.full0 = static_cast<int32_t>(fin_blocks);
      fin_blocks += (gqa ? std::max<int64_t>(ceil_div(pd.n, kGqaScoreRows), 1)
                         : ceil_div(std::max<int64_t>(ceil_div(pd.n, strip_rows), 1), fin_strips)) * hkv;
    }
    if (fuse_evict) {
      StepParams S;
      static_cast<AttendParams&>(S) = P;
      for (int i = 0; i < np; ++i)
        S.keep[i] = static_cast<int32_t>(std::min<int64_t>(ev->budgets[g0 + i], P.pairs[i].n));
      S.kept_idx = ev->kept_idx;
      S.row_bytes = D * (cache->dtype == XKV_F32 ? 4 : 2);
      S.pool = ev->pool;
      S.n_protect = ev->n_protect;
      const int tok = profile_begin(3, stream);
      hipLaunchKernelGGL(kern.step[step_shape], dim3(static_cast<unsigned>(np * hkv)),
                         dim3(256 << step_shape), fin_lds, stream, S);
      profile_end(tok, stream);
    } else if (gqa) {
      hipLaunchKernelGGL(kern.merge, dim3(static_cast<unsigned>(np * hkv)), dim3(kThreads), fin_lds, stream, P);
      hipLaunchKernelGGL(kern.finalize, dim3(static_cast<unsigned>(fin_blocks)), dim3(kThreads), 0, stream, P);
    } else {
      hipLaunchKernelGGL(kern.finalize, dim3(static_cast<unsigned>(fin_blocks)), dim3(kThreads), fin_lds,
                         stream, P);
    }
    if (hipGetLastError() != hipSuccess) return XKV_ERR_DEVICE;
    strips_done += strips;
  }
  if (append)
    for (int64_t i = 0; i < n_pairs; ++i) cache->len[first + i] += 1;
  if (fuse_evict) {
    for (int64_t i = 0; i < n_pairs; ++i)
      cache->len[first + i] = static_cast<int32_t>(std::min<int64_t>(ev->budgets[i], cache->len[first + i]));
    ev->done = true;
  }
  return XKV_OK;
}

extern "C" xkv_status xkv_decode_step(xkv_cache* cache, int32_t layer_begin, int32_t layer_end, const void* q,
                                      const void* k_new, const void* v_new, const int32_t* pos_new,
                                      float softmax_scale, float* out, const int32_t* budgets, int32_t pool_size,
                                      int32_t n_protect, int32_t* kept_idx_out, void* workspace,
                                      size_t workspace_bytes, void* hip_stream) {
  using namespace xkv;
  // Everything xkv_evict_compact would refuse is refused here, before the attention is enqueued.
  xkv_status st = check_cache(cache);
  if (st != XKV_OK) return st;
  st = check_layers(cache, layer_begin, layer_end);
  if (st != XKV_OK) return st;
  st = evict_check_args(cache, layer_begin, layer_end, budgets, pool_size, n_protect, k_new != nullptr ? 1 : 0,
                        workspace, workspace_bytes);
  if (st != XKV_OK) return st;
  StepEvict ev{budgets, kept_idx_out, pool_size, n_protect, false};
  st = decode_attend(cache, layer_begin, layer_end, q, k_new, v_new, pos_new, softmax_scale, out, workspace,
                     workspace_bytes, hip_stream, true, &ev);
  if (st != XKV_OK || ev.done) return st;
  return xkv_evict_compact(cache, layer_begin, layer_end, budgets, pool_size, n_protect, kept_idx_out, workspace,
                           workspace_bytes, hip_stream);
}

extern "C" xkv_status xkv_decode_attend_score(xkv_cache* cache, int32_t layer_begin,
                                              int32_t layer_end, const void* q, const void* k_new,
                                              const void* v_new, const int32_t* pos_new,
                                              float softmax_scale, float* out, void* workspace,
                                              size_t workspace_bytes, void* hip_stream) {
  return decode_attend(cache, layer_begin, layer_end, q, k_new, v_new, pos_new, softmax_scale, out, workspace,
                       workspace_bytes, hip_stream, true);
}

// ---- the entry point that allocates nothing ------------------------------------
// Its strip records live in a fixed array of the library's own device image
// instead of a caller's workspace.  In host code the array's name is only a
// stand-in: the device address of each GPU's copy is looked up once per device
// and that pointer is what the kernels receive.
namespace xkv {
namespace {
constexpr size_t kStaticScratchBytes = XKV_NOALLOC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
}  // namespace
}  // namespace xkv

static __device__ __align__(256) unsigned char scratch[xkv::kStaticScratchBytes];

namespace xkv {
namespace {
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of the current device's copy of `scratch`, resolved on the first
// call on that device; nullptr (and *err set) if the lookup fails.
void* static_scratch(xkv_status* err) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    (void)hipGetLastError();
    *err = XKV_ERR_DEVICE;
    return nullptr;
  }
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
      (void)hipGetLastError();
      *err = XKV_ERR_DEVICE;
      return nullptr;
    }
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}
}  // namespace
}  // namespace xkv

extern "C" xkv_status xkv_decode_attend_score_noalloc(xkv_cache* cache, int32_t layer_begin,
                                                      int32_t layer_end, const void* q,
                                                      const void* k_new, const void* v_new,
                                                      const int32_t* pos_new, float softmax_scale,
                                                      float* out, void* hip_stream) {
  xkv_status err = XKV_OK;
  void* ws = xkv::static_scratch(&err);
  if (ws == nullptr) return err;
  // A call that needs more than the array holds is refused with XKV_ERR_CAPACITY by
  // the same check that guards a caller's workspace.
  return decode_attend(cache, layer_begin, layer_end, q, k_new, v_new, pos_new, softmax_scale, out, ws,
                       xkv::kStaticScratchBytes, hip_stream, false);
}
