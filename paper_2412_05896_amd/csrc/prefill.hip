// xkv_prefill_evict: the eviction of the prefill phase, Alg. 2 of the paper as
// written, from a dense prompt into the ragged cache.
//
//   step 1-3  W_attn of the observation window (Eq. 2, causal), Select, Merge:
//             w[j] = sum over the G query heads and the ows window rows of the
//             probability that row gives to prompt position j  (Eq. 3, Sec. 4.1)
//   step 4    Pooling over the candidate vector w[0 .. t - ows)
//   step 5    TopK: the budget - ows best candidates; the window is always kept
//   step 6-7  EvictByIndex: the kept rows of K and V, in prompt order, are
//             gathered into the stream's slots, with score = w and pos = position
//
// The window's queries against the prompt's keys are a dense contraction with
// Nq = ows * G query rows per KV head: it runs on the matrix cores (bf16
// 16x16x32 MFMA, or the fp32 16x16x4 MFMA for fp32 caches).  The softmax needs
// each query row's maximum and sum before any probability is final, so K is read
// twice: window_stats reduces (max, sum) per (stream, strip, query row),
// window_merge folds the strips, window_mass recomputes the logits and writes w.
// Storing the Nq logits per token instead would write and read 4 Nq bytes per
// token next to a K row of 256.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <limits>
#include <type_traits>

#include "device_util.h"
#include "select_util.h"
#include "xkv_internal.h"

namespace xkv {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kSelThreads = 1024;          // prefill_select: one large workgroup per stream
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kMaxNq = 64;                 // query rows (ows * G) per KV head
constexpr int kMaxSeqLens = 256;           // sequences with a prompt length of their own
constexpr int kMaxKeyRegs = 32;            // prefill_select: keys a thread keeps in registers
constexpr int kMaxWalkRows = 256;          // prefill_select without register keys: rows of candidates
// Selection of a long stream split over several workgroups (see split_*): candidates per
// workgroup, and the words of per-stream state: 4 histograms, threshold and need, (gt, eq) per chunk.
constexpr int kSplitKeys = 8;
constexpr int kSplitChunk = kSplitKeys * kSelThreads;
constexpr int kSplitMaxChunks = kMaxWalkRows * kSelThreads / kSplitChunk;
constexpr int kSplitCounts = 4 * 256 + 2;                     // first (gt, eq) pair
constexpr int kSplitFlag = kSplitCounts + 2 * kSplitMaxChunks;  // one-launch variant: some wait of the stream gave up
constexpr int kSplitWords = kSplitFlag + 2;
constexpr unsigned kSplitSpinLimit = 1u << 16;              // most polls (some microseconds each) of a wait of the one-launch selection
constexpr unsigned kSplitValid = 0x80000000u;               // a chunk's packed (gt, eq) word has been published

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

struct WindowParams {
  const void* q_win;      // [pairs][Hq][ows][D]
  const void* k_src;      // [pairs][Hkv][t][D]
  const float* lse;       // [pairs][Hq][ows] natural-log normalisers of the window rows from the caller, or null
  float* stats;           // [streams][nstrips][nq_pad][2]  (max, sum) in the base-2 domain
  float* fin;             // [streams][nq_pad][2]           (max, 1 / sum)
  float* w;               // [streams][t]
  unsigned short* dlog;   // one-pass variant: [streams][t_pad][NQS] 16-bit logit distances
  float* tref;            // one-pass variant: [streams][t_pad / 32][NQS] reference of every tile of 32 rows
  unsigned* split;        // [streams][kSplitWords] state of the selection that follows, zeroed by window_merge (or null)
  unsigned* call_flag;    // with split: the call's 4 control words, zeroed with it
  float scale_log2e;
  int32_t t, ows, group, n_kv_heads;      // t: rows per stream of k_src and w (the longest prompt)
  int32_t strip_rows, nstrips, nq_pad;
  int32_t t_pad;                          // t rounded up to a multiple of 32 (one-pass variant)
  int32_t n_seq;                          // entries of t_seq: the batch, or 1 when all prompts have t tokens
  int32_t t_seq[kMaxSeqLens];             // prompt length of sequence b (pair % n_seq)
};

// One MFMA step over the 16 bytes that lane (j, x) holds of row x of A and of
// column x of B, at byte offset 64 sl + 16 j of both: 8 bf16 channels, or 4 fp32
// channels taken one at a time.  Which channels a step contracts does not
// matter as long as both operands agree and all are visited.
template <typename T>
__device__ __forceinline__ floatx4 mma16(const uint4& a, const uint4& b, floatx4 c) {
  if constexpr (std::is_same<T, BF16>::value) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  } else {
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
    return c;
  }
}

// (max, sum) of two parts of a softmax row, base-2 domain; an empty part has max -inf.
__device__ __forceinline__ void merge_ml(float& m, float& l, float m2, float l2) {
  const float mn = fmaxf(m, m2);
  const float ms = mn == -INFINITY ? 0.0f : mn;
  l = l * fast_exp2(m - ms) + l2 * fast_exp2(m2 - ms);
  m = mn;
}

// Logits of 16 prompt rows against the NB blocks of 16 query rows.
//   kPhase 0  window_stats: per-strip (max, sum) of every query row
//   kPhase 1  window_mass:  w[j] = sum over query rows of 2^(s - max) / sum
// Workgroup = (stream, strip); its waves take the strip's groups of 16 rows in
// turn.  Lane (j, x): an operand is 16 bytes at offset 64 sl + 16 j of K row x of
// the group and of query row 16 nb + x; the result has the logit of
// (row 4 j + i, query row 16 nb + x) in register i.
template <typename T, int D, int NB, int kPhase>
__global__ __launch_bounds__(kThreads) void window_pass(const WindowParams P) {
  constexpr int ROWB = D * T::kBytes;
  constexpr int NSL = ROWB / 64;
  __shared__ float ml_sh[kWaves][NB * 16][2];
  __shared__ __attribute__((aligned(16))) char tile_sh[kWaves][2][16 * (ROWB + 16)];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int x = lane & 15, j = lane >> 4;
  const int u = blockIdx.x / P.nstrips;             // stream = (pair, KV head)
  const int s = blockIdx.x - u * P.nstrips;
  const int pair = u / P.n_kv_heads;
  const int h = u - pair * P.n_kv_heads;
  const int t = P.t_seq[pair % P.n_seq], ows = P.ows;   // this sequence's prompt length
  const int nq = ows * P.group;
  const int r_begin = s * P.strip_rows;
  if (r_begin >= t) return;                         // strip past the end of a shorter prompt
  const int r_end = min(t, r_begin + P.strip_rows);
  const char* kbase = static_cast<const char*>(P.k_src) + static_cast<int64_t>(u) * P.t * ROWB;

  // Query operands; query row qi = g * ows + r is head g, window row r.
  uint4 qreg[NB][NSL];
  int last_col[NB];                                 // last position the lane's query row sees
  float m_fin[NB] = {}, inv_fin[NB] = {};
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const int qi = nb * 16 + x;
    const bool live = qi < nq;
    const int g = live ? qi / ows : 0;
    const int r = live ? qi - g * ows : 0;
    last_col[nb] = live ? t - ows + r : -1;
    const int64_t qrow = (static_cast<int64_t>(pair) * P.n_kv_heads * P.group + h * P.group + g) * ows + r;
#pragma unroll
    for (int sl = 0; sl < NSL; ++sl) {
      uint4 raw = make_uint4(0, 0, 0, 0);
      if (live) raw = *reinterpret_cast<const uint4*>(static_cast<const char*>(P.q_win) + qrow * ROWB + sl * 64 + j * 16);
      qreg[nb][sl] = raw;
    }
    if (kPhase == 1) {
      if (P.lse != nullptr) {
        // The caller's normalisers: 2^(s - lse log2 e), nothing to divide by.
        const int64_t row = (static_cast<int64_t>(u) * P.group + g) * ows + r;   // (pair, KV head, g) = (pair, query head)
        m_fin[nb] = live ? P.lse[row] * 1.44269504088896340736f : 0.0f;
        inv_fin[nb] = live ? 1.0f : 0.0f;
      } else {
        const float* f = P.fin + (static_cast<int64_t>(u) * P.nq_pad + qi) * 2;
        m_fin[nb] = f[0];
        inv_fin[nb] = f[1];
      }
    }
  }
  if (kPhase == 1 && P.lse != nullptr && P.split != nullptr && s == 0) {
    // No merge kernel runs on this path: the stream's first strip clears the state words of the selection.
    unsigned* st = P.split + static_cast<int64_t>(u) * kSplitWords;
    for (int i = tid; i < kSplitWords; i += kThreads) st[i] = 0u;
    if (u == 0 && tid < 4) P.call_flag[tid] = 0u;
  }

  float m_run[NB], l_run[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) { m_run[nb] = -INFINITY; l_run[nb] = 0.0f; }

  const int groups = (r_end - r_begin + 15) / 16;
  // A group's 16 K rows are read as whole rows (lane (rr, cx): 16 bytes at column cx of
  // row i * RPI + rr for load i) and turned into the operand layout (row x, 16 bytes at
  // column 4 sl + j) through a per-wave LDS tile with padded rows.
  constexpr int LPR = ROWB / 16, RPI = 64 / LPR, kPitch = ROWB + 16;
  const int rr = lane / LPR, cx = lane % LPR;
  auto load_group = [&](uint4 (&kreg)[NSL], int gi) {
#pragma unroll
    for (int i = 0; i < NSL; ++i) {
      const int row = r_begin + gi * 16 + i * RPI + rr;
      const int rc = row < t ? row : t - 1;         // rows past the end repeat the last one, masked below
      kreg[i] = load_stream16(kbase + static_cast<int64_t>(rc) * ROWB + cx * 16);
    }
  };
  auto use_group = [&](const uint4 (&kraw)[NSL], int gi, char* tile) {
    const int g0 = r_begin + gi * 16;
#pragma unroll
    for (int i = 0; i < NSL; ++i)
      *reinterpret_cast<uint4*>(tile + (i * RPI + rr) * kPitch + cx * 16) = kraw[i];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    uint4 kreg[NSL];
#pragma unroll
    for (int sl = 0; sl < NSL; ++sl)
      kreg[sl] = *reinterpret_cast<const uint4*>(tile + x * kPitch + sl * 64 + j * 16);
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    float wsum[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      floatx4 a = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
      for (int sl = 0; sl < NSL; ++sl) a = mma16<T>(kreg[sl], qreg[nb][sl], a);
      if (kPhase == 0) {
        float sv[4];
        float gm = -INFINITY;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          sv[i] = g0 + 4 * j + i <= last_col[nb] ? a[i] * P.scale_log2e : -INFINITY;   // causal
          gm = fmaxf(gm, sv[i]);
        }
        const float m_new = fmaxf(m_run[nb], gm);
        const float m_safe = m_new == -INFINITY ? 0.0f : m_new;
        float l = l_run[nb] * fast_exp2(m_run[nb] - m_safe);
#pragma unroll
        for (int i = 0; i < 4; ++i) l += fast_exp2(sv[i] - m_safe);
        m_run[nb] = m_new;
        l_run[nb] = l;
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const bool seen = g0 + 4 * j + i <= last_col[nb];
          wsum[i] += seen ? fast_exp2(a[i] * P.scale_log2e - m_fin[nb]) * inv_fin[nb] : 0.0f;
        }
      }
    }
    if (kPhase == 1) {
      // Sum over the 16 query rows that share a lane row, then lane x < 4 of row j
      // stores position g0 + 4 j + x.
      float mine = 0.0f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float tot = group_sum<16>(wsum[i]);
        if (x == i) mine = tot;
      }
      const int pos = g0 + 4 * j + x;
      if (x < 4 && pos < t) P.w[static_cast<int64_t>(u) * P.t + pos] = mine;
    }
  };
  // Two groups per turn, both requested before either is used.
  for (int gi = wave; gi < groups; gi += 2 * kWaves) {
    uint4 ka[NSL], kb[NSL];
    const bool two = gi + kWaves < groups;
    load_group(ka, gi);
    if (two) load_group(kb, gi + kWaves);
    use_group(ka, gi, tile_sh[wave][0]);
    if (two) use_group(kb, gi + kWaves, tile_sh[wave][1]);
  }

  if (kPhase == 0) {
    // Fold the four row quarters of the wave, then the waves.
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
      for (int off = 16; off < 64; off <<= 1) {
        const float m2 = __shfl_xor(m_run[nb], off);
        const float l2 = __shfl_xor(l_run[nb], off);
        merge_ml(m_run[nb], l_run[nb], m2, l2);
      }
      if (j == 0) {
        ml_sh[wave][nb * 16 + x][0] = m_run[nb];
        ml_sh[wave][nb * 16 + x][1] = l_run[nb];
      }
    }
    __syncthreads();
    if (tid < NB * 16) {
      float m = ml_sh[0][tid][0], l = ml_sh[0][tid][1];
#pragma unroll
      for (int w = 1; w < kWaves; ++w) merge_ml(m, l, ml_sh[w][tid][0], ml_sh[w][tid][1]);
      float* st = P.stats + ((static_cast<int64_t>(u) * P.nstrips + s) * P.nq_pad + tid) * 2;
      st[0] = m;
      st[1] = l;
    }
  }
}

// ---------------------------------------------------------------------------
// One-pass variant for at most 16 query rows per KV head over bf16 keys: K is read
// once.  window_stats_store computes the logits like window_pass phase 0 and,
// besides the strip statistics, stores every logit as a 16-bit fixed-point
// distance d = (ref - s) * 2^10 below a reference that is kept once per tile of 32
// rows and query row (the wave's running maximum at that tile): 2 NQS bytes per
// token next to a K row of 256, against reading K a second time.  window_mass_stored
// then needs only those: w[j] = sum over the seen query rows of
// 2^(ref - d / 2^10 - m) / l.  A probability carries a relative error of at most
// ln 2 * 2^-11 = 3.4e-4, far inside what bf16 inputs allow; fp32 caches keep the
// two K passes.
constexpr float kLogitFixScale = 1024.0f;
constexpr int kStoreTile = 32;

template <int D, int NQS>
__global__ __launch_bounds__(kThreads) void window_stats_store(const WindowParams P) {
  using T = BF16;
  constexpr int ROWB = D * T::kBytes;
  constexpr int NSL = ROWB / 64;
  constexpr int kMaxTiles = 1024 / kStoreTile;          // strips have at most 1024 rows
  __shared__ float ml_sh[kWaves][16][2];
  __shared__ __attribute__((aligned(16))) char tile_sh[kWaves][2][16 * (ROWB + 16)];
  __shared__ __attribute__((aligned(16))) unsigned short d_sh[kWaves][kStoreTile * NQS];
  __shared__ float tref_sh[kMaxTiles][NQS];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int x = lane & 15, j = lane >> 4;
  const int u = blockIdx.x / P.nstrips;
  const int s = blockIdx.x - u * P.nstrips;
  const int pair = u / P.n_kv_heads;
  const int h = u - pair * P.n_kv_heads;
  const int t = P.t_seq[pair % P.n_seq], ows = P.ows;
  const int nq = ows * P.group;
  const int r_begin = s * P.strip_rows;
  if (r_begin >= t) return;
  const int r_end = min(t, r_begin + P.strip_rows);
  const char* kbase = static_cast<const char*>(P.k_src) + static_cast<int64_t>(u) * P.t * ROWB;

  uint4 qreg[NSL];
  const bool live = x < nq;
  const int g = live ? x / ows : 0;
  const int r = live ? x - g * ows : 0;
  const int last_col = live ? t - ows + r : -1;         // last position the lane's query row sees
  {
    const int64_t qrow = (static_cast<int64_t>(pair) * P.n_kv_heads * P.group + h * P.group + g) * ows + r;
#pragma unroll
    for (int sl = 0; sl < NSL; ++sl) {
      uint4 raw = make_uint4(0, 0, 0, 0);
      if (live) raw = *reinterpret_cast<const uint4*>(static_cast<const char*>(P.q_win) + qrow * ROWB + sl * 64 + j * 16);
      qreg[sl] = raw;
    }
  }
  float m_run = -INFINITY;                  // query row x, all rows of this wave so far
  float l_run = 0.0f;                       // query row x, this lane's rows only

  constexpr int LPR = ROWB / 16, RPI = 64 / LPR, kPitch = ROWB + 16;
  const int rr = lane / LPR, cx = lane % LPR;
  auto load_group = [&](uint4 (&kreg)[NSL], int row0) {
#pragma unroll
    for (int i = 0; i < NSL; ++i) {
      const int row = row0 + i * RPI + rr;
      const int rc = row < t ? row : t - 1;             // rows past the end repeat the last one, masked below
      kreg[i] = load_stream16(kbase + static_cast<int64_t>(rc) * ROWB + cx * 16);
    }
  };
  // Stages 16 rows in the wave's LDS tile (after which their registers are free again).
  auto stage = [&](const uint4 (&kraw)[NSL], char* tile) {
#pragma unroll
    for (int i = 0; i < NSL; ++i)
      *reinterpret_cast<uint4*>(tile + (i * RPI + rr) * kPitch + cx * 16) = kraw[i];
  };
  // Logits of the 16 staged rows from row0 on: sv[i] belongs to (row0 + 4 j + i, query row x).
  auto logits = [&](int row0, const char* tile, float (&sv)[4]) {
    floatx4 a = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int sl = 0; sl < NSL; ++sl) {
      const uint4 kop = *reinterpret_cast<const uint4*>(tile + x * kPitch + sl * 64 + j * 16);
      a = mma16<T>(kop, qreg[sl], a);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) sv[i] = row0 + 4 * j + i <= last_col ? a[i] * P.scale_log2e : -INFINITY;   // causal
  };

  // A wave takes tiles wave, wave + 4, ... of the strip.  The rows of its next tile
  // are requested as soon as the current ones sit in LDS, and the tile's distances
  // are stored after that request, so that no wait for K rows covers the store.
  const int tiles = (r_end - r_begin + kStoreTile - 1) / kStoreTile;
  unsigned short* dl = P.dlog + (static_cast<int64_t>(u) * P.t_pad + r_begin) * NQS;
  uint4 ka[NSL], kb[NSL];
  if (wave < tiles) {
    load_group(ka, r_begin + wave * kStoreTile);
    load_group(kb, r_begin + wave * kStoreTile + 16);
  }
  for (int tt = wave; tt < tiles; tt += kWaves) {
    const int row0 = r_begin + tt * kStoreTile;
    stage(ka, tile_sh[wave][0]);
    stage(kb, tile_sh[wave][1]);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_sched_barrier(0);
    if (tt + kWaves < tiles) {
      load_group(ka, row0 + kWaves * kStoreTile);
      load_group(kb, row0 + kWaves * kStoreTile + 16);
    }
    __builtin_amdgcn_sched_barrier(0);
    float sa[4], sb[4];
    logits(row0, tile_sh[wave][0], sa);
    logits(row0 + 16, tile_sh[wave][1], sb);
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    float tm = fmaxf(fmaxf(fmaxf(sa[0], sa[1]), fmaxf(sa[2], sa[3])), fmaxf(fmaxf(sb[0], sb[1]), fmaxf(sb[2], sb[3])));
    tm = fmaxf(tm, __shfl_xor(tm, 16));
    tm = fmaxf(tm, __shfl_xor(tm, 32));
    const float m_new = fmaxf(m_run, tm);
    const float m_safe = m_new == -INFINITY ? 0.0f : m_new;     // padding query rows see nothing
    float ls = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i) ls += fast_exp2(sa[i] - m_safe) + fast_exp2(sb[i] - m_safe);
    l_run = fmaf(l_run, fast_exp2(m_run - m_safe), ls);
    m_run = m_new;
    if (x < NQS) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float da = fminf((m_safe - sa[i]) * kLogitFixScale, 65535.0f);
        const float db = fminf((m_safe - sb[i]) * kLogitFixScale, 65535.0f);
        d_sh[wave][(4 * j + i) * NQS + x] = static_cast<unsigned short>(__float2uint_rn(da));
        d_sh[wave][(16 + 4 * j + i) * NQS + x] = static_cast<unsigned short>(__float2uint_rn(db));
      }
      if (j == 0) tref_sh[tt][x] = m_safe;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    if (8 * lane < kStoreTile * NQS) {                  // the tile's block [row][query row], 64 NQS bytes, one store
      const uint4 dv = *reinterpret_cast<const uint4*>(&d_sh[wave][8 * lane]);
      store_stream16(dl + static_cast<int64_t>(tt) * kStoreTile * NQS + 8 * lane, dv);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_sched_barrier(0);
  }

  // The waves' statistics: every lane of a wave has the wave's maximum; the sums
  // of the four row quarters are added, then the waves merged.
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);
  if (j == 0) {
    ml_sh[wave][x][0] = m_run;
    ml_sh[wave][x][1] = l_run;
  }
  __syncthreads();
  if (tid < 16) {
    float m = ml_sh[0][tid][0], l = ml_sh[0][tid][1];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) merge_ml(m, l, ml_sh[w][tid][0], ml_sh[w][tid][1]);
    float* st = P.stats + ((static_cast<int64_t>(u) * P.nstrips + s) * P.nq_pad + tid) * 2;
    st[0] = m;
    st[1] = l;
  }
  float* tr = P.tref + (static_cast<int64_t>(u) * (P.t_pad / kStoreTile) + r_begin / kStoreTile) * NQS;
  for (int idx = tid; idx < tiles * NQS; idx += kThreads) store_stream(&tr[idx], tref_sh[idx / NQS][idx % NQS]);
}

// Final (max, 1 / sum) of query row tid of stream u, for tid < nq_pad, from the
// strips' stats: thread (slice, qi) folds every S-th strip of query row qi, then
// the slices are folded in order.  Every thread of the workgroup calls it; has a
// barrier.
__device__ __forceinline__ void stream_fin(const WindowParams& P, int u, float (*part_sh)[2], float& m_out,
                                           float& inv_l_out) {
  const int tid = threadIdx.x;
  const int nq = P.nq_pad;                    // 16, 32, 48 or 64
  const int S = kThreads / nq;
  const int qi = tid % nq, slice = tid / nq;
  const int t = P.t_seq[(u / P.n_kv_heads) % P.n_seq];
  const int nstrips = (t + P.strip_rows - 1) / P.strip_rows;   // the strips this sequence's prompt has
  float m = -INFINITY, l = 0.0f;
  if (slice < S)
    for (int s = slice; s < nstrips; s += S) {
      const float* st = P.stats + ((static_cast<int64_t>(u) * P.nstrips + s) * nq + qi) * 2;
      merge_ml(m, l, st[0], st[1]);
    }
  part_sh[tid][0] = m;
  part_sh[tid][1] = l;
  __syncthreads();
  if (tid < nq)
    for (int sl = 1; sl < S; ++sl) merge_ml(m, l, part_sh[sl * nq + tid][0], part_sh[sl * nq + tid][1]);
  m_out = m == -INFINITY ? 0.0f : m;          // padding rows: any finite value, they are never seen
  inv_l_out = l > 0.0f ? 1.0f / l : 0.0f;
}

// w[j] for 256 positions per workgroup from the stored distances.
template <int NQS>
__global__ __launch_bounds__(kThreads) void window_mass_stored(const WindowParams P) {
  typedef unsigned int uintxq __attribute__((ext_vector_type(NQS / 2)));
  typedef float floatxq __attribute__((ext_vector_type(NQS)));
  const int u = blockIdx.y;
  const int pair = u / P.n_kv_heads;
  const int t = P.t_seq[pair % P.n_seq], ows = P.ows;
  const int jpos = blockIdx.x * kThreads + threadIdx.x;
  if (jpos >= t) return;
  const int nq = ows * P.group;
  const uintxq dv = __builtin_nontemporal_load(
      reinterpret_cast<const uintxq*>(P.dlog + (static_cast<int64_t>(u) * P.t_pad + jpos) * NQS));
  const floatxq ref = *reinterpret_cast<const floatxq*>(
      P.tref + (static_cast<int64_t>(u) * (P.t_pad / kStoreTile) + jpos / kStoreTile) * NQS);
  const float* fin = P.fin + static_cast<int64_t>(u) * P.nq_pad * 2;
  float acc = 0.0f;
#pragma unroll
  for (int qi = 0; qi < NQS; ++qi) {
    const unsigned word = dv[qi >> 1];
    const float dist = static_cast<float>((qi & 1) ? (word >> 16) : (word & 0xffffu));
    const int r = qi % ows;                             // query row qi is head qi / ows, window row qi % ows
    const bool seen = qi < nq && jpos <= t - ows + r;   // causal
    const float p = fast_exp2(fmaf(dist, -1.0f / kLogitFixScale, ref[qi] - fin[2 * qi])) * fin[2 * qi + 1];
    acc += seen ? p : 0.0f;
  }
  P.w[static_cast<int64_t>(u) * P.t + jpos] = acc;
}

// One workgroup per stream: the final stats of every query row, folded from the
// strips'; it also clears the state words of the selection that follows (if one
// does).  (With the caller's normalisers the single K pass does both itself.)
__global__ __launch_bounds__(kThreads) void window_merge(const WindowParams P) {
  __shared__ float part_sh[kThreads][2];
  const int u = blockIdx.x;
  if (P.split != nullptr) {
    unsigned* st = P.split + static_cast<int64_t>(u) * kSplitWords;
    for (int i = threadIdx.x; i < kSplitWords; i += kThreads) st[i] = 0u;
    if (u == 0 && threadIdx.x < 4) P.call_flag[threadIdx.x] = 0u;
  }
  float fm, fil;
  stream_fin(P, u, part_sh, fm, fil);
  if (static_cast<int>(threadIdx.x) < P.nq_pad) {
    float* f = P.fin + (static_cast<int64_t>(u) * P.nq_pad + threadIdx.x) * 2;
    f[0] = fm;
    f[1] = fil;
  }
}

// ---- selection and gather ---------------------------------------------------
struct GatherPair {
  int64_t slot0;   // first slot of the region
  int32_t cap;     // slots per stream
  int32_t k;       // tokens kept: min(budget, t)
  int32_t t;       // prompt length of the region's sequence
};

struct GatherParams {
  const void* k_src;
  const void* v_src;
  void* k;
  void* v;
  float* score;
  int32_t* pos;
  const float* w;        // [streams][t]
  uint32_t* keys;        // [streams][t] pooled keys (only used when pool > 1)
  int32_t* idx;          // [streams][t] kept positions, ascending
  unsigned* split;       // [streams][kSplitWords]: state of the selection split over several workgroups
  unsigned* call_flag;   // 4 control words of the call (word 1: some wait of split_fused gave up), zeroed by window_merge
  int32_t check_flag;    // the gather skips streams whose selection gave up
  uint32_t spin_limit;   // polls of a wait of split_fused before it gives up
  int32_t t, ows, pool, n_kv_heads, row_bytes;   // t: rows per stream of the dense arrays
  int32_t stream0;       // index of this launch's first stream within the call
  GatherPair pairs[kMaxPairs];
};

// One workgroup per stream: pooled keys of the candidates, the threshold of
// the top kc = k - ows of them by radix select, then a walk in prompt order that
// numbers the kept candidates (equal keys: lower position first); the window's
// positions follow.  Thread `tid` owns candidates tid, tid + 1024, ...; with
// KPT > 0 it keeps their keys in KPT registers (tc <= 1024 KPT), otherwise they
// go through the workspace.
template <int KPT>
__global__ __launch_bounds__(kSelThreads) void prefill_select(const GatherParams P) {
  extern __shared__ float wpad_sh[];                // staged candidates, see below
  __shared__ RadixShared radix_sh;
  constexpr int kMaxRows = KPT > 0 ? KPT : kMaxWalkRows;
  __shared__ int eq_sh[kMaxRows * kSelWaves], keep_sh[kMaxRows * kSelWaves];
  __shared__ int tot_sh[kSelWaves + 1];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int ul = blockIdx.x;                        // stream within the launch
  const GatherPair pd = P.pairs[ul / P.n_kv_heads];
  const int64_t u = static_cast<int64_t>(P.stream0) + ul;
  const int t = P.t, tc = pd.t - P.ows;
  const int kc = pd.k - P.ows;                      // candidates to keep
  const float* w = P.w + u * t;
  uint32_t* keys = P.keys + u * t;
  int32_t* idx = P.idx + u * t;

  for (int r = tid; r < P.ows; r += kSelThreads) idx[kc + r] = tc + r;
  if (kc >= tc) {                                   // every candidate stays
    for (int jx = tid; jx < tc; jx += kSelThreads) idx[jx] = jx;
    return;
  }
  if (kc == 0) return;

  // With pooling and register-resident keys the candidate vector is staged in
  // LDS (zeros on both sides), so that the window sums read it from there.
  const int half = P.pool >> 1;
  const bool staged = KPT > 0 && P.pool > 1;
  if (staged) {
    for (int c = tid; c < tc + 2 * half; c += kSelThreads)
      wpad_sh[c] = (c >= half && c < tc + half) ? w[c - half] : 0.0f;
    __syncthreads();
  }
  auto make_key = [&](int jx) -> unsigned {
    if (P.pool == 1) return __float_as_uint(w[jx]);
    // window sum, fp32, left to right, zeros outside the candidate vector
    float acc;
    if (staged) {
      acc = wpad_sh[jx];                              // candidate jx - half
      for (int q = 1; q < P.pool; ++q) acc = acc + wpad_sh[jx + q];
    } else {
      int c = jx - half;
      acc = (c >= 0 && c < tc) ? w[c] : 0.0f;
      for (int q = 1; q < P.pool; ++q) {
        ++c;
        const float term = (c >= 0 && c < tc) ? w[c] : 0.0f;
        acc = acc + term;
      }
    }
    return __float_as_uint(acc);
  };
  constexpr int NK = KPT > 0 ? KPT : 1;
  unsigned kreg[NK];
  const bool stored = KPT == 0 && P.pool > 1;
  if (KPT > 0) {
#pragma unroll
    for (int i = 0; i < NK; ++i) {
      const int jx = i * kSelThreads + tid;
      kreg[i] = jx < tc ? make_key(jx) : 0u;
    }
  } else if (stored) {
    for (int jx = tid; jx < tc; jx += kSelThreads) keys[jx] = make_key(jx);
    __syncthreads();
  }
  auto key_at = [&](int jx) -> unsigned { return stored ? keys[jx] : __float_as_uint(w[jx]); };
  auto for_each_key = [&](auto&& fn) {
    if (KPT > 0) {
#pragma unroll
      for (int i = 0; i < NK; ++i)
        if (i * kSelThreads + tid < tc) fn(kreg[i]);
    } else {
      for (int jx = tid; jx < tc; jx += kSelThreads) fn(key_at(jx));
    }
  };

  unsigned thr, need;
  radix_select(for_each_key, kc, radix_sh, thr, need);

  // Walk in prompt order.  Row i of the walk is candidates 1024 i .. 1024 i + 1023,
  // one per thread; (row, wave) cells hold first the number of keys equal to the
  // threshold, then the number of kept keys, and a prefix sum over the cells
  // gives every wave of every row its starting rank.
  const int rows = (tc + kSelThreads - 1) / kSelThreads;
  auto for_each_row = [&](auto&& fn) {
    if (KPT > 0) {
#pragma unroll
      for (int i = 0; i < NK; ++i)
        if (i < rows) fn(i, kreg[i]);
    } else {
      for (int i = 0; i < rows; ++i) {
        const int jx = i * kSelThreads + tid;
        fn(i, jx < tc ? key_at(jx) : 0u);
      }
    }
  };
  for_each_row([&](int i, unsigned key) {
    const bool is_eq = i * kSelThreads + tid < tc && key == thr;
    const unsigned long long v_eq = __ballot(is_eq);
    if (lane == 0) eq_sh[i * kSelWaves + wave] = __popcll(v_eq);
  });
  block_exclusive_scan<kSelThreads>(eq_sh, rows * kSelWaves, tot_sh);
  auto kept = [&](int i, unsigned key) -> bool {
    const bool live = i * kSelThreads + tid < tc;
    const bool is_eq = live && key == thr;
    const unsigned long long v_eq = __ballot(is_eq);
    const int eq_rank = eq_sh[i * kSelWaves + wave] + rank_in_wave(v_eq);
    return live && (key > thr || (is_eq && eq_rank < static_cast<int>(need)));
  };
  for_each_row([&](int i, unsigned key) {
    const unsigned long long v_k = __ballot(kept(i, key));
    if (lane == 0) keep_sh[i * kSelWaves + wave] = __popcll(v_k);
  });
  block_exclusive_scan<kSelThreads>(keep_sh, rows * kSelWaves, tot_sh);
  for_each_row([&](int i, unsigned key) {
    const bool keep = kept(i, key);
    const unsigned long long v_k = __ballot(keep);
    if (keep) idx[keep_sh[i * kSelWaves + wave] + rank_in_wave(v_k)] = i * kSelThreads + tid;
  });
}

// ---- selection of a long stream by several workgroups ------------------------
// With few streams of many candidates one workgroup per stream leaves most of the
// chip idle.  Here workgroup (chunk, stream) owns kSplitChunk candidates and the
// steps of prefill_select become launches, the kernel boundaries standing in for
// its barriers: split_keys (pooled keys, histogram of the top byte), three times
// split_hist (next byte, among the keys that match the bins picked so far; every
// workgroup re-derives those bins from the stream's histograms), split_count
// (threshold; keys above it and equal to it per chunk), split_write (ranks from
// the chunk counts, then the ordered walk inside the chunk).  All counters are
// integers added with atomics: the result does not depend on the order.
struct SplitCtx {
  int ul, c, t, tc, kc, first, n;     // stream, chunk, row stride, candidates, kept, first candidate and count of the chunk
  int64_t u;
  unsigned* st;                       // the stream's state words
};

__device__ __forceinline__ SplitCtx split_ctx(const GatherParams& P) {
  SplitCtx x;
  x.ul = blockIdx.y;
  x.c = blockIdx.x;
  x.u = static_cast<int64_t>(P.stream0) + x.ul;
  x.t = P.t;
  x.tc = P.pairs[x.ul / P.n_kv_heads].t - P.ows;
  x.kc = P.pairs[x.ul / P.n_kv_heads].k - P.ows;
  x.first = x.c * kSplitChunk;
  x.n = min(kSplitChunk, x.tc - x.first);
  x.st = P.split + x.u * kSplitWords;
  return x;
}

__device__ __forceinline__ bool split_idle(const SplitCtx& x) {   // nothing to select, or no candidates here
  return x.kc >= x.tc || x.kc <= 0 || x.n <= 0;
}

// Adds the chunk's keys that match (mask, prefix) to the stream's histogram of digit `pass`.
// The top digits of attention masses take few values, and one LDS atomic per key
// would serialise on those bins: per key row a wave first counts, with two votes,
// the lanes that share the bin of its first and of its next unserved lane (one
// atomic each); whoever is left adds for itself.
__device__ __forceinline__ void split_add_hist(const SplitCtx& x, const unsigned (&kreg)[kSplitKeys], int pass,
                                               unsigned prefix, unsigned mask, unsigned* hist_sh) {
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int shift = 24 - 8 * pass;
  if (tid < 256) hist_sh[tid] = 0;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < kSplitKeys; ++i) {
    bool todo = i * kSelThreads + tid < x.n && (kreg[i] & mask) == prefix;
    const unsigned bin = (kreg[i] >> shift) & 255u;
#pragma unroll
    for (int round = 0; round < 2; ++round) {
      const unsigned long long v_todo = __ballot(todo);
      if (v_todo == 0) break;
      const int leader = __ffsll(static_cast<long long>(v_todo)) - 1;
      const unsigned lead_bin = __shfl(bin, leader);
      const bool same = todo && bin == lead_bin;
      const unsigned long long v_same = __ballot(same);
      if (lane == leader) atomicAdd(&hist_sh[lead_bin], static_cast<unsigned>(__popcll(v_same)));
      todo = todo && !same;
    }
    if (todo) atomicAdd(&hist_sh[bin], 1u);
  }
  __syncthreads();
  if (tid < 256 && hist_sh[tid] != 0) atomicAdd(&x.st[pass * 256 + tid], hist_sh[tid]);
}

// The bins of digits 0 .. passes-1 from the stream's histograms.
__device__ __forceinline__ void split_prefix(const SplitCtx& x, int passes, RadixShared& sh, unsigned& prefix,
                                             unsigned& mask, unsigned& need) {
  prefix = 0; mask = 0;
  need = static_cast<unsigned>(x.kc);
  for (int p = 0; p < passes; ++p) {
    unsigned bin;
    radix_pick_bin(x.st + p * 256, need, sh, bin, need);
    prefix |= bin << (24 - 8 * p);
    mask |= 255u << (24 - 8 * p);
  }
}

__device__ __forceinline__ void split_load_keys(const GatherParams& P, const SplitCtx& x,
                                                unsigned (&kreg)[kSplitKeys]) {
  const uint32_t* keys = P.keys + x.u * x.t;
#pragma unroll
  for (int i = 0; i < kSplitKeys; ++i) {
    const int jl = i * kSelThreads + threadIdx.x;
    kreg[i] = jl < x.n ? keys[x.first + jl] : 0u;
  }
}

__global__ __launch_bounds__(kSelThreads) void split_keys(const GatherParams P) {
  __shared__ unsigned hist_sh[256];
  __shared__ float wpad_sh[kSplitChunk + 64];
  const SplitCtx x = split_ctx(P);
  if (split_idle(x)) return;
  const int tid = threadIdx.x;
  const float* w = P.w + x.u * x.t;
  const int half = P.pool >> 1;               // pool <= 63 on this path (checked on the host)
  // candidates first - half .. first + n + half, zeros outside the candidate vector
  for (int i = tid; i < x.n + 2 * half; i += kSelThreads) {
    const int cnd = x.first - half + i;
    wpad_sh[i] = (cnd >= 0 && cnd < x.tc) ? w[cnd] : 0.0f;
  }
  __syncthreads();
  unsigned kreg[kSplitKeys];
  uint32_t* keys = P.keys + x.u * x.t;
#pragma unroll
  for (int i = 0; i < kSplitKeys; ++i) {
    const int jl = i * kSelThreads + tid;
    unsigned key = 0u;
    if (jl < x.n) {
      float acc = wpad_sh[jl];                // window sum, fp32, left to right
      for (int q = 1; q < P.pool; ++q) acc = acc + wpad_sh[jl + q];
      key = __float_as_uint(acc);
      keys[x.first + jl] = key;
    }
    kreg[i] = key;
  }
  split_add_hist(x, kreg, 0, 0u, 0u, hist_sh);
}

__global__ __launch_bounds__(kSelThreads) void split_hist(const GatherParams P, int pass) {
  __shared__ unsigned hist_sh[256];
  __shared__ RadixShared radix_sh;
  const SplitCtx x = split_ctx(P);
  if (split_idle(x)) return;
  unsigned kreg[kSplitKeys];
  split_load_keys(P, x, kreg);
  unsigned prefix, mask, need;
  split_prefix(x, pass, radix_sh, prefix, mask, need);
  split_add_hist(x, kreg, pass, prefix, mask, hist_sh);
}

__global__ __launch_bounds__(kSelThreads) void split_count(const GatherParams P) {
  __shared__ RadixShared radix_sh;
  __shared__ unsigned cnt_sh[2];
  const SplitCtx x = split_ctx(P);
  if (split_idle(x)) return;
  const int tid = threadIdx.x;
  if (tid < 2) cnt_sh[tid] = 0u;
  unsigned kreg[kSplitKeys];
  split_load_keys(P, x, kreg);
  unsigned thr, mask, need;
  split_prefix(x, 4, radix_sh, thr, mask, need);      // has barriers: cnt_sh is zero for everyone
  unsigned gt = 0, eq = 0;
#pragma unroll
  for (int i = 0; i < kSplitKeys; ++i)
    if (i * kSelThreads + tid < x.n) {
      gt += kreg[i] > thr;
      eq += kreg[i] == thr;
    }
  if (gt) atomicAdd(&cnt_sh[0], gt);
  if (eq) atomicAdd(&cnt_sh[1], eq);
  __syncthreads();
  if (tid == 0) {
    x.st[4 * 256 + 2 + 2 * x.c] = cnt_sh[0];
    x.st[4 * 256 + 2 + 2 * x.c + 1] = cnt_sh[1];
    if (x.c == 0) {
      x.st[4 * 256] = thr;
      x.st[4 * 256 + 1] = need;
    }
  }
}

__global__ __launch_bounds__(kSelThreads) void split_write(const GatherParams P) {
  __shared__ int eq_sh[kSplitKeys * kSelWaves], keep_sh[kSplitKeys * kSelWaves];
  __shared__ int tot_sh[kSelWaves + 1];
  const SplitCtx x = split_ctx(P);
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  int32_t* idx = P.idx + x.u * x.t;
  if (x.c == 0)
    for (int r = tid; r < P.ows; r += kSelThreads) idx[max(x.kc, 0) + r] = x.tc + r;
  if (x.n <= 0 || x.kc <= 0) return;
  if (x.kc >= x.tc) {                               // every candidate stays
    for (int jl = tid; jl < x.n; jl += kSelThreads) idx[x.first + jl] = x.first + jl;
    return;
  }
  unsigned kreg[kSplitKeys];
  split_load_keys(P, x, kreg);
  const unsigned thr = x.st[4 * 256];
  const int need = static_cast<int>(x.st[4 * 256 + 1]);
  // Ranks at the start of this chunk, from the counts of the chunks before it.
  int eq_before = 0, keep_before = 0;
  for (int cc = 0; cc < x.c; ++cc) {
    const int gt = static_cast<int>(x.st[4 * 256 + 2 + 2 * cc]);
    const int eq = static_cast<int>(x.st[4 * 256 + 2 + 2 * cc + 1]);
    keep_before += gt + min(max(need - eq_before, 0), eq);
    eq_before += eq;
  }
  const int rows = (x.n + kSelThreads - 1) / kSelThreads;
#pragma unroll
  for (int i = 0; i < kSplitKeys; ++i)
    if (i < rows) {
      const bool is_eq = i * kSelThreads + tid < x.n && kreg[i] == thr;
      const unsigned long long v_eq = __ballot(is_eq);
      if (lane == 0) eq_sh[i * kSelWaves + wave] = __popcll(v_eq);
    }
  block_exclusive_scan<kSelThreads>(eq_sh, rows * kSelWaves, tot_sh);
  auto kept = [&](int i) -> bool {
    const bool live = i * kSelThreads + tid < x.n;
    const bool is_eq = live && kreg[i] == thr;
    const unsigned long long v_eq = __ballot(is_eq);
    const int eq_rank = eq_before + eq_sh[i * kSelWaves + wave] + rank_in_wave(v_eq);
    return live && (kreg[i] > thr || (is_eq && eq_rank < need));
  };
#pragma unroll
  for (int i = 0; i < kSplitKeys; ++i)
    if (i < rows) {
      const unsigned long long v_k = __ballot(kept(i));
      if (lane == 0) keep_sh[i * kSelWaves + wave] = __popcll(v_k);
    }
  block_exclusive_scan<kSelThreads>(keep_sh, rows * kSelWaves, tot_sh);
#pragma unroll
  for (int i = 0; i < kSplitKeys; ++i)
    if (i < rows) {
      const bool keep = kept(i);
      const unsigned long long v_k = __ballot(keep);
      if (keep)
        idx[keep_before + keep_sh[i * kSelWaves + wave] + rank_in_wave(v_k)] = x.first + i * kSelThreads + tid;
    }
}

// ---- the same selection in one launch -------------------------------------------
// When all workgroups (chunk, stream) of the selection are resident at once (the
// host checks the grid against the occupancy), the launches above become steps
// of one kernel.  The keys stay in registers throughout.  What the workgroups of
// a stream exchange lives in the stream's state words, is added to with
// agent-scope atomics and read with agent-scope loads (nothing that crosses a
// step goes through the per-XCD caches), and tells by itself when it is
// complete: the histogram of a digit is complete when its bins add up to the
// number of keys that match the digits picked so far (all candidates for the
// first digit, the count of the picked bin afterwards), and a chunk's packed
// (gt, eq) word carries a valid bit.  So a step is: add, then poll until
// complete.  The polls are bounded: a workgroup that runs out of them raises the
// stream's flag (and the call's, for xkv_fused_status); every workgroup of the
// stream that sees the flag stops, and the gather copies nothing of a flagged
// stream.  Integer atomics only: the result does not depend on the order.
struct SplitShared {
  int scan[4];
  unsigned sel_bin, sel_need, sel_cnt;
  unsigned flag;
  unsigned chunk_word[kSplitMaxChunks];
};

__device__ __forceinline__ void split_raise_flag(const SplitCtx& x, unsigned* call_flag) {
  __hip_atomic_store(x.st + kSplitFlag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __hip_atomic_store(call_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Polls the stream's histogram of digit `pass` until its bins add up to
// `expected`, then picks the bin in which the running count, from the top bin
// down, reaches `need` (as radix_pick_bin does).  Returns true, to every thread,
// if the stream was flagged or the polls ran out.
__device__ __forceinline__ bool split_poll_pick(const SplitCtx& x, int pass, unsigned expected, unsigned need,
                                                unsigned spin_limit, unsigned* call_flag, SplitShared& sh, unsigned& bin,
                                                unsigned& need_out, unsigned& cnt_out) {
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const unsigned* hist = x.st + pass * 256;
  for (unsigned spins = 0;; ++spins) {
    if (spins >= spin_limit) {
      if (tid == 0) split_raise_flag(x, call_flag);
      return true;
    }
    unsigned cnt = 0, incl = 0;
    if (tid < 256) {
      cnt = __hip_atomic_load(hist + 255 - tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      incl = cnt;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const unsigned y = __shfl_up(incl, off);
        if (lane >= off) incl += y;
      }
      if (lane == 63) sh.scan[wave] = static_cast<int>(incl);
    } else if (tid == 256) {
      sh.flag = __hip_atomic_load(x.st + kSplitFlag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    const unsigned total = static_cast<unsigned>(sh.scan[0] + sh.scan[1] + sh.scan[2] + sh.scan[3]);
    const bool flagged = sh.flag != 0u;
    if (total == expected && !flagged) {
      if (tid < 256) {
        for (int w = 0; w < wave; ++w) incl += static_cast<unsigned>(sh.scan[w]);
        const unsigned before = incl - cnt;
        if (before < need && need <= incl) {
          sh.sel_bin = 255u - static_cast<unsigned>(tid);
          sh.sel_need = need - before;
          sh.sel_cnt = cnt;
        }
      }
      __syncthreads();
      bin = sh.sel_bin;
      need_out = sh.sel_need;
      cnt_out = sh.sel_cnt;
      __syncthreads();
      return false;
    }
    if (flagged) return true;
    __syncthreads();                              // everyone has read sh before the next poll rewrites it
    __builtin_amdgcn_s_sleep(2);
  }
}

__global__ __launch_bounds__(kSelThreads) void split_fused(const GatherParams P) {
  unsigned* call_flag = P.call_flag + 1;
  __shared__ unsigned hist_sh[256];
  __shared__ SplitShared sh;
  __shared__ float wpad_sh[kSplitChunk + 64];
  __shared__ unsigned cnt_sh[2];
  __shared__ int eq_sh[kSplitKeys * kSelWaves], keep_sh[kSplitKeys * kSelWaves];
  __shared__ int tot_sh[kSelWaves + 1];

  const SplitCtx x = split_ctx(P);
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  int32_t* idx = P.idx + x.u * x.t;
  if (x.c == 0)
    for (int r = tid; r < P.ows; r += kSelThreads) idx[max(x.kc, 0) + r] = x.tc + r;
  if (x.n <= 0 || x.kc <= 0) return;              // no candidates in this chunk, or none to keep
  if (x.kc >= x.tc) {                             // every candidate stays
    for (int jl = tid; jl < x.n; jl += kSelThreads) idx[x.first + jl] = x.first + jl;
    return;
  }

  // ---- keys of this chunk, in registers ---------------------------------------------
  const float* w = P.w + x.u * x.t;
  const int half = P.pool >> 1;                   // pool <= 63 on this path (checked on the host)
  {
    // candidates first - half .. first + n + half, zeros outside the candidate vector; all requested
    // before the first is stored
    float wv[kSplitKeys + 1];
#pragma unroll
    for (int k = 0; k <= kSplitKeys; ++k) {
      const int i = k * kSelThreads + tid;
      const int cnd = x.first - half + i;
      wv[k] = (i < x.n + 2 * half && cnd >= 0 && cnd < x.tc) ? w[cnd] : 0.0f;
    }
#pragma unroll
    for (int k = 0; k <= kSplitKeys; ++k) {
      const int i = k * kSelThreads + tid;
      if (i < x.n + 2 * half) wpad_sh[i] = wv[k];
    }
  }
  __syncthreads();
  unsigned kreg[kSplitKeys];
#pragma unroll
  for (int i = 0; i < kSplitKeys; ++i) {
    const int jl = i * kSelThreads + tid;
    unsigned key = 0u;
    if (jl < x.n) {
      float acc = wpad_sh[jl];                    // window sum, fp32, left to right
      for (int q = 1; q < P.pool; ++q) acc = acc + wpad_sh[jl + q];
      key = __float_as_uint(acc);
    }
    kreg[i] = key;
  }

  // ---- four digits: add to the stream's histogram, poll until complete, pick the bin --------
  unsigned prefix = 0, mask = 0, need = static_cast<unsigned>(x.kc);
  unsigned expected = static_cast<unsigned>(x.tc);
  for (int pass = 0; pass < 4; ++pass) {
    split_add_hist(x, kreg, pass, prefix, mask, hist_sh);
    unsigned bin;
    if (split_poll_pick(x, pass, expected, need, P.spin_limit, call_flag, sh, bin, need, expected)) return;
    prefix |= bin << (24 - 8 * pass);
    mask |= 255u << (24 - 8 * pass);
  }
  const unsigned thr = prefix;

  // ---- keys above and equal to the threshold per chunk ---------------------------------
  if (tid < 2) cnt_sh[tid] = 0u;
  __syncthreads();
  unsigned gt = 0, eq = 0;
#pragma unroll
  for (int i = 0; i < kSplitKeys; ++i)
    if (i * kSelThreads + tid < x.n) {
      gt += kreg[i] > thr;
      eq += kreg[i] == thr;
    }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    gt += __shfl_xor(gt, off);
    eq += __shfl_xor(eq, off);
  }
  if (lane == 0) {
    if (gt) atomicAdd(&cnt_sh[0], gt);
    if (eq) atomicAdd(&cnt_sh[1], eq);
  }
  __syncthreads();
  if (tid == 0)                                   // both counts are at most kSplitChunk = 2^13
    __hip_atomic_store(x.st + kSplitCounts + x.c, kSplitValid | (cnt_sh[0] << 14) | cnt_sh[1], __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
  // the words of the chunks before this one
  for (unsigned spins = 0;; ++spins) {
    if (spins >= P.spin_limit) {
      if (tid == 0) split_raise_flag(x, call_flag);
      return;
    }
    unsigned word = kSplitValid;
    if (tid < x.c)
      word = __hip_atomic_load(x.st + kSplitCounts + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else if (tid == 256)
      sh.flag = __hip_atomic_load(x.st + kSplitFlag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (tid < x.c) sh.chunk_word[tid] = word;
    const int complete = __syncthreads_and((word & kSplitValid) != 0u);
    const bool flagged = sh.flag != 0u;
    if (complete && !flagged) break;
    if (flagged) return;
    __syncthreads();
    __builtin_amdgcn_s_sleep(2);
  }

  // ---- ranks at the start of this chunk, then the ordered walk inside it -----------------
  int eq_before = 0, keep_before = 0;
  for (int cc = 0; cc < x.c; ++cc) {
    const unsigned word = sh.chunk_word[cc];
    const int g = static_cast<int>((word >> 14) & 0x3fffu);
    const int e = static_cast<int>(word & 0x3fffu);
    keep_before += g + min(max(static_cast<int>(need) - eq_before, 0), e);
    eq_before += e;
  }
  const int rows = (x.n + kSelThreads - 1) / kSelThreads;
#pragma unroll
  for (int i = 0; i < kSplitKeys; ++i)
    if (i < rows) {
      const bool is_eq = i * kSelThreads + tid < x.n && kreg[i] == thr;
      const unsigned long long v_eq = __ballot(is_eq);
      if (lane == 0) eq_sh[i * kSelWaves + wave] = __popcll(v_eq);
    }
  block_exclusive_scan<kSelThreads>(eq_sh, rows * kSelWaves, tot_sh);
  auto kept = [&](int i) -> bool {
    const bool live = i * kSelThreads + tid < x.n;
    const bool is_eq = live && kreg[i] == thr;
    const unsigned long long v_eq = __ballot(is_eq);
    const int eq_rank = eq_before + eq_sh[i * kSelWaves + wave] + rank_in_wave(v_eq);
    return live && (kreg[i] > thr || (is_eq && eq_rank < static_cast<int>(need)));
  };
#pragma unroll
  for (int i = 0; i < kSplitKeys; ++i)
    if (i < rows) {
      const unsigned long long v_k = __ballot(kept(i));
      if (lane == 0) keep_sh[i * kSelWaves + wave] = __popcll(v_k);
    }
  block_exclusive_scan<kSelThreads>(keep_sh, rows * kSelWaves, tot_sh);
#pragma unroll
  for (int i = 0; i < kSplitKeys; ++i)
    if (i < rows) {
      const bool keep = kept(i);
      const unsigned long long v_k = __ballot(keep);
      if (keep)
        idx[keep_before + keep_sh[i * kSelWaves + wave] + rank_in_wave(v_k)] = x.first + i * kSelThreads + tid;
    }
}

// EvictByIndex as a gather: workgroup (chunk, stream) copies kept tokens
// [256 chunk, 256 chunk + 256) of the stream; a wave moves four rows of up to
// 256 bytes per instruction.
__global__ __launch_bounds__(kThreads) void prefill_gather(const GatherParams P) {
  const int tid = threadIdx.x;
  const int ul = blockIdx.y;
  const int pl = ul / P.n_kv_heads;
  const int h = ul - pl * P.n_kv_heads;
  const GatherPair pd = P.pairs[pl];
  const int first = blockIdx.x * kThreads;
  if (first >= pd.k) return;
  const int64_t u = static_cast<int64_t>(P.stream0) + ul;
  const int t = P.t;
  // A selection that gave up a wait leaves no trustworthy index list: nothing of that stream is copied.
  if (P.check_flag &&
      __hip_atomic_load(P.split + u * kSplitWords + kSplitFlag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u)
    return;
  const int32_t* idx = P.idx + u * t;
  const int64_t stream_slot = pd.slot0 + static_cast<int64_t>(h) * pd.cap;
  const int last = min(pd.k, first + kThreads);

  const int sdst = first + tid;
  if (sdst < last) {
    const int src = idx[sdst];
    P.score[stream_slot + sdst] = P.w[u * t + src];
    P.pos[stream_slot + sdst] = src;
  }
  const int frags = P.row_bytes >> 4;               // 16-byte pieces per row: 8, 16 or 32
  const int rows_per_pass = kThreads / frags;
  const int fr = tid % frags;
  const char* ks = static_cast<const char*>(P.k_src) + u * t * P.row_bytes;
  const char* vs = static_cast<const char*>(P.v_src) + u * t * P.row_bytes;
  char* kd = static_cast<char*>(P.k) + stream_slot * P.row_bytes;
  char* vd = static_cast<char*>(P.v) + stream_slot * P.row_bytes;
  // kPasses passes at a time: their loads are all requested before the first store.
  constexpr int kPasses = 8;
  for (int s0 = first + tid / frags; s0 < last; s0 += kPasses * rows_per_pass) {
    uint4 a[kPasses], b[kPasses];
#pragma unroll
    for (int p = 0; p < kPasses; ++p) {
      const int s = min(s0 + p * rows_per_pass, last - 1);      // past the end: a kept row again, not stored
      const int64_t so = static_cast<int64_t>(idx[s]) * P.row_bytes + fr * 16;
      a[p] = load_stream16(ks + so);
      b[p] = load_stream16(vs + so);
    }
#pragma unroll
    for (int p = 0; p < kPasses; ++p) {
      const int s = s0 + p * rows_per_pass;
      if (s < last) {
        const int64_t dof = static_cast<int64_t>(s) * P.row_bytes + fr * 16;
        store_nt16(kd + dof, a[p]);
        store_nt16(vd + dof, b[p]);
      }
    }
  }
}

// Attention score distribution vector of a (layer, sequence): the streams' masses
// added over the KV heads in index order, then the window sum over the
// candidates (fp32, left to right, zeros outside).
__global__ __launch_bounds__(kThreads) void heads_pool(const WindowParams P, float* out, int pool) {
  const int pair = blockIdx.y;
  const int t = P.t, n_kv_heads = P.n_kv_heads;
  const int tc = P.t_seq[pair % P.n_seq] - P.ows;     // this sequence's candidates
  const int j = blockIdx.x * kThreads + threadIdx.x;
  if (j >= tc) return;
  const float* wp = P.w + static_cast<int64_t>(pair) * n_kv_heads * t;
  const int half = pool >> 1;
  float acc = 0.0f;
  for (int q = 0; q < pool; ++q) {
    const int c = j - half + q;
    float hs = 0.0f;
    if (c >= 0 && c < tc) {
      hs = wp[c];
      for (int h = 1; h < n_kv_heads; ++h) hs = hs + wp[static_cast<int64_t>(h) * t + c];
    }
    acc = q == 0 ? hs : acc + hs;
  }
  out[static_cast<int64_t>(pair) * (t - P.ows) + j] = acc;
}

using WindowFn = void (*)(const WindowParams);

template <typename T, int D>
bool pick_window_nb(int nb, WindowFn* stats, WindowFn* mass) {
  switch (nb) {
    case 1: *stats = window_pass<T, D, 1, 0>; *mass = window_pass<T, D, 1, 1>; return true;
    case 2: *stats = window_pass<T, D, 2, 0>; *mass = window_pass<T, D, 2, 1>; return true;
    case 3: *stats = window_pass<T, D, 3, 0>; *mass = window_pass<T, D, 3, 1>; return true;
    case 4: *stats = window_pass<T, D, 4, 0>; *mass = window_pass<T, D, 4, 1>; return true;
    default: return false;
  }
}

bool pick_window(int dtype, int head_dim, int nb, WindowFn* stats, WindowFn* mass) {
  if (dtype == XKV_F32 && head_dim == 64) return pick_window_nb<F32, 64>(nb, stats, mass);
  if (dtype == XKV_F32 && head_dim == 128) return pick_window_nb<F32, 128>(nb, stats, mass);
  if (dtype == XKV_BF16 && head_dim == 64) return pick_window_nb<BF16, 64>(nb, stats, mass);
  if (dtype == XKV_BF16 && head_dim == 128) return pick_window_nb<BF16, 128>(nb, stats, mass);
  return false;
}

// Largest grid of split_fused: one workgroup per compute unit (0 if the kernel does
// not fit a compute unit, or on an error).  The occupancy query allows two per unit,
// but measured launches of more than one per unit run in rounds of that many
// (54 us for 512 workgroups against 26 us for 128 to 256), and then one workgroup per
// stream (prefill_select) or the launch-per-step split are as fast or faster.
int split_fused_capacity() {
  static int cap = -1;
  if (cap < 0) {
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess &&
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(split_fused), kSelThreads, 0) ==
            hipSuccess)
      cap = per_cu >= 1 ? cus : 0;
    else
      cap = 0;
    (void)hipGetLastError();
  }
  return cap;
}

// Workspace layout for `streams` streams of t tokens; every part starts on a
// 256-byte boundary.  Returns the total; the offsets are in bytes.
struct PrefillLayout { size_t stats, fin, w, keys, idx, split, flag, dlog, tref, total; };

size_t round256(size_t b) { return (b + 255) / 256 * 256; }

int prefill_strip_rows(int64_t streams, int t) {
  int rows = 1024;
  while (rows > 64 && streams * ceil_div(t, rows) < 2048) rows >>= 1;
  return rows;
}

// Whether the window masses of a call come from one K pass with stored logit
// distances (bf16 keys, at most 16 query rows per KV head), and how many query
// rows are stored per token then.
bool one_pass_window(int dtype, int nb) { return dtype == XKV_BF16 && nb == 1; }
int stored_query_rows(int nq) { return nq <= 8 ? 8 : 16; }
int round32(int t) { return (t + 31) / 32 * 32; }

PrefillLayout prefill_layout(int64_t streams, int t, int nq_pad, bool own_w, bool pooled, int nqs) {
  // The strip length depends on the call; 64 rows is the shortest, so this bounds the statistics.
  PrefillLayout L;
  const int64_t max_strips = ceil_div(t, prefill_strip_rows(streams, t));
  size_t off = 0;
  L.stats = off; off += round256(static_cast<size_t>(streams) * max_strips * nq_pad * 2 * sizeof(float));
  L.fin = off;   off += round256(static_cast<size_t>(streams) * nq_pad * 2 * sizeof(float));
  L.w = off;     off += own_w ? round256(static_cast<size_t>(streams) * t * sizeof(float)) : 0;
  L.keys = off;  off += pooled ? round256(static_cast<size_t>(streams) * t * sizeof(uint32_t)) : 0;
  L.idx = off;   off += round256(static_cast<size_t>(streams) * t * sizeof(int32_t));
  L.split = off; off += round256(static_cast<size_t>(streams) * kSplitWords * sizeof(unsigned));
  L.flag = off;  off += 256;
  // one-pass variant (nqs > 0): 16-bit distances per (token, stored query row), a reference per tile
  L.dlog = off;  off += nqs > 0 ? round256(static_cast<size_t>(streams) * round32(t) * nqs * 2) : 0;
  L.tref = off;  off += nqs > 0 ? round256(static_cast<size_t>(streams) * (round32(t) / 32) * nqs * sizeof(float)) : 0;
  L.total = off;
  return L;
}

// Fills the per-sequence prompt lengths of a launch (one entry meaning "all t").
xkv_status fill_seq_lens(const xkv_cache* cache, int32_t t, int32_t ows, const int32_t* t_per_seq,
                         WindowParams* W) {
  if (t_per_seq == nullptr) {
    W->n_seq = 1;
    W->t_seq[0] = t;
    return XKV_OK;
  }
  if (cache->batch > kMaxSeqLens) return XKV_ERR_UNSUPPORTED;
  W->n_seq = cache->batch;
  for (int b = 0; b < cache->batch; ++b) {
    if (t_per_seq[b] < ows || t_per_seq[b] > t) return XKV_ERR_INVALID_ARG;
    W->t_seq[b] = t_per_seq[b];
  }
  return XKV_OK;
}

xkv_status check_prefill_shape(const xkv_cache* cache, int32_t t, int32_t ows, int* nb_out) {
  if (t < 1 || ows < 1 || ows > t) return XKV_ERR_INVALID_ARG;
  if (t - ows > kMaxWalkRows * kSelThreads) return XKV_ERR_UNSUPPORTED;
  const int nq = ows * (cache->n_q_heads / cache->n_kv_heads);
  if (nq > kMaxNq) return XKV_ERR_UNSUPPORTED;
  *nb_out = (nq + 15) / 16;
  return XKV_OK;
}

// The three launches that turn (q_win, k_src) into the per-stream masses w.
// W arrives with its sequence lengths filled in and leaves complete.  nqs > 0
// selects the one-pass variant with that many stored query rows per token.
xkv_status launch_window_mass(const xkv_cache* cache, int64_t streams, const void* q_win,
                              const void* k_src, int32_t t, int32_t ows, int nb, float softmax_scale,
                              WindowFn stats_fn, WindowFn mass_fn, char* ws, const PrefillLayout& L, float* w,
                              int nqs, bool selection_follows, const float* lse_win, hipStream_t stream,
                              WindowParams& W) {
  const int D = cache->head_dim;
  const int strip_rows = prefill_strip_rows(streams, t);
  const int64_t nstrips = ceil_div(t, strip_rows);
  if (streams * nstrips > std::numeric_limits<int32_t>::max()) return XKV_ERR_UNSUPPORTED;
  W.q_win = q_win;
  W.k_src = k_src;
  W.lse = lse_win;
  W.stats = reinterpret_cast<float*>(ws + L.stats);
  W.fin = reinterpret_cast<float*>(ws + L.fin);
  W.w = w;
  W.dlog = reinterpret_cast<unsigned short*>(ws + L.dlog);
  W.tref = reinterpret_cast<float*>(ws + L.tref);
  W.split = selection_follows ? reinterpret_cast<unsigned*>(ws + L.split) : nullptr;
  W.call_flag = reinterpret_cast<unsigned*>(ws + L.flag);
  const float scale = softmax_scale > 0.0f ? softmax_scale : 1.0f / std::sqrt(static_cast<float>(D));
  W.scale_log2e = scale * 1.44269504088896340736f;
  W.t = t; W.ows = ows;
  W.t_pad = round32(t);
  W.group = cache->n_q_heads / cache->n_kv_heads;
  W.n_kv_heads = cache->n_kv_heads;
  W.strip_rows = strip_rows;
  W.nstrips = static_cast<int32_t>(nstrips);
  W.nq_pad = nb * 16;
  const unsigned grid = static_cast<unsigned>(streams * nstrips);
  if (nqs > 0) {
    stats_fn = D == 128 ? (nqs == 8 ? window_stats_store<128, 8> : window_stats_store<128, 16>)
                        : (nqs == 8 ? window_stats_store<64, 8> : window_stats_store<64, 16>);
    mass_fn = nqs == 8 ? window_mass_stored<8> : window_mass_stored<16>;
  }
  if (lse_win != nullptr) {
    // The rows' normalisers are given: no statistics pass and no merge, K is read once.
    const int tok = profile_begin(2, stream);
    hipLaunchKernelGGL(mass_fn, dim3(grid), dim3(kThreads), 0, stream, W);
    profile_end(tok, stream);
    return hipGetLastError() == hipSuccess ? XKV_OK : XKV_ERR_DEVICE;
  }
  const int tok = profile_begin(2, stream);
  hipLaunchKernelGGL(stats_fn, dim3(grid), dim3(kThreads), 0, stream, W);
  profile_end(tok, stream);
  if (hipGetLastError() != hipSuccess) return XKV_ERR_DEVICE;
  hipLaunchKernelGGL(window_merge, dim3(static_cast<unsigned>(streams)), dim3(kThreads), 0, stream, W);
  if (hipGetLastError() != hipSuccess) return XKV_ERR_DEVICE;
  if (nqs > 0)
    hipLaunchKernelGGL(mass_fn, dim3(static_cast<unsigned>(ceil_div(t, kThreads)), static_cast<unsigned>(streams)),
                       dim3(kThreads), 0, stream, W);
  else
    hipLaunchKernelGGL(mass_fn, dim3(grid), dim3(kThreads), 0, stream, W);
  if (hipGetLastError() != hipSuccess) return XKV_ERR_DEVICE;
  return XKV_OK;
}

xkv_status window_importance_impl(const xkv_cache* cache, int32_t layer_begin, int32_t layer_end,
                                  const void* q_win, const void* k_src, int32_t t, const int32_t* t_per_seq,
                                  int32_t ows, int32_t pool_size, float softmax_scale, const float* lse_win,
                                  float* w_out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  xkv_status st = check_cache(cache);
  if (st != XKV_OK) return st;
  st = check_layers(cache, layer_begin, layer_end);
  if (st != XKV_OK) return st;
  if (q_win == nullptr || k_src == nullptr || w_out == nullptr) return XKV_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(q_win) & 15u) || (reinterpret_cast<uintptr_t>(k_src) & 15u) ||
      (reinterpret_cast<uintptr_t>(w_out) & 3u))
    return XKV_ERR_INVALID_ARG;
  if (pool_size < 1 || (pool_size & 1) == 0) return XKV_ERR_INVALID_ARG;
  if (!(softmax_scale >= 0.0f) || std::isinf(softmax_scale)) return XKV_ERR_INVALID_ARG;
  int nb = 0;
  st = check_prefill_shape(cache, t, ows, &nb);
  if (st != XKV_OK) return st;
  WindowParams W;
  st = fill_seq_lens(cache, t, ows, t_per_seq, &W);
  if (st != XKV_OK) return st;
  const int64_t n_pairs = static_cast<int64_t>(layer_end - layer_begin) * cache->batch;
  const int64_t streams = n_pairs * cache->n_kv_heads;
  WindowFn stats_fn = nullptr, mass_fn = nullptr;
  if (!pick_window(cache->dtype, cache->head_dim, nb, &stats_fn, &mass_fn)) return XKV_ERR_UNSUPPORTED;
  const int nqs = lse_win == nullptr && one_pass_window(cache->dtype, nb)
                      ? stored_query_rows(ows * (cache->n_q_heads / cache->n_kv_heads)) : 0;
  const PrefillLayout L = prefill_layout(streams, t, nb * 16, true, false, nqs);
  if (workspace == nullptr || L.total > workspace_bytes) return XKV_ERR_CAPACITY;
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return XKV_ERR_INVALID_ARG;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  char* ws = static_cast<char*>(workspace);
  float* w_dense = reinterpret_cast<float*>(ws + L.w);
  st = launch_window_mass(cache, streams, q_win, k_src, t, ows, nb, softmax_scale, stats_fn, mass_fn, ws, L,
                          w_dense, nqs, false, lse_win, stream, W);
  if (st != XKV_OK) return st;
  const int tc = t - ows;
  if (tc > 0) {
    hipLaunchKernelGGL(heads_pool, dim3(static_cast<unsigned>(ceil_div(tc, kThreads)), static_cast<unsigned>(n_pairs)),
                       dim3(kThreads), 0, stream, W, w_out, pool_size);
    if (hipGetLastError() != hipSuccess) return XKV_ERR_DEVICE;
  }
  return XKV_OK;
}

xkv_status prefill_evict_impl(xkv_cache* cache, int32_t layer_begin, int32_t layer_end, const void* q_win,
                              const void* k_src, const void* v_src, int32_t t, const int32_t* t_per_seq,
                              int32_t ows, int32_t pool_size, const int32_t* budgets, float softmax_scale,
                              const float* lse_win, float* w_out, void* workspace, size_t workspace_bytes,
                              void* hip_stream) {
  xkv_status st = check_cache(cache);
  if (st != XKV_OK) return st;
  st = check_layers(cache, layer_begin, layer_end);
  if (st != XKV_OK) return st;
  if (q_win == nullptr || k_src == nullptr || v_src == nullptr || budgets == nullptr)
    return XKV_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(q_win) & 15u) || (reinterpret_cast<uintptr_t>(k_src) & 15u) ||
      (reinterpret_cast<uintptr_t>(v_src) & 15u) || (reinterpret_cast<uintptr_t>(w_out) & 3u))
    return XKV_ERR_INVALID_ARG;
  if (pool_size < 1 || (pool_size & 1) == 0) return XKV_ERR_INVALID_ARG;
  if (!(softmax_scale >= 0.0f) || std::isinf(softmax_scale)) return XKV_ERR_INVALID_ARG;
  int nb = 0;
  st = check_prefill_shape(cache, t, ows, &nb);
  if (st != XKV_OK) return st;

  const int B = cache->batch, hkv = cache->n_kv_heads, D = cache->head_dim;
  const int64_t first = static_cast<int64_t>(layer_begin) * B;
  const int64_t n_pairs = static_cast<int64_t>(layer_end - layer_begin) * B;
  const int64_t streams = n_pairs * hkv;
  WindowParams W;
  st = fill_seq_lens(cache, t, ows, t_per_seq, &W);
  if (st != XKV_OK) return st;
  auto seq_len = [&](int64_t pair) { return W.t_seq[pair % W.n_seq]; };   // pairs are [layer][sequence]
  for (int64_t i = 0; i < n_pairs; ++i) {
    if (budgets[i] < ows) return XKV_ERR_INVALID_ARG;
    if (std::min<int64_t>(budgets[i], seq_len(i)) > cache->cap[first + i]) return XKV_ERR_CAPACITY;
  }
  WindowFn stats_fn = nullptr, mass_fn = nullptr;
  if (!pick_window(cache->dtype, D, nb, &stats_fn, &mass_fn)) return XKV_ERR_UNSUPPORTED;
  if (streams * ceil_div(t, prefill_strip_rows(streams, t)) > std::numeric_limits<int32_t>::max())
    return XKV_ERR_UNSUPPORTED;
  const bool pooled = pool_size > 1;
  // Few long streams: the selection of a stream is split over several workgroups.
  const bool use_split = streams < 256 && t - ows >= 4 * kSplitChunk && pool_size <= 63;
  const int nqs = lse_win == nullptr && one_pass_window(cache->dtype, nb)
                      ? stored_query_rows(ows * (cache->n_q_heads / hkv)) : 0;
  const PrefillLayout L = prefill_layout(streams, t, nb * 16, w_out == nullptr, pooled || use_split, nqs);
  if (workspace == nullptr || L.total > workspace_bytes) return XKV_ERR_CAPACITY;
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return XKV_ERR_INVALID_ARG;

  // The selection kernel of the call and its dynamic LDS (the staged candidate
  // vector of the pooled, register-key variants), settled before anything is
  // enqueued: if the device refuses that much LDS the variant that keeps its keys
  // in the workspace takes over.
  const int tc_all = t - ows;
  void (*select_fn)(const GatherParams) =
      tc_all <= 8 * kSelThreads ? prefill_select<8>
      : tc_all <= kMaxKeyRegs * kSelThreads ? prefill_select<kMaxKeyRegs> : prefill_select<0>;
  size_t select_lds = 0;
  if (!use_split && pooled && tc_all <= kMaxKeyRegs * kSelThreads) {
    select_lds = static_cast<size_t>(tc_all + pool_size) * sizeof(float);
    if (select_lds > 48 * 1024 &&
        hipFuncSetAttribute(reinterpret_cast<const void*>(select_fn), hipFuncAttributeMaxDynamicSharedMemorySize,
                            static_cast<int>(select_lds)) != hipSuccess) {
      (void)hipGetLastError();
      select_fn = prefill_select<0>;
      select_lds = 0;
    }
  }

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  char* ws = static_cast<char*>(workspace);
  float* w_dense = w_out != nullptr ? w_out : reinterpret_cast<float*>(ws + L.w);
  st = launch_window_mass(cache, streams, q_win, k_src, t, ows, nb, softmax_scale, stats_fn, mass_fn, ws, L,
                          w_dense, nqs, true, lse_win, stream, W);
  if (st != XKV_OK) return st;

  GatherParams Gp;
  Gp.k_src = k_src; Gp.v_src = v_src;
  Gp.k = cache->k; Gp.v = cache->v; Gp.score = cache->score; Gp.pos = cache->pos;
  Gp.w = w_dense;
  Gp.keys = reinterpret_cast<uint32_t*>(ws + L.keys);
  Gp.idx = reinterpret_cast<int32_t*>(ws + L.idx);
  Gp.split = reinterpret_cast<unsigned*>(ws + L.split);
  Gp.call_flag = reinterpret_cast<unsigned*>(ws + L.flag);
  Gp.check_flag = 0;
  Gp.spin_limit = std::min<uint32_t>(fused_spin_limit(), kSplitSpinLimit);
  // The selection as one launch of (chunk, stream) workgroups with waits between its steps,
  // whenever a stream has at least two chunks and the grid is at most one workgroup per compute unit.
  const int64_t sel_chunks = ceil_div(t - ows, kSplitChunk);
  const bool fused_sel_possible = pool_size <= 63 && sel_chunks >= 2 && sel_chunks <= kSplitMaxChunks;
  bool any_fused_sel = false;
  note_waiting_launch(nullptr, stream);           // xkv_fused_status speaks of this call from here on
  Gp.t = t; Gp.ows = ows; Gp.pool = pool_size; Gp.n_kv_heads = hkv;
  Gp.row_bytes = D * (cache->dtype == XKV_F32 ? 4 : 2);
  for (int64_t g0 = 0; g0 < n_pairs; g0 += kMaxPairs) {
    const int np = static_cast<int>(std::min<int64_t>(kMaxPairs, n_pairs - g0));
    int64_t kmax = 0;
    for (int i = 0; i < np; ++i) {
      const int64_t idx = first + g0 + i;
      GatherPair& pd = Gp.pairs[i];
      pd.slot0 = cache->region_off[idx];
      pd.cap = cache->cap[idx];
      pd.t = seq_len(g0 + i);
      pd.k = static_cast<int32_t>(std::min<int64_t>(budgets[g0 + i], pd.t));
      kmax = std::max<int64_t>(kmax, pd.k);
    }
    Gp.stream0 = static_cast<int32_t>(g0 * hkv);
    const int tc = t - ows;
    const unsigned n_streams = static_cast<unsigned>(np * hkv);
    Gp.check_flag = 0;
    if (fused_sel_possible && sel_chunks * n_streams <= split_fused_capacity()) {
      const dim3 grid(static_cast<unsigned>(sel_chunks), n_streams);
      hipLaunchKernelGGL(split_fused, grid, dim3(kSelThreads), 0, stream, Gp);
      if (hipGetLastError() != hipSuccess) return XKV_ERR_DEVICE;
      Gp.check_flag = 1;
      any_fused_sel = true;
    } else if (use_split) {
      const dim3 grid(static_cast<unsigned>(ceil_div(tc, kSplitChunk)), n_streams);
      hipLaunchKernelGGL(split_keys, grid, dim3(kSelThreads), 0, stream, Gp);
      for (int pass = 1; pass < 4; ++pass)
        hipLaunchKernelGGL(split_hist, grid, dim3(kSelThreads), 0, stream, Gp, pass);
      hipLaunchKernelGGL(split_count, grid, dim3(kSelThreads), 0, stream, Gp);
      hipLaunchKernelGGL(split_write, grid, dim3(kSelThreads), 0, stream, Gp);
      if (hipGetLastError() != hipSuccess) return XKV_ERR_DEVICE;
    } else {
      hipLaunchKernelGGL(select_fn, dim3(n_streams), dim3(kSelThreads), select_lds, stream, Gp);
      if (hipGetLastError() != hipSuccess) return XKV_ERR_DEVICE;
    }
    hipLaunchKernelGGL(prefill_gather,
                       dim3(static_cast<unsigned>(ceil_div(kmax, kThreads)), static_cast<unsigned>(np * hkv)),
                       dim3(kThreads), 0, stream, Gp);
    if (hipGetLastError() != hipSuccess) return XKV_ERR_DEVICE;
  }
  if (any_fused_sel) note_waiting_launch(Gp.call_flag, stream);
  for (int64_t i = 0; i < n_pairs; ++i)
    cache->len[first + i] = static_cast<int32_t>(std::min<int64_t>(budgets[i], seq_len(i)));
  return XKV_OK;
}

}  // namespace
}  // namespace xkv

extern "C" xkv_status xkv_prefill_workspace_bytes(const xkv_cache* cache, int32_t max_layers_per_call,
                                                  int32_t t, int32_t ows, size_t* bytes_out) {
  using namespace xkv;
  xkv_status st = check_cache(cache);
  if (st != XKV_OK) return st;
  if (bytes_out == nullptr || max_layers_per_call <= 0) return XKV_ERR_INVALID_ARG;
  int nb = 0;
  st = check_prefill_shape(cache, t, ows, &nb);
  if (st != XKV_OK) return st;
  const int64_t layers = std::min<int64_t>(max_layers_per_call, cache->n_layers);
  // A call on fewer layers has fewer streams and may pick shorter strips: take
  // the largest need over the possible layer counts' strip lengths.
  size_t worst = 0;
  for (int64_t l = 1; l <= layers; ++l) {
    const int64_t streams = l * cache->batch * cache->n_kv_heads;
    worst = std::max(worst, prefill_layout(streams, t, nb * 16, true, true,
                                           one_pass_window(cache->dtype, nb)
                                               ? stored_query_rows(ows * (cache->n_q_heads / cache->n_kv_heads)) : 0).total);
  }
  *bytes_out = worst;
  return XKV_OK;
}

extern "C" xkv_status xkv_window_importance(const xkv_cache* cache, int32_t layer_begin,
                                            int32_t layer_end, const void* q_win, const void* k_src,
                                            int32_t t, const int32_t* t_per_seq, int32_t ows,
                                            int32_t pool_size,
                                            float softmax_scale, float* w_out, void* workspace,
                                            size_t workspace_bytes, void* hip_stream) {
  return xkv::window_importance_impl(cache, layer_begin, layer_end, q_win, k_src, t, t_per_seq, ows, pool_size,
                                     softmax_scale, nullptr, w_out, workspace, workspace_bytes, hip_stream);
}

extern "C" xkv_status xkv_window_importance_lse(const xkv_cache* cache, int32_t layer_begin,
                                                int32_t layer_end, const void* q_win, const void* k_src,
                                                int32_t t, const int32_t* t_per_seq, int32_t ows,
                                                int32_t pool_size, float softmax_scale, const float* lse_win,
                                                float* w_out, void* workspace, size_t workspace_bytes,
                                                void* hip_stream) {
  if (lse_win == nullptr || (reinterpret_cast<uintptr_t>(lse_win) & 3u)) return XKV_ERR_INVALID_ARG;
  return xkv::window_importance_impl(cache, layer_begin, layer_end, q_win, k_src, t, t_per_seq, ows, pool_size,
                                     softmax_scale, lse_win, w_out, workspace, workspace_bytes, hip_stream);
}

extern "C" xkv_status xkv_prefill_evict(xkv_cache* cache, int32_t layer_begin, int32_t layer_end,
                                        const void* q_win, const void* k_src, const void* v_src,
                                        int32_t t, const int32_t* t_per_seq, int32_t ows,
                                        int32_t pool_size,
                                        const int32_t* budgets, float softmax_scale, float* w_out,
                                        void* workspace, size_t workspace_bytes, void* hip_stream) {
  return xkv::prefill_evict_impl(cache, layer_begin, layer_end, q_win, k_src, v_src, t, t_per_seq, ows, pool_size,
                                 budgets, softmax_scale, nullptr, w_out, workspace, workspace_bytes, hip_stream);
}

extern "C" xkv_status xkv_prefill_evict_lse(xkv_cache* cache, int32_t layer_begin, int32_t layer_end,
                                            const void* q_win, const void* k_src, const void* v_src,
                                            int32_t t, const int32_t* t_per_seq, int32_t ows,
                                            int32_t pool_size, const int32_t* budgets, float softmax_scale,
                                            const float* lse_win, float* w_out, void* workspace,
                                            size_t workspace_bytes, void* hip_stream) {
  if (lse_win == nullptr || (reinterpret_cast<uintptr_t>(lse_win) & 3u)) return XKV_ERR_INVALID_ARG;
  return xkv::prefill_evict_impl(cache, layer_begin, layer_end, q_win, k_src, v_src, t, t_per_seq, ows, pool_size,
                                 budgets, softmax_scale, lse_win, w_out, workspace, workspace_bytes, hip_stream);
}
