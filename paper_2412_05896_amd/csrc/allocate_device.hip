// xkv_allocate_budgets_device: the adaptive allocation of Alg. 1 for the
// total-size problem (Eq. 17), on score vectors that already live on the device
// (the mini-prefill's attention score distribution vectors, Sec. 4.1).
//
// The greedy of Alg. 1 takes, N times, the waiting token with the largest
// normalised contribution w / Sum(w_l) (the marginal gain of Eq. 21).  Each
// layer's contributions do not increase with rank, so what it takes is the N
// largest contributions over all layers, equal ones by lower layer.  Here the
// N-th largest is found by a radix select over the 64-bit patterns of the
// contributions (non-negative doubles order like unsigned integers): 8 passes of
// 8 bits, each a histogram kernel over all layers' values plus a one-workgroup
// kernel that picks the bin.  A counting kernel then gives every layer the
// number of its contributions above the threshold and equal to it.
//
// Floors and caps: the unconstrained counts are computed first; if they break
// bounds, the layers on the side with the larger total violation are fixed at
// their bound and the rest is solved again with what is left (the marginal
// gains being non-increasing, a layer below its floor at one threshold stays
// below it at every higher one, and likewise for caps).  At most n_layers
// rounds; each round brings n_layers counts to the host.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <vector>

#include "xkv_internal.h"

namespace xkv {
namespace {

constexpr int kThreads = 256;
constexpr int kPerThread = 32;
constexpr int kChunkElems = kThreads * kPerThread;   // values per workgroup
constexpr int kMaxLayers = 256;

struct SelectState {
  unsigned long long prefix, mask, need;   // radix select progress
  unsigned long long tau;                  // final threshold (bit pattern of a double)
  unsigned long long need_eq;              // contributions equal to tau that are taken
};

struct AllocParams {
  const float* w;            // layer l starts at w + l * stride and has len values
  long long len, stride;
  int n_layers, chunks;
  double* part_sum;          // [n_layers][chunks]
  double* layer_sum;         // [n_layers]
  unsigned* hist;            // [8][256]
  SelectState* state;
  long long* part_gt;        // [n_layers][chunks]
  long long* part_eq;        // [n_layers][chunks]
  double* part_kept;         // [n_layers][chunks] sum of contributions above tau
  long long* out_n;          // [n_layers]
  double* out_r;             // [n_layers] retained importance of the layer (fraction)
  unsigned long long free_mask[kMaxLayers / 64];   // layers that take part in this round
};

__device__ __forceinline__ bool layer_free(const AllocParams& P, int l) {
  return (P.free_mask[l >> 6] >> (l & 63)) & 1ull;
}

// Contribution of one value; a layer whose values sum to zero contributes 0 per token.
__device__ __forceinline__ unsigned long long contribution_bits(float x, double sum) {
  const double p = (sum > 0.0 && x > 0.0f) ? static_cast<double>(x) / sum : 0.0;   // also maps -0 to +0
  return static_cast<unsigned long long>(__double_as_longlong(p));
}

// Sum of a double over the workgroup, in a fixed order; valid in thread 0.
__device__ __forceinline__ double block_sum(double v, double* sh) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off);
  if ((tid & 63) == 0) sh[tid >> 6] = v;
  __syncthreads();
  double tot = 0.0;
  if (tid == 0)
    for (int wv = 0; wv < kThreads / 64; ++wv) tot += sh[wv];
  __syncthreads();
  return tot;
}

__global__ __launch_bounds__(kThreads) void alloc_partial_sums(const AllocParams P) {
  __shared__ double sh[kThreads / 64];
  const int l = blockIdx.y, c = blockIdx.x;
  const float* w = P.w + static_cast<long long>(l) * P.stride;
  const long long base = static_cast<long long>(c) * kChunkElems;
  double s = 0.0;
#pragma unroll 4
  for (int i = 0; i < kPerThread; ++i) {
    const long long j = base + static_cast<long long>(i) * kThreads + threadIdx.x;
    if (j < P.len) s += static_cast<double>(w[j]);
  }
  const double tot = block_sum(s, sh);
  if (threadIdx.x == 0) P.part_sum[l * P.chunks + c] = tot;
}

__global__ __launch_bounds__(kThreads) void alloc_layer_sums(const AllocParams P) {
  const int l = blockIdx.x * kThreads + threadIdx.x;
  if (l >= P.n_layers) return;
  double s = 0.0;
  for (int c = 0; c < P.chunks; ++c) s += P.part_sum[l * P.chunks + c];
  P.layer_sum[l] = s;
}

// Start of a round: the select looks for the `need`-th largest contribution.
__global__ void alloc_begin_round(const AllocParams P, unsigned long long need) {
  for (int i = threadIdx.x; i < 8 * 256; i += blockDim.x) P.hist[i] = 0u;
  if (threadIdx.x == 0) {
    P.state->prefix = 0ull;
    P.state->mask = 0ull;
    P.state->need = need;
  }
}

__global__ __launch_bounds__(kThreads) void alloc_histogram(const AllocParams P, int pass) {
  __shared__ unsigned hist[256];
  const int l = blockIdx.y, c = blockIdx.x;
  if (!layer_free(P, l)) return;
  const int tid = threadIdx.x;
  hist[tid] = 0u;
  __syncthreads();
  const unsigned long long prefix = P.state->prefix, mask = P.state->mask;
  const int shift = 56 - 8 * pass;
  const double sum = P.layer_sum[l];
  const float* w = P.w + static_cast<long long>(l) * P.stride;
  const long long base = static_cast<long long>(c) * kChunkElems;
  unsigned run_bin = 0, run_len = 0;
  for (int i = 0; i < kPerThread; ++i) {
    const long long j = base + static_cast<long long>(i) * kThreads + tid;
    if (j >= P.len) break;
    const unsigned long long key = contribution_bits(w[j], sum);
    if ((key & mask) == prefix) {
      const unsigned bin = static_cast<unsigned>(key >> shift) & 255u;
      if (bin != run_bin && run_len != 0) {
        atomicAdd(&hist[run_bin], run_len);
        run_len = 0;
      }
      run_bin = bin;
      ++run_len;
    }
  }
  if (run_len != 0) atomicAdd(&hist[run_bin], run_len);
  __syncthreads();
  if (hist[tid] != 0u) atomicAdd(&P.hist[pass * 256 + tid], hist[tid]);
}

// One workgroup: the bin in which the count, from the top, reaches `need`.
__global__ __launch_bounds__(kThreads) void alloc_pick_bin(const AllocParams P, int pass) {
  __shared__ unsigned long long scan_sh[kThreads / 64];
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const unsigned long long need = P.state->need;
  const unsigned long long cnt = P.hist[pass * 256 + 255 - tid];   // thread t takes bin 255 - t
  unsigned long long incl = cnt;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const unsigned long long y = __shfl_up(incl, off);
    if (lane >= off) incl += y;
  }
  if (lane == 63) scan_sh[wave] = incl;
  __syncthreads();
  for (int wv = 0; wv < wave; ++wv) incl += scan_sh[wv];
  const unsigned long long before = incl - cnt;
  __syncthreads();
  if (before < need && need <= incl) {                 // exactly one thread
    const int shift = 56 - 8 * pass;
    const unsigned long long prefix = P.state->prefix | (static_cast<unsigned long long>(255 - tid) << shift);
    P.state->prefix = prefix;
    P.state->mask = P.state->mask | (255ull << shift);
    P.state->need = need - before;
    if (pass == 7) {
      P.state->tau = prefix;
      P.state->need_eq = need - before;
    }
  }
}

__global__ __launch_bounds__(kThreads) void alloc_count(const AllocParams P) {
  __shared__ double sh[kThreads / 64];
  __shared__ long long cnt_sh[2];
  const int l = blockIdx.y, c = blockIdx.x;
  if (!layer_free(P, l)) return;
  const int tid = threadIdx.x;
  if (tid < 2) cnt_sh[tid] = 0;
  __syncthreads();
  const unsigned long long tau = P.state->tau;
  const double sum = P.layer_sum[l];
  const float* w = P.w + static_cast<long long>(l) * P.stride;
  const long long base = static_cast<long long>(c) * kChunkElems;
  int gt = 0, eq = 0;
  double kept = 0.0;
  for (int i = 0; i < kPerThread; ++i) {
    const long long j = base + static_cast<long long>(i) * kThreads + tid;
    if (j >= P.len) break;
    const unsigned long long key = contribution_bits(w[j], sum);
    if (key > tau) {
      ++gt;
      kept += __longlong_as_double(static_cast<long long>(key));
    } else if (key == tau) {
      ++eq;
    }
  }
  if (gt) atomicAdd(reinterpret_cast<unsigned long long*>(&cnt_sh[0]), static_cast<unsigned long long>(gt));
  if (eq) atomicAdd(reinterpret_cast<unsigned long long*>(&cnt_sh[1]), static_cast<unsigned long long>(eq));
  const double tot = block_sum(kept, sh);              // has the barriers the counters need
  if (tid == 0) {
    P.part_gt[l * P.chunks + c] = cnt_sh[0];
    P.part_eq[l * P.chunks + c] = cnt_sh[1];
    P.part_kept[l * P.chunks + c] = tot;
  }
}

// One thread per layer folds the chunks; thread 0 then hands the contributions
// equal to the threshold to the layers in index order.
__global__ __launch_bounds__(kThreads) void alloc_finish(const AllocParams P) {
  __shared__ long long gt_sh[kMaxLayers], eq_sh[kMaxLayers];
  __shared__ double kept_sh[kMaxLayers];
  const int l = threadIdx.x;
  if (l < P.n_layers) {
    long long gt = 0, eq = 0;
    double kept = 0.0;
    if (layer_free(P, l))
      for (int c = 0; c < P.chunks; ++c) {
        gt += P.part_gt[l * P.chunks + c];
        eq += P.part_eq[l * P.chunks + c];
        kept += P.part_kept[l * P.chunks + c];
      }
    gt_sh[l] = gt;
    eq_sh[l] = eq;
    kept_sh[l] = kept;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    long long left = static_cast<long long>(P.state->need_eq);
    const double tau = __longlong_as_double(static_cast<long long>(P.state->tau));
    for (int i = 0; i < P.n_layers; ++i) {
      if (!layer_free(P, i)) continue;
      const long long take = eq_sh[i] < left ? eq_sh[i] : left;
      left -= take;
      P.out_n[i] = gt_sh[i] + take;
      P.out_r[i] = kept_sh[i] + static_cast<double>(take) * tau;
    }
  }
}

// Retained importance of layers whose count is fixed from outside (a bound, or
// everything): the sum of the layer's n largest contributions, by a per-layer
// select on the fp32 patterns.  Used only for the R_avg report.
__global__ __launch_bounds__(kThreads) void alloc_fixed_retained(const AllocParams P, int l, long long n) {
  __shared__ unsigned hist[256];
  __shared__ unsigned long long scan_sh[kThreads / 64];
  __shared__ unsigned sel_bin;
  __shared__ unsigned long long sel_need;
  __shared__ double sh[kThreads / 64];
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const float* w = P.w + static_cast<long long>(l) * P.stride;
  const double sum = P.layer_sum[l];
  if (n <= 0 || !(sum > 0.0)) {
    if (tid == 0) P.out_r[l] = 0.0;
    return;
  }
  unsigned prefix = 0, mask = 0;
  unsigned long long need = static_cast<unsigned long long>(n);
  for (int shift = 24; shift >= 0; shift -= 8) {
    hist[tid] = 0u;
    __syncthreads();
    for (long long j = tid; j < P.len; j += kThreads) {
      const unsigned key = __float_as_uint(w[j]);
      if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
    }
    __syncthreads();
    const unsigned long long cnt = hist[255 - tid];
    unsigned long long incl = cnt;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const unsigned long long y = __shfl_up(incl, off);
      if (lane >= off) incl += y;
    }
    if (lane == 63) scan_sh[wave] = incl;
    __syncthreads();
    for (int wv = 0; wv < wave; ++wv) incl += scan_sh[wv];
    const unsigned long long before = incl - cnt;
    if (before < need && need <= incl) {
      sel_bin = 255u - static_cast<unsigned>(tid);
      sel_need = need - before;
    }
    __syncthreads();
    prefix |= sel_bin << shift;
    mask |= 255u << shift;
    need = sel_need;
    __syncthreads();
  }
  double kept = 0.0;
  for (long long j = tid; j < P.len; j += kThreads) {
    const unsigned key = __float_as_uint(w[j]);
    if (key > prefix) kept += static_cast<double>(w[j]) / sum;
  }
  const double tot = block_sum(kept, sh);
  if (tid == 0)
    P.out_r[l] = tot + static_cast<double>(need) * (static_cast<double>(__uint_as_float(prefix)) / sum);
}

size_t align256(size_t b) { return (b + 255) / 256 * 256; }

struct AllocLayout { size_t part_sum, layer_sum, hist, state, part_gt, part_eq, part_kept, out_n, out_r, total; };

AllocLayout alloc_layout(int n_layers, int chunks) {
  AllocLayout L;
  size_t off = 0;
  const size_t cells = static_cast<size_t>(n_layers) * chunks;
  L.part_sum = off;  off += align256(cells * sizeof(double));
  L.layer_sum = off; off += align256(static_cast<size_t>(n_layers) * sizeof(double));
  L.hist = off;      off += align256(8 * 256 * sizeof(unsigned));
  L.state = off;     off += align256(sizeof(SelectState));
  L.part_gt = off;   off += align256(cells * sizeof(long long));
  L.part_eq = off;   off += align256(cells * sizeof(long long));
  L.part_kept = off; off += align256(cells * sizeof(double));
  L.out_n = off;     off += align256(static_cast<size_t>(n_layers) * sizeof(long long));
  L.out_r = off;     off += align256(static_cast<size_t>(n_layers) * sizeof(double));
  L.total = off;
  return L;
}

// The total-size problem for `total_size` tokens on sums already computed:
// budgets in n, R_avg of the result in *ravg (if not null).
xkv_status solve_total(AllocParams& P, const dim3& grid, hipStream_t stream, const std::vector<int64_t>& lo,
                       const std::vector<int64_t>& hi, int64_t total_size, std::vector<int64_t>& n,
                       double* ravg_out) {
  const int32_t n_layers = P.n_layers;
  const int64_t len = P.len;
  n.assign(n_layers, 0);
  std::vector<char> is_free(n_layers, 1);
  std::vector<long long> got(n_layers);
  for (int round = 0; round <= n_layers; ++round) {
    int64_t fixed = 0, free_layers = 0;
    for (auto& m : P.free_mask) m = 0ull;
    for (int32_t l = 0; l < n_layers; ++l) {
      if (is_free[l]) {
        P.free_mask[l >> 6] |= 1ull << (l & 63);
        ++free_layers;
      } else {
        fixed += n[l];
      }
    }
    const int64_t need = total_size - fixed;
    if (free_layers == 0) break;
    if (need <= 0 || need >= free_layers * len) {
      // nothing, or everything, for the free layers: no threshold to find
      for (int32_t l = 0; l < n_layers; ++l)
        if (is_free[l]) got[l] = need <= 0 ? 0 : len;
    } else {
      hipLaunchKernelGGL(alloc_begin_round, dim3(1), dim3(kThreads), 0, stream, P,
                         static_cast<unsigned long long>(need));
      for (int pass = 0; pass < 8; ++pass) {
        hipLaunchKernelGGL(alloc_histogram, grid, dim3(kThreads), 0, stream, P, pass);
        hipLaunchKernelGGL(alloc_pick_bin, dim3(1), dim3(kThreads), 0, stream, P, pass);
      }
      hipLaunchKernelGGL(alloc_count, grid, dim3(kThreads), 0, stream, P);
      hipLaunchKernelGGL(alloc_finish, dim3(1), dim3(kThreads), 0, stream, P);
      if (hipGetLastError() != hipSuccess) return XKV_ERR_DEVICE;
      if (hipMemcpyAsync(got.data(), P.out_n, static_cast<size_t>(n_layers) * sizeof(long long),
                         hipMemcpyDeviceToHost, stream) != hipSuccess ||
          hipStreamSynchronize(stream) != hipSuccess)
        return XKV_ERR_DEVICE;
    }
    int64_t under = 0, over = 0;
    for (int32_t l = 0; l < n_layers; ++l) {
      if (!is_free[l]) continue;
      n[l] = got[l];
      if (n[l] < lo[l]) under += lo[l] - n[l];
      if (n[l] > hi[l]) over += n[l] - hi[l];
    }
    if (under == 0 && over == 0) break;
    for (int32_t l = 0; l < n_layers; ++l) {
      if (!is_free[l]) continue;
      if (under >= over && n[l] < lo[l]) { n[l] = lo[l]; is_free[l] = 0; }
      if (under < over && n[l] > hi[l]) { n[l] = hi[l]; is_free[l] = 0; }
    }
  }
  if (ravg_out != nullptr) {
    // Layers that ended a threshold round hold their retained importance in
    // out_r; the others (fixed at a bound, or taken whole) get it from a
    // per-layer select.
    bool last_round_had_threshold = false;
    {
      int64_t fixed = 0, free_layers = 0;
      for (int32_t l = 0; l < n_layers; ++l) {
        if (is_free[l]) ++free_layers; else fixed += n[l];
      }
      const int64_t need = total_size - fixed;
      last_round_had_threshold = free_layers > 0 && need > 0 && need < free_layers * len;
    }
    for (int32_t l = 0; l < n_layers; ++l)
      if (!is_free[l] || !last_round_had_threshold)
        hipLaunchKernelGGL(alloc_fixed_retained, dim3(1), dim3(kThreads), 0, stream, P, l,
                           static_cast<long long>(n[l]));
    std::vector<double> r(n_layers);
    if (hipGetLastError() != hipSuccess) return XKV_ERR_DEVICE;
    if (hipMemcpyAsync(r.data(), P.out_r, static_cast<size_t>(n_layers) * sizeof(double),
                       hipMemcpyDeviceToHost, stream) != hipSuccess ||
        hipStreamSynchronize(stream) != hipSuccess)
      return XKV_ERR_DEVICE;
    double tot = 0.0;
    for (int32_t l = 0; l < n_layers; ++l) tot += r[l];
    *ravg_out = tot / n_layers;
  }
  return XKV_OK;
}

}  // namespace
}  // namespace xkv

extern "C" xkv_status xkv_allocate_device_workspace_bytes(int32_t n_layers, int64_t len, size_t* bytes_out) {
  using namespace xkv;
  if (bytes_out == nullptr || n_layers <= 0 || len < 0) return XKV_ERR_INVALID_ARG;
  if (n_layers > kMaxLayers) return XKV_ERR_UNSUPPORTED;
  const int64_t chunks = std::max<int64_t>(1, ceil_div(len, kChunkElems));
  if (chunks > 65535) return XKV_ERR_UNSUPPORTED;
  *bytes_out = alloc_layout(n_layers, static_cast<int>(chunks)).total;
  return XKV_OK;
}

extern "C" xkv_status xkv_allocate_budgets_device(int32_t n_layers, const float* w, int64_t len,
                                                  int64_t layer_stride, int32_t mode,
                                                  int64_t total_size, double target_ravg,
                                                  const int64_t* min_budget,
                                                  const int64_t* max_budget, int64_t* budgets_out,
                                                  double* ravg_out, void* workspace,
                                                  size_t workspace_bytes, void* hip_stream) {
  using namespace xkv;
  if (n_layers <= 0 || len < 0 || layer_stride < len || budgets_out == nullptr ||
      (len > 0 && w == nullptr) || (reinterpret_cast<uintptr_t>(w) & 3u))
    return XKV_ERR_INVALID_ARG;
  if (mode != XKV_ALLOC_TOTAL_SIZE && mode != XKV_ALLOC_TARGET_RAVG) return XKV_ERR_INVALID_ARG;
  if (mode == XKV_ALLOC_TARGET_RAVG && !(target_ravg >= 0.0 && target_ravg <= 1.0)) return XKV_ERR_INVALID_ARG;
  if (n_layers > kMaxLayers) return XKV_ERR_UNSUPPORTED;
  const int64_t chunks64 = std::max<int64_t>(1, ceil_div(len, kChunkElems));
  if (chunks64 > 65535) return XKV_ERR_UNSUPPORTED;
  const int chunks = static_cast<int>(chunks64);
  std::vector<int64_t> lo(n_layers), hi(n_layers);
  int64_t sum_lo = 0, sum_hi = 0;
  for (int32_t l = 0; l < n_layers; ++l) {
    lo[l] = min_budget ? min_budget[l] : 0;
    hi[l] = max_budget ? std::min<int64_t>(max_budget[l], len) : len;
    if (lo[l] < 0 || lo[l] > hi[l]) return XKV_ERR_INFEASIBLE;
    sum_lo += lo[l];
    sum_hi += hi[l];
  }
  if (mode == XKV_ALLOC_TOTAL_SIZE && (total_size < sum_lo || total_size > sum_hi)) return XKV_ERR_INFEASIBLE;
  const AllocLayout L = alloc_layout(n_layers, chunks);
  if (workspace == nullptr || L.total > workspace_bytes) return XKV_ERR_CAPACITY;
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return XKV_ERR_INVALID_ARG;

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  char* ws = static_cast<char*>(workspace);
  AllocParams P;
  P.w = w;
  P.len = len;
  P.stride = layer_stride;
  P.n_layers = n_layers;
  P.chunks = chunks;
  P.part_sum = reinterpret_cast<double*>(ws + L.part_sum);
  P.layer_sum = reinterpret_cast<double*>(ws + L.layer_sum);
  P.hist = reinterpret_cast<unsigned*>(ws + L.hist);
  P.state = reinterpret_cast<SelectState*>(ws + L.state);
  P.part_gt = reinterpret_cast<long long*>(ws + L.part_gt);
  P.part_eq = reinterpret_cast<long long*>(ws + L.part_eq);
  P.part_kept = reinterpret_cast<double*>(ws + L.part_kept);
  P.out_n = reinterpret_cast<long long*>(ws + L.out_n);
  P.out_r = reinterpret_cast<double*>(ws + L.out_r);
  for (auto& m : P.free_mask) m = 0ull;

  const dim3 grid(static_cast<unsigned>(chunks), static_cast<unsigned>(n_layers));
  hipLaunchKernelGGL(alloc_partial_sums, grid, dim3(kThreads), 0, stream, P);
  hipLaunchKernelGGL(alloc_layer_sums, dim3((n_layers + kThreads - 1) / kThreads), dim3(kThreads), 0, stream, P);
  if (hipGetLastError() != hipSuccess) return XKV_ERR_DEVICE;

  std::vector<int64_t> n;
  xkv_status st = XKV_OK;
  if (mode == XKV_ALLOC_TOTAL_SIZE) {
    st = solve_total(P, grid, stream, lo, hi, total_size, n, ravg_out);
    if (st != XKV_OK) return st;
  } else {
    // Eq. 18: the smallest total whose R_avg reaches the target.  R_avg does not
    // decrease with the total, so the total-size solver is bisected over
    // [sum of floors, sum of caps]; if even all tokens fall short, all are taken
    // (the greedy of Alg. 1 ends the same way, with an empty wait list).
    double r = 0.0;
    int64_t a = sum_lo, b = sum_hi;
    st = solve_total(P, grid, stream, lo, hi, a, n, &r);
    if (st != XKV_OK) return st;
    if (r < target_ravg) {
      while (b - a > 1) {                       // invariant: R(a) < target, and b is the answer so far
        const int64_t mid = a + (b - a) / 2;
        st = solve_total(P, grid, stream, lo, hi, mid, n, &r);
        if (st != XKV_OK) return st;
        if (r >= target_ravg) b = mid; else a = mid;
      }
      st = solve_total(P, grid, stream, lo, hi, b, n, &r);
      if (st != XKV_OK) return st;
    }
    if (ravg_out != nullptr) *ravg_out = r;
  }
  for (int32_t l = 0; l < n_layers; ++l) budgets_out[l] = n[l];
  return XKV_OK;
}
