// Top-k threshold search shared by the selection kernels (Alg. 2 step 5, TopK):
// a radix select over fp32 bit patterns, for one workgroup per stream.
#ifndef XKV_SELECT_UTIL_H
#define XKV_SELECT_UTIL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace xkv {

constexpr int kMaxSelWaves = 16;    // the helpers serve workgroups of up to 1024 threads

struct RadixShared {
  unsigned hist[256];
  int scan[kMaxSelWaves];
  unsigned sel_bin, sel_need;
};

// Number of set bits of a wave-wide vote below this lane.
__device__ __forceinline__ int rank_in_wave(unsigned long long vote) {
  return __builtin_amdgcn_mbcnt_hi(static_cast<unsigned>(vote >> 32),
                                   __builtin_amdgcn_mbcnt_lo(static_cast<unsigned>(vote), 0));
}

// One digit of a radix select: given the 256 counts of the current digit
// (`hist`, LDS or global), finds the bin in which the running count, from the
// top bin down, reaches `need`, and how many of that bin's keys are still
// needed.  Thread t < 256 takes bin 255 - t and an inclusive scan over t locates
// the bin.  Every thread of the workgroup (at least 256 threads) must call it;
// begins and ends with a barrier.
__device__ __forceinline__ void radix_pick_bin(const unsigned* hist, unsigned need, RadixShared& sh,
                                               unsigned& bin, unsigned& need_out) {
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  __syncthreads();
  unsigned cnt = 0, incl = 0;
  if (tid < 256) {
    cnt = hist[255 - tid];
    incl = cnt;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const unsigned y = __shfl_up(incl, off);
      if (lane >= off) incl += y;
    }
    if (lane == 63) sh.scan[wave] = static_cast<int>(incl);
  }
  __syncthreads();
  if (tid < 256) {
    for (int w = 0; w < wave; ++w) incl += static_cast<unsigned>(sh.scan[w]);
    const unsigned before = incl - cnt;
    if (before < need && need <= incl) {
      sh.sel_bin = 255u - static_cast<unsigned>(tid);
      sh.sel_need = need - before;
    }
  }
  __syncthreads();
  bin = sh.sel_bin;
  need_out = sh.sel_need;
  __syncthreads();
}

// The kk-th largest of the workgroup's keys, 1 <= kk <= number of keys, compared
// as unsigned integers (for non-negative floats that is the float order): four
// passes over 8 bits each, every pass a 256-bin histogram of the keys that
// still match the prefix found so far.  `for_each_key(fn)` calls fn(key) for
// every key of the calling thread, in any fixed order; each key belongs to one
// thread.  A thread adds runs of equal bins with one atomic: the top byte of
// scores that lie within a few powers of two of each other takes few values,
// and one atomic per key would serialise on those bins.  On return `thr` is the
// kk-th largest key and `need` says how many of the keys equal to it belong to
// the top kk (the keys above it all do).  Every thread of the workgroup (at
// least 256 threads) must call it; ends with a barrier.
template <typename ForEachKey>
__device__ __forceinline__ void radix_select(ForEachKey for_each_key, int kk, RadixShared& sh,
                                             unsigned& thr, unsigned& need) {
  const int tid = threadIdx.x;
  unsigned prefix = 0, mask = 0;
  need = static_cast<unsigned>(kk);
  for (int shift = 24; shift >= 0; shift -= 8) {
    if (tid < 256) sh.hist[tid] = 0;
    __syncthreads();
    unsigned run_bin = 0, run_len = 0;
    for_each_key([&](unsigned key) {
      if ((key & mask) == prefix) {
        const unsigned bin = (key >> shift) & 255u;
        if (bin != run_bin && run_len != 0) {
          atomicAdd(&sh.hist[run_bin], run_len);
          run_len = 0;
        }
        run_bin = bin;
        ++run_len;
      }
    });
    if (run_len != 0) atomicAdd(&sh.hist[run_bin], run_len);
    __syncthreads();
    unsigned bin;
    radix_pick_bin(sh.hist, need, sh, bin, need);
    prefix |= bin << shift;
    mask |= 255u << shift;
  }
  thr = prefix;
}

// Exclusive prefix sum, in place, of the n ints at `a` (LDS) by the whole
// workgroup of kThreadsT threads; `tot_sh` is scratch for one int per wave.
// Begins and ends with a barrier.
template <int kThreadsT>
__device__ __forceinline__ void block_exclusive_scan(int* a, int n, int* tot_sh) {
  constexpr int kSelThreads = kThreadsT, kSelWaves = kThreadsT / 64;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  int carry = 0;
  for (int base = 0; base < n; base += kSelThreads) {
    __syncthreads();
    const int e = base + tid;
    const int v = e < n ? a[e] : 0;
    int incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int y = __shfl_up(incl, off);
      if (lane >= off) incl += y;
    }
    if (lane == 63) tot_sh[wave] = incl;
    __syncthreads();
    int before = carry;
    int tile = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) {
      const int tw = tot_sh[w];
      if (w < wave) before += tw;
      tile += tw;
    }
    if (e < n) a[e] = before + incl - v;
    carry += tile;
  }
  __syncthreads();
}

}  // namespace xkv

#endif  // XKV_SELECT_UTIL_H
