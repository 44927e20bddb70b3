// Top-k threshold search shared by the selection kernels (Alg. 2 step 5, TopK):
// a radix select over fp32 bit patterns, for one workgroup of kSelThreads
// threads per stream.
#ifndef XKV_SELECT_UTIL_H
#define XKV_SELECT_UTIL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace xkv {

constexpr int kSelThreads = 512;
constexpr int kSelWaves = kSelThreads / 64;

struct RadixShared {
  unsigned hist[256];
  int scan[kSelWaves];
  unsigned sel_bin, sel_need;
};

// Number of set bits of a wave-wide vote below this lane.
__device__ __forceinline__ int rank_in_wave(unsigned long long vote) {
  return __builtin_amdgcn_mbcnt_hi(static_cast<unsigned>(vote >> 32),
                                   __builtin_amdgcn_mbcnt_lo(static_cast<unsigned>(vote), 0));
}

// The kk-th largest of the n keys key_at(0 .. n-1), 1 <= kk <= n, compared as
// unsigned integers (for non-negative floats that is the float order): four
// passes over 8 bits each, every pass a 256-bin histogram of the keys that
// still match the prefix found so far.  On return `thr` is that key and `need`
// says how many of the keys equal to it belong to the top kk (the keys above it
// all do).  Every thread of the workgroup must call it; ends with a barrier.
template <typename KeyAt>
__device__ __forceinline__ void radix_select(KeyAt key_at, int n, int kk, RadixShared& sh,
                                             unsigned& thr, unsigned& need) {
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  unsigned prefix = 0, mask = 0;
  need = static_cast<unsigned>(kk);
  for (int shift = 24; shift >= 0; shift -= 8) {
    if (tid < 256) sh.hist[tid] = 0;
    __syncthreads();
    for (int j = tid; j < n; j += kSelThreads) {
      const unsigned key = key_at(j);
      if ((key & mask) == prefix) atomicAdd(&sh.hist[(key >> shift) & 255u], 1u);
    }
    __syncthreads();
    // Thread t < 256 takes bin 255 - t; an inclusive scan over t finds the bin
    // in which the running count, from the top, reaches `need`.
    unsigned cnt = 0, incl = 0;
    if (tid < 256) {
      cnt = sh.hist[255 - tid];
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
    prefix |= sh.sel_bin << shift;
    mask |= 255u << shift;
    need = sh.sel_need;
    __syncthreads();
  }
  thr = prefix;
}

}  // namespace xkv

#endif  // XKV_SELECT_UTIL_H
