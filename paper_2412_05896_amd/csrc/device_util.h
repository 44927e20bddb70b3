// Device helpers for gfx950 (wave64): cross-lane reductions and the unpacking
// of 16-byte row fragments into fp32.
#ifndef XKV_DEVICE_UTIL_H
#define XKV_DEVICE_UTIL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace xkv {

// Element tags.  A row fragment is always one 16-byte load per lane.
struct F32 { static constexpr int kBytes = 4; static constexpr int kPerLane = 4; };
struct BF16 { static constexpr int kBytes = 2; static constexpr int kPerLane = 8; };

template <typename T> struct Unpack;
template <> struct Unpack<F32> {
  static __device__ __forceinline__ void run(const uint4& r, float (&f)[4]) {
    f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
    f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
  }
};
// bfloat16 is the upper half of an fp32: widening is a shift or a mask.
template <> struct Unpack<BF16> {
  static __device__ __forceinline__ void run(const uint4& r, float (&f)[8]) {
    f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xffff0000u);
    f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xffff0000u);
    f[4] = __uint_as_float(r.z << 16); f[5] = __uint_as_float(r.z & 0xffff0000u);
    f[6] = __uint_as_float(r.w << 16); f[7] = __uint_as_float(r.w & 0xffff0000u);
  }
};

// 16-byte load of data that is read once per kernel: the non-temporal hint keeps
// the stream from displacing other lines in the caches, which measurably raises
// the HBM read rate of a pure streaming kernel on this GPU.
__device__ __forceinline__ uint4 load_stream16(const void* p) {
  typedef unsigned int v4u __attribute__((ext_vector_type(4)));
  const v4u t = __builtin_nontemporal_load(static_cast<const v4u*>(p));
  return make_uint4(t.x, t.y, t.z, t.w);
}

// Store of a result that the same kernel never reads back, next to a large
// streaming read.  Stores cost read bandwidth far beyond their volume on this GPU;
// of the cache policies of the store instruction, system scope (sc0 sc1: written
// through, nothing kept) measured cheapest (3 KiB of stores per 128 KiB read:
// 6.3 TB/s of reads, against 6.15 with the non-temporal hint and 5.98 with none).
__device__ __forceinline__ void store_stream(float* p, float v) {
  asm volatile("global_store_dword %0, %1, off sc0 sc1" : : "v"(p), "v"(v) : "memory");
}
// 16 bytes; p must be 16-byte aligned.
__device__ __forceinline__ void store_stream16(float* p, const float (&v)[4]) {
  typedef float f4 __attribute__((ext_vector_type(4)));
  const f4 t = {v[0], v[1], v[2], v[3]};
  asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" : : "v"(p), "v"(t) : "memory");
}
__device__ __forceinline__ void store_stream16(void* p, const uint4& v) {
  typedef unsigned int u4 __attribute__((ext_vector_type(4)));
  const u4 t = {v.x, v.y, v.z, v.w};
  asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" : : "v"(p), "v"(t) : "memory");
}
// 16-byte store of a row that this kernel and the next ones do not read back.
__device__ __forceinline__ void store_nt16(void* p, const uint4& v) {
  typedef unsigned int u4 __attribute__((ext_vector_type(4)));
  const u4 t = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(t, static_cast<u4*>(p));
}
// One DPP move: every lane reads the lane that `kCtrl` names within its row of
// 16 lanes.  Only controls whose source lane always exists are used here.
template <int kCtrl>
__device__ __forceinline__ float dpp_read(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), kCtrl, 0xf, 0xf, false));
}

constexpr int kDppQuadSwap1 = 0xB1;      // quad_perm [1,0,3,2]
constexpr int kDppQuadSwap2 = 0x4E;      // quad_perm [2,3,0,1]
constexpr int kDppRowHalfMirror = 0x141; // lane i <-> 7-i within 8
constexpr int kDppRowMirror = 0x140;     // lane i <-> 15-i within 16

// Sum over aligned groups of kLanes consecutive lanes (4, 8, 16, 32 or 64); every lane of
// a group ends with the same bits (each step adds a value to its mirror image).
template <int kLanes>
__device__ __forceinline__ float group_sum(float x) {
  static_assert(kLanes == 4 || kLanes == 8 || kLanes == 16 || kLanes == 32 || kLanes == 64, "");
  x += dpp_read<kDppQuadSwap1>(x);
  x += dpp_read<kDppQuadSwap2>(x);
  if (kLanes >= 8) x += dpp_read<kDppRowHalfMirror>(x);
  if (kLanes >= 16) x += dpp_read<kDppRowMirror>(x);
  if (kLanes >= 32) x += __shfl_xor(x, 16);
  if (kLanes >= 64) x += __shfl_xor(x, 32);
  return x;
}

__device__ __forceinline__ float wave_max(float x) {
  x = fmaxf(x, dpp_read<kDppQuadSwap1>(x));
  x = fmaxf(x, dpp_read<kDppQuadSwap2>(x));
  x = fmaxf(x, dpp_read<kDppRowHalfMirror>(x));
  x = fmaxf(x, dpp_read<kDppRowMirror>(x));
  x = fmaxf(x, __shfl_xor(x, 16));
  x = fmaxf(x, __shfl_xor(x, 32));
  return x;
}

__device__ __forceinline__ float wave_sum(float x) { return group_sum<64>(x); }

// 2^x with the hardware instruction (1 ulp; results below the normal range
// flush to zero, which is what a vanishing probability should do).
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

}  // namespace xkv

#endif  // XKV_DEVICE_UTIL_H
