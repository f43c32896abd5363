// Shared device/host definitions for libechokv (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace echokv {

constexpr int kMaxSeqPerLaunch = 128;  // sequences described by one kernarg block
constexpr int kSlotTokens = 128;       // tokens covered by one split-K partial slot

// Per-launch description of up to kMaxSeqPerLaunch sequences, passed by value
// in the kernel arguments (no device-side metadata, nothing to upload).
struct SeqMeta {
  int64_t start[kMaxSeqPerLaunch];    // first cache-pool row of the sequence
  int32_t len[kMaxSeqPerLaunch];      // valid tokens
  int32_t tbase[kMaxSeqPerLaunch + 1];  // prefix sum of this launch's tiles per sequence
  int32_t sbase[kMaxSeqPerLaunch + 1];  // prefix sum of partial slots per sequence
  int32_t n;
};

// Largest b with base[b] <= x, for a prefix-sum array base[0..n].
__device__ __forceinline__ int find_seq(const int32_t* base, int n, int x) {
  int lo = 0, hi = n;
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (base[mid] <= x) lo = mid; else hi = mid;
  }
  return lo;
}

typedef uint16_t bf16_t;  // raw bfloat16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t h) {
  return __uint_as_float(((uint32_t)h) << 16);
}
// round-to-nearest-even, NaN kept quiet
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

template <typename T> struct Elem;
template <> struct Elem<bf16_t> {
  static constexpr int kVec = 8;  // elements per 16-byte load
  __device__ static __forceinline__ float to_f32(bf16_t x) { return bf16_to_f32(x); }
  __device__ static __forceinline__ bf16_t from_f32(float x) { return f32_to_bf16(x); }
};
template <> struct Elem<float> {
  static constexpr int kVec = 4;
  __device__ static __forceinline__ float to_f32(float x) { return x; }
  __device__ static __forceinline__ float from_f32(float x) { return x; }
};

// 16-byte vector of T unpacked to floats
template <typename T>
__device__ __forceinline__ void load16(const T* p, float (&out)[Elem<T>::kVec]) {
  uint4 raw = *reinterpret_cast<const uint4*>(p);
  if constexpr (sizeof(T) == 2) {
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      out[2 * i] = __uint_as_float(w[i] << 16);
      out[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  } else {
    out[0] = __uint_as_float(raw.x); out[1] = __uint_as_float(raw.y);
    out[2] = __uint_as_float(raw.z); out[3] = __uint_as_float(raw.w);
  }
}

__device__ __forceinline__ float wave_max(float v, int width) {
  for (int o = width >> 1; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v, int width) {
  for (int o = width >> 1; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Sum over aligned groups of W consecutive lanes (every lane gets its group's total).  The steps
// inside a row of 16 lanes are data-parallel-primitive moves folded into the add (no trip through
// the LDS crossbar, which is what a generic lane shuffle costs): swap neighbours, swap pairs,
// mirror inside 8 lanes, mirror inside 16 lanes -- after each step both halves of the next larger
// group hold their own total, so a mirror pairs them as well as a rotation would.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
template <int W>
__device__ __forceinline__ float row_sum(float v) {
  static_assert(W == 1 || W == 2 || W == 4 || W == 8 || W == 16 || W == 32 || W == 64, "power of two");
  if constexpr (W >= 2) v += dpp_move<0xB1>(v);      // quad_perm [1, 0, 3, 2]
  if constexpr (W >= 4) v += dpp_move<0x4E>(v);      // quad_perm [2, 3, 0, 1]
  if constexpr (W >= 8) v += dpp_move<0x141>(v);     // row_half_mirror
  if constexpr (W >= 16) v += dpp_move<0x140>(v);    // row_mirror
  if constexpr (W >= 32) v += __shfl_xor(v, 16, 64);
  if constexpr (W >= 64) v += __shfl_xor(v, 32, 64);
  return v;
}

}  // namespace echokv
