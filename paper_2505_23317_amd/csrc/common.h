// Shared device/host helpers for the cfdetr kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cfdetr {

constexpr int kWave = 64;
constexpr int kMaxLevels = 3;
constexpr int kMaxBatch = 64;

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef uint16_t bf16_t;  // storage type: raw bf16 bit pattern

// Geometry of the patch pyramid, passed by value to kernels.
struct Pyramid {
  int n_levels;
  int patch[kMaxLevels];
  int rows[kMaxLevels];
  int cols[kMaxLevels];
  int img_h, img_w;
};

__device__ __forceinline__ float bf16_to_f32(bf16_t v) {
  return __uint_as_float(static_cast<uint32_t>(v) << 16);
}

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;

// Two floats -> two bf16 in one dword (lo in bits 0..15), round-to-nearest-even:
// this is the hardware's packed convert (v_cvt_pk_bf16_f32).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2 v = {lo, hi};
  bf16x2 b = __builtin_convertvector(v, bf16x2);
  return *reinterpret_cast<uint32_t*>(&b);
}

__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  return static_cast<bf16_t>(pack_bf16x2(f, 0.f) & 0xFFFFu);
}

__device__ __forceinline__ int tok_level(int32_t t) { return (t >> 28) & 0x7; }
__device__ __forceinline__ int tok_row(int32_t t) { return (t >> 14) & 0x3FFF; }
__device__ __forceinline__ int tok_col(int32_t t) { return t & 0x3FFF; }

// Frame index of global token t: the i with cu[i] <= t < cu[i+1] (cu[0] = 0, offsets
// ascending; frames may be empty, and the last i with cu[i] <= t is the one that holds t).
// A bisection: its loads depend on each other, and a walk from the front costs up to B of
// those round trips in front of a tile's first instruction.
__device__ __forceinline__ int frame_of_token(const int32_t* __restrict__ cu, int B, int t) {
  int lo = 0, hi = B - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (cu[mid] <= t) lo = mid; else hi = mid - 1;
  }
  return lo;
}

template <typename T>
__device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

}  // namespace cfdetr
