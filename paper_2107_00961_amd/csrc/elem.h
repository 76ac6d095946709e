// Device-side element access for the two storage types of activations: fp32 and bf16.
// A thread always moves 16 bytes: 4 fp32 or 8 bf16 values, widened to fp32 registers on load and
// rounded to nearest even on store.  All arithmetic between a load and a store is fp32 (or fp64).
#pragma once
#include <hip/hip_runtime.h>

namespace resist {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

// fp32 -> bf16 bits, round to nearest even (NaN stays NaN)
__device__ inline unsigned bf16_bits(float f) {
  const __bf16 h = (__bf16)f;
  return (unsigned)__builtin_bit_cast(unsigned short, h);
}
__device__ inline unsigned pack_bf16x2(float lo, float hi) { return bf16_bits(lo) | (bf16_bits(hi) << 16); }
// a bf16 is the upper half of the fp32 of the same value
__device__ inline float bf16_lo(unsigned u) { return __builtin_bit_cast(float, u << 16); }
__device__ inline float bf16_hi(unsigned u) { return __builtin_bit_cast(float, u & 0xffff0000u); }

template <typename T> struct Vec;

template <> struct Vec<float> {
  static constexpr int N = 4;   // elements per 16-byte access
  __device__ static inline void load(const float *p, float (&v)[4]) {
    const f32x4 t = *reinterpret_cast<const f32x4 *>(p);
    v[0] = t[0]; v[1] = t[1]; v[2] = t[2]; v[3] = t[3];
  }
  __device__ static inline void store(float *p, const float (&v)[4]) {
    f32x4 t = {v[0], v[1], v[2], v[3]};
    *reinterpret_cast<f32x4 *>(p) = t;
  }
  __device__ static inline float get(const float *p) { return *p; }
  __device__ static inline void put(float *p, float v) { *p = v; }
  // the 16 bytes as they are in memory (requested now, widened when used)
  typedef f32x4 Raw;
  __device__ static inline Raw load_raw(const float *p) { return *reinterpret_cast<const f32x4 *>(p); }
  __device__ static inline void unpack(const Raw &t, float (&v)[4]) {
    v[0] = t[0]; v[1] = t[1]; v[2] = t[2]; v[3] = t[3];
  }
};

template <> struct Vec<__bf16> {
  static constexpr int N = 8;
  __device__ static inline void load(const __bf16 *p, float (&v)[8]) {
    const u32x4 t = *reinterpret_cast<const u32x4 *>(p);
#pragma unroll
    for (int i = 0; i < 4; ++i) { v[2 * i] = bf16_lo(t[i]); v[2 * i + 1] = bf16_hi(t[i]); }
  }
  __device__ static inline void store(__bf16 *p, const float (&v)[8]) {
    u32x4 t;
#pragma unroll
    for (int i = 0; i < 4; ++i) t[i] = pack_bf16x2(v[2 * i], v[2 * i + 1]);
    *reinterpret_cast<u32x4 *>(p) = t;
  }
  __device__ static inline float get(const __bf16 *p) { return (float)*p; }
  __device__ static inline void put(__bf16 *p, float v) { *p = (__bf16)v; }
  typedef u32x4 Raw;
  __device__ static inline Raw load_raw(const __bf16 *p) { return *reinterpret_cast<const u32x4 *>(p); }
  __device__ static inline void unpack(const Raw &t, float (&v)[8]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) { v[2 * i] = bf16_lo(t[i]); v[2 * i + 1] = bf16_hi(t[i]); }
  }
};

}  // namespace resist
