// Element types and small device helpers shared by the LiSA kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lisa {

// Storage tags.  bf16 is kept as its raw 16 bits; half is the native _Float16.
struct bf16_t { uint16_t bits; };
typedef _Float16 half_t;

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t bits) {
  return __uint_as_float(bits << 16);
}
// Round-to-nearest-even float -> bf16 bits (NaN kept quiet).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t x = __float_as_uint(f);
  if ((x & 0x7fffffffu) > 0x7f800000u) return 0x7fc0u;
  x += 0x7fffu + ((x >> 16) & 1u);
  return x >> 16;
}
// Saturating float -> half: scores beyond the half range are clamped to +-65504 instead
// of becoming infinities that would poison the softmax of the next layer.
__device__ __forceinline__ half_t f32_to_half_sat(float f) {
  return (half_t)__builtin_amdgcn_fmed3f(f, -65504.0f, 65504.0f);   // one median-of-three
}

template <typename T> struct elem;
template <> struct elem<float> {
  static __device__ __forceinline__ float load(const float* p) { return *p; }
  static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct elem<bf16_t> {
  static __device__ __forceinline__ float load(const bf16_t* p) { return bf16_bits_to_f32(p->bits); }
  static __device__ __forceinline__ void store(bf16_t* p, float v) { p->bits = (uint16_t)f32_to_bf16_bits(v); }
};
template <> struct elem<half_t> {
  static __device__ __forceinline__ float load(const half_t* p) { return (float)*p; }
  static __device__ __forceinline__ void store(half_t* p, float v) { *p = f32_to_half_sat(v); }
};

// Number of keys visible to query row i.
__device__ __host__ __forceinline__ int n_visible(int i, int Lq, int Lk, int causal) {
  if (!causal) return Lk;
  int n = i + 1 + (Lk - Lq);
  return n < 0 ? 0 : (n > Lk ? Lk : n);
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

}  // namespace lisa
