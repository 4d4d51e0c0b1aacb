// Reference kernels for benchmarks: what a plain read stream and a plain chain of MFMAs reach on the
// chip the library runs on (and a plain write stream).  They compute nothing of the method; bench.py times them next to the
// library's kernels so that a roofline fraction can also be read against what is reachable.
#pragma once
#include "mfma_ffn.h"

namespace lisa {

typedef float probe_f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned probe_u32x4 __attribute__((ext_vector_type(4)));

// Reads n16 16-byte pieces once, a workgroup 32 KB at a time with 8 loads in flight per lane; writes nothing unless the data match a
// pattern that random or zero data do not have (keeps the loads alive).  Any grid, block 256.
__global__ __launch_bounds__(256) void k_probe_read(const probe_u32x4* __restrict__ src, size_t n16, probe_u32x4* sink) {
  probe_u32x4 acc = {0u, 0u, 0u, 0u};
  const size_t n_chunks = n16 / 2048;                       // chunks of 32 KB, dealt to the workgroups in turn
  for (size_t ch = blockIdx.x; ch < n_chunks; ch += gridDim.x) {
    const probe_u32x4* p = src + ch * 2048 + threadIdx.x;
    probe_u32x4 r[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) r[u] = __builtin_nontemporal_load(p + u * 256);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= r[u];
  }
  for (size_t i = n_chunks * 2048 + (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256)
    acc ^= src[i];
  if (acc[0] == 0x9e3779b9u && acc[1] == 0x7f4a7c15u && acc[2] == 0xf39cc060u && acc[3] == 0x5cedc834u) sink[0] = acc;
}

// Writes n16 16-byte pieces once with non-temporal stores, a workgroup 32 KB at a time: piece i gets
// {seed, low word of i, high word of i, ~seed}.  Any grid, block 256.
__global__ __launch_bounds__(256) void k_probe_write(probe_u32x4* __restrict__ dst, size_t n16, unsigned seed) {
  const size_t n_chunks = n16 / 2048;
  for (size_t ch = blockIdx.x; ch < n_chunks; ch += gridDim.x) {
    const size_t i0 = ch * 2048 + threadIdx.x;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const size_t i = i0 + u * 256;
      const probe_u32x4 v = {seed, (unsigned)i, (unsigned)(i >> 32), ~seed};
      __builtin_nontemporal_store(v, dst + i);
    }
  }
  for (size_t i = n_chunks * 2048 + (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) {
    const probe_u32x4 v = {seed, (unsigned)i, (unsigned)(i >> 32), ~seed};
    dst[i] = v;
  }
}

// iters rounds of independent MFMAs on constant operands per wave: SHAPE 0: 8 x 16x16x32 f16 (the
// shape of the library's FFNs), 1: 4 x 32x32x16 f16 (the same flops per round).  block 256.
template <int SHAPE>
__global__ __launch_bounds__(256) void k_probe_mfma(int iters, float seed, float* sink) {
  f16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    a[e] = (_Float16)(seed + (threadIdx.x & 63) * 0.001f);
    b[e] = (_Float16)(seed * 0.5f);
  }
  float s = 0.f;
  if (SHAPE == 0) {
    f32x4 acc[8];
#pragma unroll
    for (int n = 0; n < 8; ++n) acc[n] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int n = 0; n < 8; ++n) acc[n] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, acc[n], 0, 0, 0);
    }
#pragma unroll
    for (int n = 0; n < 8; ++n) s += acc[n][0] + acc[n][3];
  } else {
    probe_f32x16 acc[4];
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[n][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int n = 0; n < 4; ++n) acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[n], 0, 0, 0);
    }
#pragma unroll
    for (int n = 0; n < 4; ++n) s += acc[n][0] + acc[n][7];
  }
  if (s == 12345.678f) sink[0] = s;
}

}  // namespace lisa
