// Regression term of the knowledge-distillation loss (Sec. 5.1 "Training strategy"; App. C.1
// "Huber loss function"): for one LiSA layer, the mean over the visible entries of
//   L_delta(a, t) = (a - t)^2 / 2            if |a - t| <= delta
//                   delta (|a - t| - delta / 2) otherwise,
// a = A_n of the student, t = A_n^* of the teacher.  Two passes over nothing but the two score
// tensors: HBM-bound, 2 x 2 bytes per visible entry.
//
// k_kd_huber_part: one wave per score row (b, h, i), or per tile of a head in the tiled layout;
// lanes take runs of 8 keys (16-byte loads where the layout allows), float32 within a lane, float64 from the wave sum on; one partial sum per
// workgroup, in a fixed place.  k_kd_huber_finish: one workgroup adds the partial sums in a fixed
// order (the result does not depend on scheduling) and writes
//   out[0] = (accumulate ? out[0] : 0) + weight * mean,   out[1] = mean
// so that L_KD = (1 / |S|) sum over the layers of S is |S| calls with weight 1 / |S|.
#pragma once
#include "lisa_types.h"

namespace lisa {

constexpr int KD_UN = 4;   // tiles of a wave whose loads are in flight together (tiled layout)

struct KdArgs {
  const void* a;          // student scores
  const void* t;          // teacher scores, same layout
  double* part;           // [n_blocks] partial sums
  double* out;            // [2]
  int B, H, Lq, Lk, causal, tiled;
  float delta, weight;
  int accumulate, n_blocks;
  long long n_rows;       // B * H * Lq
  double count;           // visible entries of the whole tensor
};

__device__ __forceinline__ float huber1(float a, float t, float delta) {
  const float d = fabsf(a - t);
  return d <= delta ? 0.5f * d * d : delta * (d - 0.5f * delta);
}

// S = score element type (half_t or float)
template <typename S>
__global__ __launch_bounds__(256) void k_kd_huber_part(KdArgs g) {
  __shared__ double s_part[4];
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int shift = g.Lk - g.Lq;
  const int n_rb = (g.Lq + 15) / 16, n_kt = (g.Lk + 31) / 32;
  const S* a = (const S*)g.a;
  const S* t = (const S*)g.t;
  double acc = 0.0;
  if (g.tiled) {
    // [B, n_rb, n_kt, H, 16, 32]: one wave per tile of a head (1 KB of each tensor, lane -> row
    // lane / 4, 8 keys); tiles that no row of their block can see are skipped unread
    const long long n_tiles = (long long)g.B * n_rb * n_kt * g.H;
    const long long stride = (long long)gridDim.x * 4;
    for (long long tile0 = (long long)blockIdx.x * 4 + wv; tile0 < n_tiles; tile0 += KD_UN * stride) {
      uint4 av[KD_UN], tv[KD_UN];
      int nvis[KD_UN], j8[KD_UN];
#pragma unroll
      for (int u = 0; u < KD_UN; ++u) {
        const long long tile = tile0 + u * stride;
        nvis[u] = 0;
        j8[u] = 0;
        av[u] = tv[u] = uint4{0, 0, 0, 0};
        if (tile >= n_tiles) continue;                        // (wave-uniform)
        const int kt = (int)((tile / g.H) % n_kt);
        const int rb = (int)((tile / g.H / n_kt) % n_rb);
        const int i_last = min(16 * rb + 15, g.Lq - 1);
        if (32 * kt >= (g.causal ? min(g.Lk, i_last + 1 + shift) : g.Lk)) continue;   // (wave-uniform)
        const int i = 16 * rb + (lane >> 2);
        j8[u] = 32 * kt + 8 * (lane & 3);
        nvis[u] = i < g.Lq ? (g.causal ? min(g.Lk, i + 1 + shift) : g.Lk) : 0;
        const size_t at = (size_t)tile * 512 + lane * 8;
        if (sizeof(S) == 2) {
          av[u] = *(const uint4*)(a + at);
          tv[u] = *(const uint4*)(t + at);
        } else {
          float s = 0.f;
#pragma unroll
          for (int e = 0; e < 8; ++e)
            if (j8[u] + e < nvis[u]) s += huber1(elem<S>::load(a + at + e), elem<S>::load(t + at + e), g.delta);
          acc += (double)s;
          nvis[u] = 0;
        }
      }
#pragma unroll
      for (int u = 0; u < KD_UN; ++u) {
        const half_t* ah = (const half_t*)&av[u];
        const half_t* th = (const half_t*)&tv[u];
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (j8[u] + e < nvis[u]) s += huber1((float)ah[e], (float)th[e], g.delta);
        acc += (double)s;
      }
    }
  } else {
    for (long long row = (long long)blockIdx.x * 4 + wv; row < g.n_rows; row += (long long)gridDim.x * 4) {
      const int i = (int)(row % g.Lq);
      const int nvis = g.causal ? min(g.Lk, i + 1 + shift) : g.Lk;
      float s = 0.f;
      const size_t base = (size_t)row * g.Lk;
      const bool vec = sizeof(S) == 2 && g.Lk % 8 == 0;      // 16-byte aligned runs of 8 (bases are checked on the host)
      for (int j8 = lane * 8; j8 < nvis; j8 += 512) {
        if (vec) {
          const uint4 av = *(const uint4*)(a + base + j8), tv = *(const uint4*)(t + base + j8);
          const half_t* ah = (const half_t*)&av;
          const half_t* th = (const half_t*)&tv;
#pragma unroll
          for (int e = 0; e < 8; ++e)
            if (j8 + e < nvis) s += huber1((float)ah[e], (float)th[e], g.delta);
        } else {
          for (int e = 0; e < 8 && j8 + e < nvis; ++e)
            s += huber1(elem<S>::load(a + base + j8 + e), elem<S>::load(t + base + j8 + e), g.delta);
        }
      }
      acc += (double)s;
    }
  }
  // per lane: float32 within a run of 8 keys, float64 across the runs; one wave sum at the end
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
  if (lane == 0) s_part[wv] = acc;
  __syncthreads();
  if (threadIdx.x == 0) g.part[blockIdx.x] = (s_part[0] + s_part[1]) + (s_part[2] + s_part[3]);
}

__global__ __launch_bounds__(256) void k_kd_huber_finish(KdArgs g) {
  __shared__ double s_sum[256];
  double s = 0.0;
  for (int k = threadIdx.x; k < g.n_blocks; k += 256) s += g.part[k];
  s_sum[threadIdx.x] = s;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) s_sum[threadIdx.x] += s_sum[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double mean = s_sum[0] / g.count;
    g.out[0] = (g.accumulate ? g.out[0] : 0.0) + (double)g.weight * mean;
    g.out[1] = mean;
  }
}

}  // namespace lisa
