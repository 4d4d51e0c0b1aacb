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

// 16 bytes of a score tensor, read once by this kernel: a non-temporal load
template <class P>
__device__ __forceinline__ uint4 kd_ld16(const P* p) {
  typedef unsigned kd_u32x4 __attribute__((ext_vector_type(4)));
  const kd_u32x4 v = __builtin_nontemporal_load((const kd_u32x4*)p);
  return make_uint4(v[0], v[1], v[2], v[3]);
}

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
    // [B, n_rb, n_kt, H, 16, 32]: the visible tiles of a row block (key tiles 0 .. last, all heads)
    // are one run of consecutive KB in each tensor.  A workgroup takes a long and a short row block
    // at a time (equal work), a wave every fourth KB of the run, KD_UN of them in flight; the
    // loads of the run's tail are clamped, not branched around (a load behind a branch makes the
    // compiler wait for all earlier ones), and count nothing.  Tiles above the diagonal are not read.
    // (few pairs: each is cut into `parts` interleaved shares of its runs, so that the grid has work)
    const int n_half = (n_rb + 1) / 2;
    const long long n_pairs = (long long)g.B * n_half;
    const int parts = (int)max(1LL, min((long long)gridDim.x / n_pairs, 64LL));
    for (long long item = blockIdx.x; item < n_pairs * parts; item += gridDim.x) {
      const long long pair = item / parts;
      const int part = (int)(item % parts), kw = 4 * parts;   // this wave: every kw-th KB from 4 part + wv
      const int b = (int)(pair / n_half), p = (int)(pair % n_half);
#pragma unroll 1
      for (int side = 0; side < 2; ++side) {
        const int rb = side ? p : n_rb - 1 - p;
        if (side && rb >= n_rb - 1 - p) break;               // (the middle block of an odd count is alone)
        const int i_last = min(16 * rb + 15, g.Lq - 1);
        const int n_keys = g.causal ? min(g.Lk, i_last + 1 + shift) : g.Lk;
        const int run = (n_keys + 31) / 32 * g.H;            // KB of this row block that hold visible entries
        if (run <= 0) continue;
        const size_t base = ((size_t)b * n_rb + rb) * n_kt * g.H * 512 + lane * 8;
        const int i = 16 * rb + (lane >> 2);
        const int vis_row = i < g.Lq ? (g.causal ? min(g.Lk, i + 1 + shift) : g.Lk) : 0;
        for (int k0 = 4 * part + wv; k0 < run; k0 += kw * KD_UN) {
          uint4 av[KD_UN], tv[KD_UN];
#pragma unroll
          for (int u = 0; u < KD_UN; ++u) {
            const size_t at = base + (size_t)min(k0 + kw * u, run - 1) * 512;
            if (sizeof(S) == 2) {
              av[u] = kd_ld16(a + at);
              tv[u] = kd_ld16(t + at);
            }
          }
#pragma unroll
          for (int u = 0; u < KD_UN; ++u) {
            const int k = k0 + kw * u;
            const int j8 = 32 * (k / g.H) + 8 * (lane & 3);
            const int nvis = k < run ? vis_row : 0;
            float sm = 0.f;
            if (sizeof(S) == 2) {
              const half_t* ah = (const half_t*)&av[u];
              const half_t* th = (const half_t*)&tv[u];
#pragma unroll
              for (int e = 0; e < 8; ++e)
                if (j8 + e < nvis) sm += huber1((float)ah[e], (float)th[e], g.delta);
            } else {
              const size_t at = base + (size_t)min(k, run - 1) * 512;
#pragma unroll
              for (int e = 0; e < 8; ++e)
                if (j8 + e < nvis) sm += huber1(elem<S>::load(a + at + e), elem<S>::load(t + at + e), g.delta);
            }
            acc += (double)sm;
          }
        }
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
          const uint4 av = kd_ld16(a + base + j8), tv = kd_ld16(t + base + j8);
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
