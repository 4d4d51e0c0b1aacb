// Shape-generic kernels of the LiSA path: correct for every supported descriptor, fp32
// arithmetic on the vector ALUs.  They are the fp32 path and the fallback of the bf16 path
// for shapes the MFMA kernels do not cover.
//
// Three kernels mirror the three stages of the layer:
//   k_std_scores     A = Q K^T * scale                      (Sec. 2.1 Eq. 2, bracketed term)
//   k_lisa_scores    A_n = Integrate(FFN(A_{n-1}), A_delta)  (Sec. 5.1, Eq. 3-4)
//   k_softmax_v      O = Softmax(A) V over visible keys      (Sec. 2.1 Eq. 1-2)
// Key-side tensors are addressed through explicit strides so that the same kernels serve
// prefill tensors and decode caches (row- or dimension-major K_LR).
#pragma once
#include "lisa_types.h"

namespace lisa {

struct KeyStrides {      // element strides of a [B, Hkv, key, feature] tensor
  long long b, h, j, t;
};

// ---------------------------------------------------------------------------------------
// A[b,h,i,j] = scale * sum_t Q[b,h,i,t] K[b,kv,j,t]   for visible (i,j)
// `scores` (score type, may be null) is the tensor shared with the next layer; `exact`
// (float32, may be null) is the unrounded copy the softmax of this layer consumes.
// grid (ceil(Lk/64), ceil(Lq/64), B*H), block 256; each thread a 4x4 patch of a 64x64 tile.
// ---------------------------------------------------------------------------------------
template <typename T, typename S>
__global__ __launch_bounds__(256) void k_std_scores(const T* __restrict__ q, const T* __restrict__ k,
                                                    KeyStrides ks, S* __restrict__ scores,
                                                    float* __restrict__ exact, int H, int Hkv,
                                                    int Lq, int Lk, int dk, float scale,
                                                    int causal) {
  __shared__ float qs[16][65];
  __shared__ float kt[16][65];
  const int j0 = blockIdx.x * 64, i0 = blockIdx.y * 64;
  const int b = blockIdx.z / H, h = blockIdx.z % H;
  const int kv = h / (H / Hkv);
  const int i_last = min(i0 + 63, Lq - 1);
  if (j0 >= n_visible(i_last, Lq, Lk, causal)) return;   // tile wholly invisible
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const T* qb = q + ((size_t)(b * H + h) * Lq) * dk;
  const T* kb = k + b * ks.b + kv * ks.h;
  float acc[4][4] = {};
  for (int t0 = 0; t0 < dk; t0 += 16) {
    for (int e = threadIdx.x; e < 64 * 16; e += 256) {
      const int row = e >> 4, t = e & 15;
      const bool tin = t0 + t < dk;
      const int i = i0 + row, j = j0 + row;
      qs[t][row] = (tin && i < Lq) ? elem<T>::load(qb + (size_t)i * dk + t0 + t) : 0.f;
      kt[t][row] = (tin && j < Lk) ? elem<T>::load(kb + j * ks.j + (t0 + t) * ks.t) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int t = 0; t < 16; ++t) {
      float a[4], c[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) { a[u] = qs[t][ty * 4 + u]; c[u] = kt[t][tx * 4 + u]; }
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int w = 0; w < 4; ++w) acc[u][w] += a[u] * c[w];
    }
    __syncthreads();
  }
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int i = i0 + ty * 4 + u;
    if (i >= Lq) continue;
    const int nv = n_visible(i, Lq, Lk, causal);
    const size_t row = ((size_t)(b * H + h) * Lq + i) * Lk;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const int j = j0 + tx * 4 + w;
      if (j < nv) {
        if (scores) elem<S>::store(scores + row + j, acc[u][w] * scale);
        if (exact) exact[row + j] = acc[u][w] * scale;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// A_n for one block = 64 consecutive keys of one query row, all heads; written to `scores`
// (score type, may be null) and, unrounded, to `exact` (float32, may be null).  Four waves; wave s takes
// heads / hidden units s, s+4, ...  Dynamic LDS: x[Din][64], hid[F][64], a_delta[H][64].
// grid (ceil(Lk/64), Lq, B), block 256.
// `mix`: 0 A_n = FFN(A_{n-1}) + A_delta, 1 A_n = FFN([A_{n-1}; A_delta]) (Sec. 5.1, Eq. 4),
// 2 A_n = A_{n-1} + A_delta (LiSA_plus, Sec. 5.5), 3 A_n = A_{n-1} (direct sharing, Sec. 4).
// `act`: 0 ReLU, 1 SiLU, 2 single layer y = W1^T x with F = H (Sec. 5.7).
// ---------------------------------------------------------------------------------------
template <typename T, typename S>
__global__ __launch_bounds__(256) void k_lisa_scores(const T* __restrict__ q_lr,
                                                     const T* __restrict__ k_lr, KeyStrides ks,
                                                     const S* __restrict__ prev,
                                                     const T* __restrict__ w1,
                                                     const T* __restrict__ w2,
                                                     S* __restrict__ scores,
                                                     float* __restrict__ exact, int H, int Hkv,
                                                     int Lq, int Lk, int r, int F, int mix, int act,
                                                     float dscale, int causal) {
  extern __shared__ float sm[];
  const bool concat = mix == 1, has_ffn = mix <= 1, has_delta = mix != 3;
  const int Din = concat ? 2 * H : H;
  float* xs = sm;
  float* hs = xs + Din * 64;
  float* ds = hs + F * 64;
  const int j0 = blockIdx.x * 64, i = blockIdx.y, b = blockIdx.z;
  const int nv = n_visible(i, Lq, Lk, causal);
  if (j0 >= nv) return;
  const int pj = threadIdx.x & 63, sl = threadIdx.x >> 6;
  const int j = j0 + pj;
  const bool live = j < nv;
  const int group = H / Hkv;
  for (int h = sl; h < H; h += 4) {
    float acc = 0.f, x = 0.f;
    if (live) {
      if (has_delta) {
        const T* qp = q_lr + ((size_t)(b * H + h) * Lq + i) * r;
        const T* kp = k_lr + b * ks.b + (h / group) * ks.h + j * ks.j;
        for (int t = 0; t < r; ++t) acc += elem<T>::load(qp + t) * elem<T>::load(kp + t * ks.t);
      }
      x = elem<S>::load(prev + ((size_t)(b * H + h) * Lq + i) * Lk + j);
    }
    acc *= dscale;
    if (!has_ffn) {                                        // no alignment module: done with this head
      if (live) {
        const size_t at = ((size_t)(b * H + h) * Lq + i) * Lk + j;
        if (scores) elem<S>::store(scores + at, x + acc);
        if (exact) exact[at] = x + acc;
      }
      continue;
    }
    ds[h * 64 + pj] = acc;
    xs[h * 64 + pj] = x;
    if (concat) xs[(H + h) * 64 + pj] = acc;
  }
  if (!has_ffn) return;
  __syncthreads();
  for (int f = sl; f < F; f += 4) {
    float acc = 0.f;
    for (int c = 0; c < Din; ++c) acc += xs[c * 64 + pj] * elem<T>::load(w1 + (size_t)c * F + f);
    hs[f * 64 + pj] = act == 0 ? fmaxf(acc, 0.f) : act == 1 ? acc / (1.f + expf(-acc)) : acc;
  }
  __syncthreads();
  for (int h = sl; h < H; h += 4) {
    float acc = 0.f;
    if (act == 2) {
      acc = hs[h * 64 + pj];
    } else {
      for (int f = 0; f < F; ++f) acc += hs[f * 64 + pj] * elem<T>::load(w2 + (size_t)f * H + h);
    }
    if (!concat) acc += ds[h * 64 + pj];
    if (live) {
      const size_t at = ((size_t)(b * H + h) * Lq + i) * Lk + j;
      if (scores) elem<S>::store(scores + at, acc);
      if (exact) exact[at] = acc;
    }
  }
}

// ---------------------------------------------------------------------------------------
// Online softmax over the visible keys of 8 query rows of one (b,h), times V.
// grid (ceil(Lq/8), H, B), block 256.  Phase 1 (per 128-key chunk): wave w owns rows 2w, 2w+1,
// updates the running max / sum and leaves exp(s - m) in LDS.  Phase 2: every thread owns
// up to 8 output elements (row, d) and accumulates p * V.
// ---------------------------------------------------------------------------------------
template <typename T, typename S, typename O>
__global__ __launch_bounds__(256) void k_softmax_v(const S* __restrict__ scores,
                                                   const T* __restrict__ v, KeyStrides vs,
                                                   O* __restrict__ out, long long out_stride_b,
                                                   long long out_stride_i, long long out_stride_h,
                                                   int H, int Hkv, int Lq, int Lk, int dk,
                                                   int causal) {
  constexpr int R = 8, CH = 128, MAXU = 8;
  __shared__ float ps[R][CH];
  __shared__ float alpha_s[R];
  __shared__ float linv_s[R];
  const int i0 = blockIdx.x * R, h = blockIdx.y, b = blockIdx.z;
  const int kv = h / (H / Hkv);
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int i_last = min(i0 + R - 1, Lq - 1);
  const int nv_max = n_visible(i_last, Lq, Lk, causal);
  const T* vb = v + b * vs.b + kv * vs.h;
  float m_run[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.f, 0.f};
  float acc[MAXU];
#pragma unroll
  for (int u = 0; u < MAXU; ++u) acc[u] = 0.f;
  const int n_out = R * dk;
  for (int c0 = 0; c0 < nv_max; c0 += CH) {
#pragma unroll
    for (int rr = 0; rr < 2; ++rr) {
      const int row = wv * 2 + rr, i = i0 + row;
      const int nv = i < Lq ? n_visible(i, Lq, Lk, causal) : 0;
      const S* sr = scores + ((size_t)(b * H + h) * Lq + (i < Lq ? i : 0)) * Lk;
      const int ja = c0 + lane, jb = c0 + lane + 64;
      const float sa = ja < nv ? elem<S>::load(sr + ja) : -INFINITY;
      const float sb = jb < nv ? elem<S>::load(sr + jb) : -INFINITY;
      const float m_new = fmaxf(m_run[rr], wave_max(fmaxf(sa, sb)));
      float pa = 0.f, pb = 0.f, alpha = 1.f;
      if (m_new > -INFINITY) {
        pa = ja < nv ? __expf(sa - m_new) : 0.f;
        pb = jb < nv ? __expf(sb - m_new) : 0.f;
        alpha = m_run[rr] > -INFINITY ? __expf(m_run[rr] - m_new) : 0.f;
      }
      l_run[rr] = l_run[rr] * alpha + wave_sum(pa + pb);
      m_run[rr] = m_new;
      ps[row][lane] = pa;
      ps[row][lane + 64] = pb;
      if (lane == 0) alpha_s[row] = alpha;
    }
    __syncthreads();
    const int jn = min(CH, nv_max - c0);
#pragma unroll
    for (int u = 0; u < MAXU; ++u) {
      const int idx = threadIdx.x + 256 * u;
      if (idx < n_out) {
        const int row = idx / dk, d = idx - row * dk;
        float a = acc[u] * alpha_s[row];
        const T* vp = vb + (size_t)c0 * vs.j + d * vs.t;
        for (int jj = 0; jj < jn; ++jj) a += ps[row][jj] * elem<T>::load(vp + (size_t)jj * vs.j);
        acc[u] = a;
      }
    }
    __syncthreads();
  }
#pragma unroll
  for (int rr = 0; rr < 2; ++rr)
    if (lane == 0) linv_s[wv * 2 + rr] = l_run[rr] > 0.f ? 1.f / l_run[rr] : 0.f;
  __syncthreads();
#pragma unroll
  for (int u = 0; u < MAXU; ++u) {
    const int idx = threadIdx.x + 256 * u;
    if (idx < n_out) {
      const int row = idx / dk, d = idx - row * dk, i = i0 + row;
      if (i < Lq)
        elem<O>::store(out + b * out_stride_b + i * out_stride_i + h * out_stride_h + d,
                       acc[u] * linv_s[row]);
    }
  }
}

// Store the new token's K_LR and V rows at key index `pos` of the caches.
// grid (Hkv, B), block 128.
template <typename T>
__global__ void k_append(const T* __restrict__ k_new, const T* __restrict__ v_new, T* k_cache,
                         KeyStrides ks, T* v_cache, KeyStrides vs, int Hkv, int r, int dk, int pos) {
  const int kvh = blockIdx.x, b = blockIdx.y;
  for (int t = threadIdx.x; t < r; t += blockDim.x)
    k_cache[b * ks.b + kvh * ks.h + pos * ks.j + t * ks.t] = k_new[((size_t)b * Hkv + kvh) * r + t];
  for (int t = threadIdx.x; t < dk; t += blockDim.x)
    v_cache[b * vs.b + kvh * vs.h + pos * vs.j + t * vs.t] = v_new[((size_t)b * Hkv + kvh) * dk + t];
}

// Prefill -> decode hand-over of the K_LR cache in the dimension-major layout:
// cache[b][kv][t][j] = k_lr[b][kv][j][t] for j < Lk, through a 64-token LDS tile so that both
// sides move contiguous runs.  grid (ceil(Lk / 64), Hkv, B), block 256; r <= 128.
template <typename T>
__global__ __launch_bounds__(256) void k_kcache_fill_dim_major(const T* __restrict__ k_lr, T* __restrict__ cache,
                                                               int Hkv, int Lk, int r, int Lmax) {
  __shared__ T tile[64 * 129];
  const int j0 = blockIdx.x * 64, n = min(64, Lk - j0);
  const size_t bh = (size_t)blockIdx.z * Hkv + blockIdx.y;
  const T* src = k_lr + (bh * Lk + j0) * r;              // n * r contiguous elements
  for (int e = threadIdx.x; e < n * r; e += 256) tile[(e / r) * (r + 1) + e % r] = src[e];
  __syncthreads();
  T* dst = cache + bh * r * Lmax + j0;
  for (int e = threadIdx.x; e < r * 64; e += 256) {
    const int t = e >> 6, j = e & 63;
    if (j < n) dst[(size_t)t * Lmax + j] = tile[j * (r + 1) + t];
  }
}

// Row copy of n_rows rows of row_elems elements from a dense [B*Hkv][n_rows] tensor into the
// first rows of a [B*Hkv][Lmax] cache.  grid (ceil(n_rows * row_elems / 1024), B * Hkv), block 256.
template <typename T>
__global__ __launch_bounds__(256) void k_cache_fill_rows(const T* __restrict__ src, T* __restrict__ cache,
                                                         int n_rows, int row_elems, int Lmax) {
  const size_t bh = blockIdx.y;
  const size_t n = (size_t)n_rows * row_elems;
  const T* s = src + bh * n;
  T* d = cache + bh * (size_t)Lmax * row_elems;
  for (size_t e = (size_t)blockIdx.x * 1024 + threadIdx.x; e < min(n, ((size_t)blockIdx.x + 1) * 1024); e += 256)
    d[e] = s[e];
}

// ---------------------------------------------------------------------------------------
// Two-layer ReLU network that equals a linear map exactly: relu(u) - relu(-u) = u.
//   w1o [Din][2H] = [W, -W],  w2o [2H][H] = [I; -I]     (W = w1_user [Din][H], or the identity when
// w1_user is null, Din = H).  Lets the single-layer alignment FFN (Sec. 5.7; LiSA_SL: 2h x h on the
// concatenation) and LiSA_plus (Sec. 5.5: no FFN, i.e. the identity) run on the kernels built for
// the two-layer ReLU form.
// grid ceil((2 Din H + 2 H H) / 256), block 256.
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_synth_relu_ffn(const T* __restrict__ w1_user, T* __restrict__ w1o,
                                                        T* __restrict__ w2o, int Din, int H) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  const int n1 = 2 * Din * H, n2 = 2 * H * H;
  if (idx < n1) {
    const int c = idx / (2 * H), f = idx % (2 * H);        // w1o[c][f]
    const int fo = f < H ? f : f - H;
    const float w = w1_user ? elem<T>::load(w1_user + (size_t)c * H + fo) : (c == fo ? 1.f : 0.f);
    elem<T>::store(w1o + idx, f < H ? w : -w);
  } else if (idx < n1 + n2) {
    const int j = idx - n1, f = j / H, h = j % H;          // w2o[f][h]
    elem<T>::store(w2o + j, f == h ? 1.f : (f == H + h ? -1.f : 0.f));
  }
}

// Zero fill in 16-byte pieces (n16 of them), for scratch operands; a kernel rather than a memset so
// that callers may capture the launch in a graph.  grid ceil(n16 / 256), block 256.
__global__ __launch_bounds__(256) void k_zero16(uint4* __restrict__ p, size_t n16) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n16) p[i] = make_uint4(0u, 0u, 0u, 0u);
}

}  // namespace lisa
