// Decode-step kernels (one query row per sequence, Sec. 2.2 / Sec. 5.2): a split-over-context
// pass that streams the key-side cache once, then a small combine.
//
// k_decode_part: one workgroup = one sequence x DEC_CK consecutive keys x ALL heads (the
// alignment FFN couples the heads of a position, Sec. 5.1).  Stages:
//   S1  scores of the chunk into LDS:   LiSA  a_delta[h][j] = scale <q_lr[h], K_LR[kv][j]>  (Eq. 3)
//                                       std   a[h][j]       = scale <q[h],    K[kv][j]>     (Eq. 2)
//                                       direct sharing (Sec. 4): a[h][j] = A_{n-1}[h][j], no key cache
//   S2  (LiSA) A_n = FFN(A_{n-1}) + a_delta, or A_n = FFN([A_{n-1}; a_delta]) in CONCAT form, on
//       the matrix cores, 16 positions per MFMA block
//   S3  per head: chunk maximum, p = exp(a - max), chunk sum; the score row is stored here
//   S4  per head: partial O = sum_j p[j] V[kv][j][:]  -- the HBM stream that dominates
// k_decode_combine merges the per-chunk (max, sum, O) triples of each (sequence, head).
//
// The V (and, for a standard layer, K) stream is read with 16-byte loads, 8 features per lane,
// 64 / (d_k / 8) keys per wave instruction, so every wave instruction covers 1 KB contiguous.
#pragma once
#include "kernels_generic.h"
#include "mfma_ffn.h"

namespace lisa {

constexpr int DEC_CK = 128;      // keys per workgroup
constexpr int DEC_THREADS = 256;

struct DecodeArgs {
  const bf16_t* q;       // LiSA: q_lr [B,H,r]; std: q [B,H,d_k]
  const bf16_t* kc;      // LiSA: K_LR cache; std: K cache
  KeyStrides ks;
  const bf16_t* vc;      // V cache
  KeyStrides vs;
  const half_t* prev;    // [B,H,Lk]   (LiSA)
  const bf16_t* w1;      // [H,F]      (LiSA)
  const bf16_t* w2;      // [F,H]      (LiSA)
  half_t* row_out;       // [B,H,Lk] or null
  float* part_o;         // [B][n_chunk][H][d_k]
  float* part_ml;        // [B][n_chunk][H][2]  (max, sum)
  int H, Hkv, Lk, r, F, n_chunk;
  float scale;
  // The combine of the layer before, which a stack leaves to the next layer's launch (none in a
  // single call): unit u = head u % cmb_H of sequence u / cmb_H, cmb_units of them, the same d_k as
  // this launch.
  int B;
  const float* cmb_o;
  const float* cmb_ml;
  void* cmb_out;
  int cmb_units, cmb_H, cmb_nchunk, cmb_out_f32;
};

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// 16 bytes of a K / K_LR / V cache, read once per step and never again before the whole cache has
// passed: a non-temporal load.  A read stream shaped like this kernel's (2112 regions of 1 MB, a
// wave per head, 256-byte pieces 8 KB apart) reaches 5.7 TB/s with plain loads and 6.4 - 6.6 TB/s
// with these.
__device__ __forceinline__ u32x4 ld_stream(const bf16_t* p) { return __builtin_nontemporal_load((const u32x4*)p); }

// out[b][h][:] = sum_c e^{m_c - M} O_c / sum_c e^{m_c - M} s_c,  M = max_c m_c, for one (h, b) by a
// workgroup of 256 threads: the chunks are dealt to 256 / (DK / 4) groups of DK / 4 lanes (four
// features per lane, independent 16-byte loads), the groups' sums are merged through `lds`
// (4.2 KB, 16-byte aligned).
template <typename O, int DK>
__device__ __forceinline__ void decode_combine_unit(const float* __restrict__ part_o,
                                                    const float* __restrict__ part_ml, O* __restrict__ out,
                                                    int H, int n_chunk, int h, int b, float* lds) {
  constexpr int LPG = DK / 4, NGRP = 256 / LPG;
  float4* s_num = (float4*)lds;                              // [NGRP][LPG]
  float* s_den = lds + NGRP * LPG * 4;                       // [NGRP]
  float* s_max = s_den + NGRP;
  const int tid = threadIdx.x;
  const size_t row0 = (size_t)b * n_chunk * H + h;            // chunk c: row0 + c * H
  if (tid < 64) {
    float m = -INFINITY;
    for (int c = tid; c < n_chunk; c += 64) m = fmaxf(m, part_ml[(row0 + (size_t)c * H) * 2]);
    m = wave_max(m);
    if (tid == 0) *s_max = m;
  }
  __syncthreads();
  const float M = *s_max;
  const int grp = tid / LPG, l = tid % LPG;
  float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
  float den = 0.f;
  for (int c = grp; c < n_chunk; c += NGRP) {
    const size_t at = row0 + (size_t)c * H;
    const float2 ml = *(const float2*)(part_ml + at * 2);
    const float4 po = *(const float4*)(part_o + at * DK + 4 * l);
    const float w = __expf(ml.x - M);
    den += w * ml.y;
    num.x += w * po.x;
    num.y += w * po.y;
    num.z += w * po.z;
    num.w += w * po.w;
  }
  s_num[grp * LPG + l] = num;
  if (l == 0) s_den[grp] = den;
  __syncthreads();
  if (tid < LPG) {
    float4 n = s_num[tid];
    float dsum = s_den[0];
#pragma unroll
    for (int gi = 1; gi < NGRP; ++gi) {
      const float4 x = s_num[gi * LPG + tid];
      n.x += x.x;
      n.y += x.y;
      n.z += x.z;
      n.w += x.w;
      dsum += s_den[gi];
    }
    const float inv = 1.f / dsum;
    O* o = out + ((size_t)b * H + h) * DK + 4 * tid;
    elem<O>::store(o, n.x * inv);
    elem<O>::store(o + 1, n.y * inv);
    elem<O>::store(o + 2, n.z * inv);
    elem<O>::store(o + 3, n.w * inv);
  }
}

// grid (H, B), block 256
template <typename O, int DK>
__global__ __launch_bounds__(256) void k_decode_combine(const float* __restrict__ part_o,
                                                        const float* __restrict__ part_ml,
                                                        O* __restrict__ out, int H, int n_chunk) {
  __shared__ __align__(16) float s_lds[256 * 4 + 64];
  decode_combine_unit<O, DK>(part_o, part_ml, out, H, n_chunk, blockIdx.x, blockIdx.y, s_lds);
}

// LISA_MODE: 0 = standard layer, 1 = LiSA layer in ADD form (HB = blocks of 16 heads), 2 = LiSA
// layer in CONCAT form (HB = blocks of 16 FFN inputs, 2H of them; (HB + 1) / 2 output blocks; the
// FFN weights stay in LDS), 3 = direct sharing: the scores are the previous layer's row as it
// stands (no key-side operand, no FFN; HB, FS unused).  DK: head dimension (64 or 128).
// (four workgroups per compute unit where the kernel is within a few registers of 128 per lane: with
// the caches streamed past the L2 that is worth 2 - 3 % of the step; with plain loads it was not)
template <int LISA_MODE, int HB, int FS, int DK, int ACT = 0>
__global__ __launch_bounds__(DEC_THREADS, (LISA_MODE != 2 && HB <= 2 && FS <= 2 && DK == 128) ? 4 : 1)
void k_decode_part(DecodeArgs a) {
  constexpr int LPK = DK / 8;        // lanes per key in the 16-byte streams
  constexpr int KPW = 64 / LPK;      // keys per wave instruction
  constexpr int UN = 8;              // independent loads in flight per lane in the streams
  extern __shared__ float dec_lds[];
  const int H = a.H, Lk = a.Lk;
  float* a_s = dec_lds;                       // [H][DEC_CK] scores, later probabilities
  float* q_s = a_s + H * DEC_CK;              // LiSA: [H][r], then the FFN weights
  unsigned short* w_s = (unsigned short*)(q_s + ((H * a.r + 3) & ~3));   // 16-byte aligned
  const int chunk = blockIdx.x, b = blockIdx.y;
  const int j0 = chunk * DEC_CK;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int group = H / a.Hkv;
  const int n_here = min(DEC_CK, Lk - j0);    // keys of this chunk that exist (>= 1)

  // ---- S4's stream starts here ------------------------------------------------------------
  // The addresses of the V stream do not depend on the scores: the first batch of every wave is
  // in flight while S1 - S3 run.
  constexpr int V_NBATCH = DEC_CK / KPW / UN;
  static_assert(V_NBATCH % 2 == 0, "items are taken in pairs");
  const int v_js = lane / LPK, v_dc = lane % LPK;
  const int v_items = ((H - wv + 3) / 4) * V_NBATCH;
  auto v_issue = [&](int item, u32x4 (&vv)[UN]) {
    item = min(item, v_items - 1);
    const int h = wv + 4 * (item / V_NBATCH), it = (item % V_NBATCH) * UN;
    const bf16_t* vb = a.vc + b * a.vs.b + (h / group) * a.vs.h + v_dc * 8;
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int jc = min(v_js + (it + u) * KPW, n_here - 1);
      vv[u] = ld_stream(vb + (size_t)(j0 + jc) * a.vs.j);
    }
  };
  u32x4 va[UN];
  if (v_items > 0) v_issue(0, va);
  // ADD form: the A_{n-1} operands of this wave's FFN blocks do not depend on S1 either (clamped
  // addresses; what lies past the heads or the context is zeroed where it is used)
  constexpr int XKS = LISA_MODE == 1 ? MfmaFfn<HB, FS, HB, ACT>::KS : 1;
  constexpr int XNB = DEC_CK / 16 / 4;                     // blocks of 16 positions per wave
  f16x8 xpre[XNB][XKS];
  if (LISA_MODE == 1) {
    const int c = lane & 15, g = lane >> 4;
#pragma unroll
    for (int q = 0; q < XNB; ++q)
#pragma unroll
      for (int ks = 0; ks < XKS; ++ks)
#pragma unroll
        for (int e = 0; e < 8; ++e)
          xpre[q][ks][e] = a.prev[((size_t)b * H + min(32 * ks + 8 * g + e, H - 1)) * Lk +
                                  min(j0 + (wv + 4 * q) * 16 + c, Lk - 1)];
  }

  // ---- S1 ------------------------------------------------------------------------------
  if (LISA_MODE == 3) {
    for (int e = tid; e < H * DEC_CK; e += DEC_THREADS) {
      const int h = e / DEC_CK, pj = e % DEC_CK;
      a_s[e] = pj < n_here ? (float)a.prev[((size_t)b * H + h) * Lk + j0 + pj] : 0.f;
    }
  } else if (LISA_MODE) {
    for (int e = tid; e < H * a.r; e += DEC_THREADS)
      q_s[e] = elem<bf16_t>::load(a.q + (size_t)b * H * a.r + e);
    if (LISA_MODE == 2)
      MfmaFfn<HB, FS, (HB + 1) / 2, ACT>::stage(a.w1, a.w2, 2 * H, a.F, w_s, tid, DEC_THREADS, 0, H, H);
    else
      MfmaFfn<HB, FS, HB, ACT>::stage(a.w1, a.w2, H, a.F, w_s, tid, DEC_THREADS);
    __syncthreads();
    if (a.ks.j == 1 && (a.ks.t & 7) == 0 && (a.ks.h & 7) == 0 && (a.ks.b & 7) == 0) {
      // dimension-major cache with 16-byte aligned rows: 8 keys per lane and load
      const int jo = tid & 15, sl = tid >> 4;                    // 16 head slices
      const int jb = j0 + jo * 8;
      for (int h = sl; h < H; h += DEC_THREADS / 16) {
        float acc[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = 0.f;
        if (jb < Lk) {      // the cache holds Lmax >= 8 ceil(Lk / 8) keys per row (ks.t % 8 == 0)
          const bf16_t* kp = a.kc + b * a.ks.b + (h / group) * a.ks.h + jb;
          // UN rows of the rank axis per batch of independent loads (a row past the rank repeats
          // the last one with a zero factor)
          for (int t0 = 0; t0 < a.r; t0 += UN) {
            u32x4 kvv[UN];
#pragma unroll
            for (int u = 0; u < UN; ++u) kvv[u] = ld_stream(kp + (size_t)min(t0 + u, a.r - 1) * a.ks.t);
#pragma unroll
            for (int u = 0; u < UN; ++u) {
              const float qt = t0 + u < a.r ? q_s[h * a.r + t0 + u] : 0.f;
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                acc[2 * e] += qt * bf16_bits_to_f32(kvv[u][e] & 0xffffu);
                acc[2 * e + 1] += qt * bf16_bits_to_f32(kvv[u][e] >> 16);
              }
            }
          }
        }
        float4* dst = (float4*)(a_s + h * DEC_CK + jo * 8);
        dst[0] = make_float4(acc[0] * a.scale, acc[1] * a.scale, acc[2] * a.scale, acc[3] * a.scale);
        dst[1] = make_float4(acc[4] * a.scale, acc[5] * a.scale, acc[6] * a.scale, acc[7] * a.scale);
      }
    } else {
      const int pj = tid & (DEC_CK - 1), sl = tid / DEC_CK;       // 2 head slices
      const int j = j0 + pj;
      for (int h = sl; h < H; h += DEC_THREADS / DEC_CK) {
        float acc = 0.f;
        if (j < Lk) {
          const bf16_t* kp = a.kc + b * a.ks.b + (h / group) * a.ks.h + j * a.ks.j;
          for (int t = 0; t < a.r; ++t) acc += q_s[h * a.r + t] * elem<bf16_t>::load(kp + t * a.ks.t);
        }
        a_s[h * DEC_CK + pj] = acc * a.scale;
      }
    }
  } else {
    // (items and two register sets as in S4 below)
    constexpr int NBATCH = DEC_CK / KPW / UN;
    const int js = lane / LPK, dc = lane % LPK;
    const int n_items = ((H - wv + 3) / 4) * NBATCH;
    auto issue = [&](int item, u32x4 (&kvv)[UN]) {
      item = min(item, n_items - 1);
      const int h = wv + 4 * (item / NBATCH), it = (item % NBATCH) * UN;
      const bf16_t* kb = a.kc + b * a.ks.b + (h / group) * a.ks.h + dc * 8;
#pragma unroll
      for (int u = 0; u < UN; ++u) {
        const int jc = min(js + (it + u) * KPW, n_here - 1);     // clamped, result unused
        kvv[u] = ld_stream(kb + (size_t)(j0 + jc) * a.ks.j);
      }
    };
    float qf[8];
    auto consume = [&](int item, const u32x4 (&kvv)[UN]) {
      const int h = wv + 4 * (item / NBATCH), bt = item % NBATCH, it = bt * UN;
      if (bt == 0) {
        const u32x4 qv = *(const u32x4*)(a.q + ((size_t)b * H + h) * DK + dc * 8);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          qf[2 * e] = bf16_bits_to_f32(qv[e] & 0xffffu);
          qf[2 * e + 1] = bf16_bits_to_f32(qv[e] >> 16);
        }
      }
#pragma unroll
      for (int u = 0; u < UN; ++u) {
        float acc = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          acc += qf[2 * e] * bf16_bits_to_f32(kvv[u][e] & 0xffffu);
          acc += qf[2 * e + 1] * bf16_bits_to_f32(kvv[u][e] >> 16);
        }
#pragma unroll
        for (int o = LPK / 2; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
        if (dc == 0) a_s[h * DEC_CK + js + (it + u) * KPW] = acc * a.scale;
      }
    };
    u32x4 ka[UN], kb2[UN];
    if (n_items > 0) {
      issue(0, ka);
      for (int item = 0; item < n_items; item += 2) {
        issue(item + 1, kb2);
        consume(item, ka);
        issue(item + 2, ka);
        consume(item + 1, kb2);
      }
    }
  }
  __syncthreads();

  // ---- S2: A_n = FFN(A_{n-1}) + a_delta, or FFN([A_{n-1}; a_delta]) ---------------------------
  if (LISA_MODE == 2) {
    typedef MfmaFfn<HB, FS, (HB + 1) / 2, ACT> Ffn;
    const int c = lane & 15, g = lane >> 4;
    for (int nb = wv; nb < DEC_CK / 16; nb += 4) {
      // a wave owns its 16 positions: it reads their a_delta of all heads, then overwrites them
      const int pj = nb * 16 + c, j = j0 + pj;
      f16x8 x[1][Ffn::KS];
#pragma unroll
      for (int ks = 0; ks < Ffn::KS; ++ks)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int ch = 32 * ks + 8 * g + e;
          _Float16 xv = (_Float16)0.f;
          if (j < Lk) {
            if (ch < H) xv = a.prev[((size_t)b * H + ch) * Lk + j];
            else if (ch < 2 * H) xv = f32_to_half_sat(a_s[(ch - H) * DEC_CK + pj]);
          }
          x[0][ks][e] = xv;
        }
      f32x4 y[1][(HB + 1) / 2];
      Ffn::template apply_lds_lean<1>(w_s, x, y);
#pragma unroll
      for (int hb = 0; hb < (HB + 1) / 2; ++hb)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int h = 16 * hb + 4 * g + v;
          if (h < H) a_s[h * DEC_CK + pj] = y[0][hb][v];
        }
    }
    __syncthreads();
  } else if (LISA_MODE == 1) {
    MfmaFfn<HB, FS, HB, ACT> ffn;
    ffn.fetch(w_s);
    const int c = lane & 15, g = lane >> 4;
#pragma unroll
    for (int q = 0; q < XNB; ++q) {
      const int nb = wv + 4 * q;
      const int pj = nb * 16 + c, j = j0 + pj;
      f16x8 x[1][MfmaFfn<HB, FS, HB, ACT>::KS];
#pragma unroll
      for (int ks = 0; ks < MfmaFfn<HB, FS, HB, ACT>::KS; ++ks)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int ch = 32 * ks + 8 * g + e;
          x[0][ks][e] = (ch < H && j < Lk) ? xpre[q][ks][e] : (_Float16)0.f;
        }
      f32x4 y[1][HB];
      ffn.template apply<1>(x, y);
#pragma unroll
      for (int hb = 0; hb < HB; ++hb)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int h = 16 * hb + 4 * g + v;
          if (h < H) a_s[h * DEC_CK + pj] += y[0][hb][v];
        }
    }
    __syncthreads();
  }

  // ---- S3: chunk softmax statistics, score row ------------------------------------------
  for (int h = wv; h < H; h += 4) {
    float* row = a_s + h * DEC_CK;
    const bool va = lane < n_here, vb = lane + 64 < n_here;
    const float sa = va ? row[lane] : -INFINITY, sb = vb ? row[lane + 64] : -INFINITY;
    if (a.row_out) {
      half_t* ro = a.row_out + ((size_t)b * H + h) * Lk + j0;
      if (va) ro[lane] = f32_to_half_sat(sa);
      if (vb) ro[lane + 64] = f32_to_half_sat(sb);
    }
    const float m = wave_max(fmaxf(sa, sb));
    const float pa = va ? __expf(sa - m) : 0.f, pb = vb ? __expf(sb - m) : 0.f;
    const float s = wave_sum(pa + pb);
    row[lane] = pa;
    row[lane + 64] = pb;
    if (lane == 0) {
      float* ml = a.part_ml + (((size_t)b * a.n_chunk + chunk) * H + h) * 2;
      ml[0] = m;
      ml[1] = s;
    }
  }
  __syncthreads();

  // ---- S4: partial O ---------------------------------------------------------------------
  {
    // The wave's heads and their batches of UN independent 16-byte loads form one sequence of
    // items; the loads of item i + 1 are issued before item i is consumed (two register sets), so
    // that a wave keeps loads in flight while it computes.  Keys past the end of the chunk are
    // clamped to its last key and carry probability 0 (set in S3), so no lane branches on
    // validity; the item after the last is clamped to the last (a load around a branch would make
    // the compiler wait for every earlier one).
    constexpr int NBATCH = V_NBATCH;
    const int js = v_js, dc = v_dc, n_items = v_items;
    float acc[8];
    auto consume = [&](int item, const u32x4 (&vv)[UN]) {
      const int h = wv + 4 * (item / NBATCH), bt = item % NBATCH, it = bt * UN;
      const float* p = a_s + h * DEC_CK;
      if (bt == 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = 0.f;
      }
#pragma unroll
      for (int u = 0; u < UN; ++u) {
        const float pj = p[js + (it + u) * KPW];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          acc[2 * e] += pj * bf16_bits_to_f32(vv[u][e] & 0xffffu);
          acc[2 * e + 1] += pj * bf16_bits_to_f32(vv[u][e] >> 16);
        }
      }
      if (bt == NBATCH - 1) {
#pragma unroll
        for (int e = 0; e < 8; ++e)
#pragma unroll
          for (int o = LPK; o < 64; o <<= 1) acc[e] += __shfl_xor(acc[e], o, 64);
        if (js == 0) {
          float* po = a.part_o + (((size_t)b * a.n_chunk + chunk) * H + h) * DK + dc * 8;
          *(float4*)po = make_float4(acc[0], acc[1], acc[2], acc[3]);
          *(float4*)(po + 4) = make_float4(acc[4], acc[5], acc[6], acc[7]);
        }
      }
    };
    u32x4 vb2[UN];
    if (n_items > 0) {
      for (int item = 0; item < n_items; item += 2) {
        v_issue(item + 1, vb2);
        consume(item, va);
        v_issue(item + 2, va);
        consume(item + 1, vb2);
      }
    }
  }
  // ---- the combine that the layer before left behind (stacks only) ----------------------------
  // Its (head, sequence) units are dealt to the workgroups of this launch, which take them when
  // their own work is done: a unit waits on a few loads from the L2 while the other workgroups
  // of the compute unit stream.  The partial results lie in the other half of the stack's
  // workspace; nothing of this layer depends on them.
  if (a.cmb_units > 0) {                                     // (uniform over the grid)
    const int n_wg = (int)(gridDim.x * gridDim.y);
    for (int unit = b * (int)gridDim.x + chunk; unit < a.cmb_units; unit += n_wg) {
      __syncthreads();                                       // dec_lds: done with as scores / by the unit before
      if (a.cmb_out_f32)
        decode_combine_unit<float, DK>(a.cmb_o, a.cmb_ml, (float*)a.cmb_out, a.cmb_H, a.cmb_nchunk, unit % a.cmb_H,
                                       unit / a.cmb_H, dec_lds);
      else
        decode_combine_unit<bf16_t, DK>(a.cmb_o, a.cmb_ml, (bf16_t*)a.cmb_out, a.cmb_H, a.cmb_nchunk,
                                        unit % a.cmb_H, unit / a.cmb_H, dec_lds);
    }
  }
}

}  // namespace lisa
