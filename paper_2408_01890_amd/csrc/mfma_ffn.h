// The head-alignment FFN of Sec. 5.1 on the matrix cores, for one block of 16 positions.
//
//   hid = ReLU(W1^T x),  y = W2^T hid,   x in R^H (scores of all heads at one position)
//
// Both products use the 16x16x32 MFMA with the *positions* as the N dimension, so the lane
// that owns position n after the first product owns it again as B operand of the second: the
// two products chain through registers with no shuffle.
//
// 16x16x32 MFMA operand layout (wave of 64 lanes, g = lane / 16, c = lane % 16):
//   A (M x K):  lane holds row m = c,  k = 8 g + e        (e = 0..7)
//   B (K x N):  lane holds col n = c,  k = 8 g + e
//   D (M x N):  lane holds col n = c,  rows m = 4 g + v    (v = 0..3)
// The contraction index may be numbered in any order as long as A and B agree.  For the
// second product it is numbered so that slot (k-step s, g, e) is hidden unit
//   f = 16 (2 s + e / 4) + 4 g + e % 4,
// which is exactly the D register v = e % 4 of f-block 2 s + e / 4 of the first product.
//
// Precision: both products run in half (11-bit significand) with float32 accumulation.  x
// arrives as half (the score type).  W1 and W2 are converted from bfloat16 to half once (exact
// for |w| >= 2^-14, absolute error < 2^-25 below).  The hidden units are rounded to half, not
// bfloat16: with an identity-like FFN they carry the scores themselves, and 8 significant bits
// there would move A_n by up to 2^-9 |A_n|, which the softmax turns into percent-level errors.
// ReLU and the saturation at the half range are one v_med3; SiLU costs an exp2 and a reciprocal.
#pragma once
#include "lisa_types.h"

namespace lisa {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ bf16x8 bf16x8_from_bits(u16x8 b) { return __builtin_bit_cast(bf16x8, b); }

__device__ __forceinline__ unsigned short half_bits(float f) {
  const _Float16 h = (_Float16)f;
  return __builtin_bit_cast(unsigned short, h);
}

// HB = ceil(H / 16) input head blocks (KS = ceil(H / 32) k-steps of the first product),
// FS = ceil(F / 32) hidden k-steps (2 FS hidden blocks of 16), HBO = blocks of 16 output heads
// (the caller may ask for a sub-range of the H output heads: h_first .. h_first + n_out - 1).
// ACT: activation of the hidden units, 0 = ReLU (Sec. 5.3), 1 = SiLU u * sigmoid(u) (ablated in
// Sec. 5.7); both saturate at the half range.
template <int HB, int FS, int HBO = HB, int ACT = 0>
struct MfmaFfn {
  static constexpr int KS = (HB + 1) / 2;
  static constexpr int FB = 2 * FS;

  static __device__ __forceinline__ _Float16 activate(float u) {
    if (ACT == 0) return (_Float16)__builtin_amdgcn_fmed3f(u, 0.f, 65504.f);
    // exp2(-u log2 e) overflows to +inf for very negative u: 1 / inf = 0 and the product is -0
    const float sg = __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * u));
    return (_Float16)fminf(u * sg, 65504.f);
  }
  f16x8 w1[FB][KS];   // A operands of the first product:  W1^T, rows f, contraction c
  f16x8 w2[HBO][FS];  // A operands of the second product: W2^T, rows h, contraction f

  // Bytes of LDS that stage() fills.
  static constexpr int kStageBytes = (FB * KS + HBO * FS) * 64 * 16;

  // All `nthreads` threads of the workgroup convert the weights (w1g [H][F], w2g [F][H],
  // bfloat16, global memory) once into `lds` in operand order (operand o, lane l -> 16 bytes at
  // (o * 64 + l) * 16); after a barrier every wave fetches its registers with fetch().
  __device__ __forceinline__ static void stage(const bf16_t* __restrict__ w1g,
                                               const bf16_t* __restrict__ w2g, int H, int F,
                                               unsigned short* lds, int tid, int nthreads,
                                               int h_first = 0, int n_out = 1 << 30, int h_total = -1) {
    // h_total: number of output heads (columns of w2g) when it differs from the input width H
    const int HO = h_total < 0 ? H : h_total;
    for (int idx = tid; idx < FB * KS * 512; idx += nthreads) {
      const int e = idx & 7, l = (idx >> 3) & 63, o = idx >> 9;
      const int fb = o / KS, ks = o % KS, c = l & 15, g = l >> 4;
      const int f = 16 * fb + c, ch = 32 * ks + 8 * g + e;
      const float w = (f < F && ch < H) ? elem<bf16_t>::load(w1g + (size_t)ch * F + f) : 0.f;
      lds[idx] = half_bits(w);
    }
    unsigned short* lds2 = lds + FB * KS * 512;
    for (int idx = tid; idx < HBO * FS * 512; idx += nthreads) {
      const int e = idx & 7, l = (idx >> 3) & 63, o = idx >> 9;
      const int hb = o / FS, s = o % FS, c = l & 15, g = l >> 4;
      const int hl = 16 * hb + c, h = h_first + hl, f = 16 * (2 * s + e / 4) + 4 * g + e % 4;
      const float w = (f < F && h < HO && hl < n_out) ? elem<bf16_t>::load(w2g + (size_t)f * HO + h) : 0.f;
      lds2[idx] = half_bits(w);
    }
  }

  __device__ __forceinline__ void fetch(const unsigned short* lds) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int fb = 0; fb < FB; ++fb)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        w1[fb][ks] = *(const f16x8*)(lds + ((fb * KS + ks) * 64 + lane) * 8);
    const unsigned short* lds2 = lds + FB * KS * 512;
#pragma unroll
    for (int hb = 0; hb < HBO; ++hb)
#pragma unroll
      for (int s = 0; s < FS; ++s)
        w2[hb][s] = *(const f16x8*)(lds2 + ((hb * FS + s) * 64 + lane) * 8);
  }

  // apply() with the weight operands read from the staged LDS image as the products need them
  // (no weight registers held by the caller).
  // skip_last: the last block of 16 hidden units is all padding (F <= 32 FS - 16, e.g.
  // the 40 -> 80 -> 40 network of the LLaMA2-13B shape): its products are left out, its hidden
  // units are the activation of zero, which is zero for both activations.
  template <int NBLK, bool skip_last = false>
  __device__ __forceinline__ static void apply_lds(const unsigned short* lds, const f16x8 (&x)[NBLK][KS],
                                                   f32x4 (&y)[NBLK][HBO]) {
    const int lane = threadIdx.x & 63;
    const unsigned short* l1 = lds + lane * 8;
    const unsigned short* l2 = l1 + FB * KS * 512;
    f16x8 hid[NBLK][FS];
#pragma unroll
    for (int s = 0; s < FS; ++s) {
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        f32x4 acc[NBLK];
#pragma unroll
        for (int n = 0; n < NBLK; ++n) acc[n] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (!(s == FS - 1 && half == 1 && skip_last)) {
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) {
            const f16x8 w = *(const f16x8*)(l1 + ((2 * s + half) * KS + ks) * 512);
#pragma unroll
            for (int n = 0; n < NBLK; ++n)
              acc[n] = __builtin_amdgcn_mfma_f32_16x16x32_f16(w, x[n][ks], acc[n], 0, 0, 0);
          }
        }
#pragma unroll
        for (int n = 0; n < NBLK; ++n)
#pragma unroll
          for (int v = 0; v < 4; ++v)
            hid[n][s][4 * half + v] = activate(acc[n][v]);
      }
    }
#pragma unroll
    for (int hb = 0; hb < HBO; ++hb) {
      f32x4 acc[NBLK];
#pragma unroll
      for (int n = 0; n < NBLK; ++n) acc[n] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < FS; ++s) {
        const f16x8 w = *(const f16x8*)(l2 + (hb * FS + s) * 512);
#pragma unroll
        for (int n = 0; n < NBLK; ++n)
          acc[n] = __builtin_amdgcn_mfma_f32_16x16x32_f16(w, hid[n][s], acc[n], 0, 0, 0);
      }
#pragma unroll
      for (int n = 0; n < NBLK; ++n) y[n][hb] = acc[n];
    }
  }

  // apply_lds() for wide networks (many weight operands): the weight operands of the next groups
  // of products are read while the current group runs, and scheduling fences between the groups
  // keep the compiler from hoisting all weight reads to the top, which would need more registers
  // than a wave has.
  template <int NBLK>
  __device__ __forceinline__ static void apply_lds_lean(const unsigned short* lds, const f16x8 (&x)[NBLK][KS],
                                                        f32x4 (&y)[NBLK][HBO]) {
    const int lane = threadIdx.x & 63;
    const unsigned short* l1 = lds + lane * 8;
    const unsigned short* l2 = l1 + FB * KS * 512;
    f16x8 hid[NBLK][FS];
    constexpr int PD = 3;                                   // groups of weight operands in flight
    f16x8 wq[PD][KS];
#pragma unroll
    for (int p = 0; p < PD; ++p)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        if (p < FB) wq[p][ks] = *(const f16x8*)(l1 + (p * KS + ks) * 512);
#pragma unroll
    for (int fb = 0; fb < FB; ++fb) {                       // hidden block fb = 2 s + half
      f16x8 w[KS];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) w[ks] = wq[fb % PD][ks];
      if (fb + PD < FB) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) wq[fb % PD][ks] = *(const f16x8*)(l1 + ((fb + PD) * KS + ks) * 512);
      }
      f32x4 acc[NBLK];
#pragma unroll
      for (int n = 0; n < NBLK; ++n) acc[n] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int n = 0; n < NBLK; ++n)
          acc[n] = __builtin_amdgcn_mfma_f32_16x16x32_f16(w[ks], x[n][ks], acc[n], 0, 0, 0);
#pragma unroll
      for (int n = 0; n < NBLK; ++n)
#pragma unroll
        for (int v = 0; v < 4; ++v) hid[n][fb >> 1][4 * (fb & 1) + v] = activate(acc[n][v]);
      __builtin_amdgcn_sched_barrier(0);
    }
    constexpr int N2 = HBO * FS, PD2 = 4;
    f16x8 vq[PD2];
#pragma unroll
    for (int p = 0; p < PD2; ++p)
      if (p < N2) vq[p] = *(const f16x8*)(l2 + p * 512);
#pragma unroll
    for (int hb = 0; hb < HBO; ++hb) {
      f32x4 acc[NBLK];
#pragma unroll
      for (int n = 0; n < NBLK; ++n) acc[n] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < FS; ++s) {
        const int o = hb * FS + s;
        const f16x8 w = vq[o % PD2];
        if (o + PD2 < N2) vq[o % PD2] = *(const f16x8*)(l2 + (o + PD2) * 512);
#pragma unroll
        for (int n = 0; n < NBLK; ++n)
          acc[n] = __builtin_amdgcn_mfma_f32_16x16x32_f16(w, hid[n][s], acc[n], 0, 0, 0);
        if ((s & 1) == 1) __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int n = 0; n < NBLK; ++n) y[n][hb] = acc[n];
    }
  }

  // The same network with the hidden units taken SC k-steps (32 SC units) at a time: the second
  // product is linear in the hidden units, so their chunks are folded into its accumulators one
  // after the other and only one chunk is alive.  That leaves registers for more blocks per call,
  // and every weight operand is read from LDS once per call: with all blocks of a wave in one
  // call the weight traffic, which is what a wide FFN costs, is the least possible.
  // `between(gi)` is called at the head of MFMA group gi = 0 .. (FS / SC) (2 SC + HBO) - 1 (a group =
  // the MFMAs of one hidden block, or of one output block and chunk): the caller's memory operations
  // placed there run in the shadow of the matrix cores.
  template <int NBLK, int SC, class Between>
  __device__ __forceinline__ static void apply_lds_chunked(const unsigned short* lds,
                                                           const f16x8 (&x)[NBLK][KS], f32x4 (&y)[NBLK][HBO],
                                                           Between&& between) {
    static_assert(FS % SC == 0, "chunk size");
    constexpr int GPC = 2 * SC + HBO;                       // groups per chunk
    const int lane = threadIdx.x & 63;
    const unsigned short* l1 = lds + lane * 8;
    const unsigned short* l2 = l1 + FB * KS * 512;
#pragma unroll
    for (int n = 0; n < NBLK; ++n)
#pragma unroll
      for (int hb = 0; hb < HBO; ++hb) y[n][hb] = f32x4{0.f, 0.f, 0.f, 0.f};
    // the operands of a group of MFMAs are read while the group before it runs
    f16x8 wa[2][KS], wb[2][SC];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) wa[0][ks] = *(const f16x8*)(l1 + ks * 512);
#pragma unroll
    for (int s0 = 0; s0 < FS; s0 += SC) {
      f16x8 hid[NBLK][SC];
#pragma unroll
      for (int fb = 2 * s0; fb < 2 * (s0 + SC); ++fb) {     // hidden block fb = 2 s + half
        between((s0 / SC) * GPC + fb - 2 * s0);
        if (fb + 1 < 2 * (s0 + SC)) {
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) wa[(fb + 1) & 1][ks] = *(const f16x8*)(l1 + ((fb + 1) * KS + ks) * 512);
        } else {
#pragma unroll
          for (int s = 0; s < SC; ++s) wb[0][s] = *(const f16x8*)(l2 + (s0 + s) * 512);
        }
        f32x4 acc[NBLK];
#pragma unroll
        for (int n = 0; n < NBLK; ++n) acc[n] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
          for (int n = 0; n < NBLK; ++n)
            acc[n] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wa[fb & 1][ks], x[n][ks], acc[n], 0, 0, 0);
#pragma unroll
        for (int n = 0; n < NBLK; ++n)
#pragma unroll
          for (int v = 0; v < 4; ++v) hid[n][(fb >> 1) - s0][4 * (fb & 1) + v] = activate(acc[n][v]);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int hb = 0; hb < HBO; ++hb) {
        between((s0 / SC) * GPC + 2 * SC + hb);
        if (hb + 1 < HBO) {
#pragma unroll
          for (int s = 0; s < SC; ++s) wb[(hb + 1) & 1][s] = *(const f16x8*)(l2 + ((hb + 1) * FS + s0 + s) * 512);
        } else if (s0 + SC < FS) {
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) wa[0][ks] = *(const f16x8*)(l1 + (2 * (s0 + SC) * KS + ks) * 512);
        }
#pragma unroll
        for (int s = 0; s < SC; ++s)
#pragma unroll
          for (int n = 0; n < NBLK; ++n)
            y[n][hb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wb[hb & 1][s], hid[n][s], y[n][hb], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }

  // apply_lds_chunked() with the weight operands of a group read two groups ahead, into three
  // rotating operand sets: with eight waves reading at once an operand takes longer to arrive than
  // the 64 - 128 cycles of one group of MFMAs.
  template <int NBLK, int SC, class Between>
  __device__ __forceinline__ static void apply_lds_chunked_ahead(const unsigned short* lds,
                                                                 const f16x8 (&x)[NBLK][KS],
                                                                 f32x4 (&y)[NBLK][HBO], Between&& between) {
    static_assert(FS % SC == 0, "chunk size");
    constexpr int GPC = 2 * SC + HBO;                       // groups per chunk
    constexpr int NGR = (FS / SC) * GPC;
    constexpr int MAXOP = KS > SC ? KS : SC;
    constexpr int AH = 2, NBUF = AH + 1;                     // groups ahead, operand sets
    const int lane = threadIdx.x & 63;
    const unsigned short* l1 = lds + lane * 8;
    const unsigned short* l2 = l1 + FB * KS * 512;
#pragma unroll
    for (int n = 0; n < NBLK; ++n)
#pragma unroll
      for (int hb = 0; hb < HBO; ++hb) y[n][hb] = f32x4{0.f, 0.f, 0.f, 0.f};
    f16x8 w[NBUF][MAXOP];
    auto read_ops = [&](int gi) {                           // the operands of group gi
      const int s0 = (gi / GPC) * SC, idx = gi % GPC;
      if (idx < 2 * SC) {
        const int fb = 2 * s0 + idx;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) w[gi % NBUF][ks] = *(const f16x8*)(l1 + (fb * KS + ks) * 512);
      } else {
        const int hb = idx - 2 * SC;
#pragma unroll
        for (int s = 0; s < SC; ++s) w[gi % NBUF][s] = *(const f16x8*)(l2 + (hb * FS + s0 + s) * 512);
      }
    };
#pragma unroll
    for (int gi = 0; gi < AH && gi < NGR; ++gi) read_ops(gi);
    f16x8 hid[NBLK][SC];
#pragma unroll
    for (int gi = 0; gi < NGR; ++gi) {
      const int s0 = (gi / GPC) * SC, idx = gi % GPC;
      between(gi);
      if (gi + AH < NGR) read_ops(gi + AH);
      if (idx < 2 * SC) {                                   // hidden block fb = 2 s + half
        const int fb = 2 * s0 + idx;
        f32x4 acc[NBLK];
#pragma unroll
        for (int n = 0; n < NBLK; ++n) acc[n] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
          for (int n = 0; n < NBLK; ++n)
            acc[n] = __builtin_amdgcn_mfma_f32_16x16x32_f16(w[gi % NBUF][ks], x[n][ks], acc[n], 0, 0, 0);
#pragma unroll
        for (int n = 0; n < NBLK; ++n)
#pragma unroll
          for (int v = 0; v < 4; ++v) hid[n][(fb >> 1) - s0][4 * (fb & 1) + v] = activate(acc[n][v]);
      } else {
        const int hb = idx - 2 * SC;
#pragma unroll
        for (int s = 0; s < SC; ++s)
#pragma unroll
          for (int n = 0; n < NBLK; ++n)
            y[n][hb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(w[gi % NBUF][s], hid[n][s], y[n][hb], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  // NBLK independent blocks of 16 positions at once: the MFMAs of the blocks are interleaved so
  // that none has to wait for the result of the one issued just before it.
  // x[n][ks]: B operand of the first product of block n: lane (c, g) holds x[head 32 ks + 8 g + e]
  // of its position (zero for heads >= H).  y[n][hb][v] = FFN output of head h_first + 16 hb + 4 g + v.
  template <int NBLK>
  __device__ __forceinline__ void apply(const f16x8 (&x)[NBLK][KS], f32x4 (&y)[NBLK][HBO]) const {
    f16x8 hid[NBLK][FS];
#pragma unroll
    for (int s = 0; s < FS; ++s) {
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        f32x4 acc[NBLK];
#pragma unroll
        for (int n = 0; n < NBLK; ++n) acc[n] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
          for (int n = 0; n < NBLK; ++n)
            acc[n] = __builtin_amdgcn_mfma_f32_16x16x32_f16(w1[2 * s + half][ks], x[n][ks], acc[n], 0, 0, 0);
#pragma unroll
        for (int n = 0; n < NBLK; ++n)
#pragma unroll
          for (int v = 0; v < 4; ++v)
            hid[n][s][4 * half + v] = activate(acc[n][v]);
      }
    }
#pragma unroll
    for (int hb = 0; hb < HBO; ++hb) {
      f32x4 acc[NBLK];
#pragma unroll
      for (int n = 0; n < NBLK; ++n) acc[n] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < FS; ++s)
#pragma unroll
        for (int n = 0; n < NBLK; ++n)
          acc[n] = __builtin_amdgcn_mfma_f32_16x16x32_f16(w2[hb][s], hid[n][s], acc[n], 0, 0, 0);
#pragma unroll
      for (int n = 0; n < NBLK; ++n) y[n][hb] = acc[n];
    }
  }
};

}  // namespace lisa
