// Projection front end of a LiSA layer: Q_LR = X W^Q_LR, K_LR = X W^K_LR (the two factors of
// Eq. 3) and V = X W^V (Sec. 2.1 Eq. 1) as one product X W^T over the stacked weight rows, with
// the rotary position embedding of the LLaMA models (Sec. 5.3) applied to the Q_LR / K_LR heads
// before they are stored, and the results written where the attention kernels and the decode
// caches expect them.
//
// bf16 kernel (k_project_mfma): a workgroup of 8 waves owns a 256 x 256 (or 256 x 192) tile of the product and
// streams the reduction axis in steps of 64 through two LDS buffers, filled straight from global
// memory (global_load_lds_dwordx4), one barrier per step: the loads of step k+1 are issued during
// the first MFMAs of step k into the buffer that step k-1 used.  A CU fetches at most 64 bytes per clock from
// its vector memory path and its MFMAs eat 2 * 256 * 256 / (256 + 256) = 256 flops per fetched
// element at this tile size, twice what the fetch path must sustain; a 128 x 128 tile would run at
// that limit.  Wave (wm, wn) of the 2 x 4 arrangement owns 128 x 64 outputs = 4 x 2 blocks
// of the 32x32x16 MFMA (A = token rows, B = feature rows, so lane % 32 is the feature).
//
// The feature axis of the product is *virtual*: every Q_LR / K_LR head takes 32 columns, of
// which the first r are real (the others repeat a weight row and are dropped), so that one
// MFMA block is one head: the two partners of a rotary pair (t, t + r/2) sit in two lanes of
// the same accumulator register and one lane permute fetches the partner.  With r = 22 this
// spends 12 % more MFMA work on the LLaMA2-7B shape than the real columns need.
// LDS rows are 128 bytes (64 reduction elements); the 16-byte chunk c of row m is kept at
// chunk c ^ ((m / 2) % 8), which makes both the tile writes and the operand reads free of
// bank conflicts without padding.
#pragma once
#include "lisa_types.h"

namespace lisa {

struct ProjectArgs {
  const void* x;     // [B*L, D]
  const void* w;     // [H*r + Hkv*r + Hkv*dk, D]
  void* q_lr;        // [B,H,L,r]
  void* k_lr;        // [B,Hkv,Lmax,r] or [B,Hkv,r,Lmax]
  void* v;           // [B,Hkv,Lmax,dk]
  int B, L, D, H, Hkv, r, dk, Lmax, pos0, k_dim_major;
  int rope;          // 1: rotate Q_LR / K_LR
  double freq_log2;  // inverse frequency of pair t = 2^(t * freq_log2), freq_log2 = -2 log2(theta) / r
  int n_m, n_n, own_n;
};

// cos and sin of pos * inv_freq.  The angle (up to ~1e5 rad) is formed and reduced to
// [-pi, pi] in double; the float32 functions then work on a small argument.
__device__ __forceinline__ void rope_cos_sin(int pos, double inv_freq, float& c, float& s) {
  const double ang = (double)pos * inv_freq;
  const double k = rint(ang * 0.15915494309189535);        // 1 / (2 pi)
  double red = fma(-k, 6.283185307179586, ang);
  red = fma(-k, 2.4492935982947064e-16, red);              // low part of 2 pi
  const float rf = (float)red;
  s = sinf(rf);
  c = cosf(rf);
}
// The same through the hardware sine / cosine (argument in revolutions, absolute error near
// 1e-6): enough for results that are rounded to bfloat16.
__device__ __forceinline__ void rope_cos_sin_fast(int pos, double inv_freq_rev, float& c, float& s) {
  const double rev = (double)pos * inv_freq_rev;           // inv_freq_rev = inv_freq / (2 pi)
  const float fr = (float)(rev - rint(rev));
  s = __builtin_amdgcn_sinf(fr);
  c = __builtin_amdgcn_cosf(fr);
}

// Where output (token row m, feature n of the stacked weight) goes.  Returns the element index
// and selects the tensor through `which` (0 Q_LR, 1 K_LR, 2 V).
__device__ __forceinline__ size_t project_dest(const ProjectArgs& a, int b, int l, int head, int c,
                                               int& which) {
  const int pos = a.pos0 + l;
  if (head < a.H) {
    which = 0;
    return (((size_t)b * a.H + head) * a.L + l) * a.r + c;
  }
  if (head < a.H + a.Hkv) {
    which = 1;
    const int kv = head - a.H;
    return a.k_dim_major ? (((size_t)b * a.Hkv + kv) * a.r + c) * a.Lmax + pos
                         : (((size_t)b * a.Hkv + kv) * a.Lmax + pos) * a.r + c;
  }
  which = 2;
  const int kv = head - a.H - a.Hkv;
  return (((size_t)b * a.Hkv + kv) * a.Lmax + pos) * a.dk + c;
}

// ---- any dtype, any shape: one thread per output element -------------------------------
template <typename T, typename AccT>
__global__ __launch_bounds__(256) void k_project_generic(ProjectArgs a) {
  const int nqk = (a.H + a.Hkv) * a.r;
  const int N = nqk + a.Hkv * a.dk;
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (size_t)a.B * a.L * N) return;
  const int m = (int)(idx / N), f = (int)(idx % N);
  const int b = m / a.L, l = m % a.L;
  const T* xr = (const T*)a.x + (size_t)m * a.D;
  auto dot = [&](int row) {
    const T* wr = (const T*)a.w + (size_t)row * a.D;
    AccT acc = 0;
    for (int c = 0; c < a.D; ++c) acc += (AccT)elem<T>::load(xr + c) * (AccT)elem<T>::load(wr + c);
    return acc;
  };
  int head, c;
  float y;
  if (f < nqk) {
    head = f / a.r;
    c = f % a.r;
    const AccT own = dot(f);
    if (a.rope) {
      const int half = a.r / 2, t = c < half ? c : c - half;
      const AccT other = dot(c < half ? f + half : f - half);
      float cs, sn;
      rope_cos_sin(a.pos0 + l, exp2((double)t * a.freq_log2), cs, sn);
      y = c < half ? (float)(own * (AccT)cs - other * (AccT)sn) : (float)(other * (AccT)sn + own * (AccT)cs);
    } else {
      y = (float)own;
    }
  } else {
    head = a.H + a.Hkv + (f - nqk) / a.dk;
    c = (f - nqk) % a.dk;
    y = (float)dot(f);
  }
  int which;
  const size_t at = project_dest(a, b, l, head, c, which);
  elem<T>::store((T*)(which == 0 ? a.q_lr : which == 1 ? a.k_lr : a.v) + at, y);
}

// ---- bf16 on MFMA -----------------------------------------------------------------------
typedef __bf16 pj_bf16x8 __attribute__((ext_vector_type(8)));
typedef float pj_f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned pj_u32x4 __attribute__((ext_vector_type(4)));

constexpr int PJ_TK = 64;                       // reduction elements per step
constexpr int PJ_ROWB = PJ_TK * 2;              // bytes per LDS row

// Tile geometry: WM x WN waves (8 in all), each BM x BN blocks of 32 x 32 outputs.
//   <2,4,4,2>  256 x 256 outputs per workgroup, the densest in MFMA work per fetched byte;
//   <4,2,2,3>  256 x 192, for problems whose 256-wide tiles would leave a quarter of the CUs
//              idle or add a nearly empty last round of workgroups.
template <int WM, int WN, int BM, int BN>
struct ProjTile {
  static_assert(WM * WN == 8, "8 waves");
  static constexpr int TM = WM * BM * 32, TN = WN * BN * 32;
  static constexpr int XN = TM / 64, WNLD = TN / 64;      // 16-byte chunks per thread and step: X, W
  static constexpr int XTILE = TM * PJ_ROWB, WTILE = TN * PJ_ROWB;
  static constexpr int STEP = XTILE + WTILE;              // one step of both operands
  static constexpr int STG_ROW = BN * 64 + 16;            // bytes per row of a wave's output staging piece (padded)
  static constexpr int STG_WAVE = BM * 32 * STG_ROW;
  static constexpr int LDS = 2 * STEP > 8 * STG_WAVE ? 2 * STEP : 8 * STG_WAVE;
  static_assert(TM % 64 == 0 && TN % 64 == 0 && LDS <= 160 * 1024, "tile shape");
};
constexpr int PJ_HEADW = 32;                    // virtual columns of a Q_LR / K_LR head

// Scheduling request for one sub-step (`n_mfma` MFMAs, up to 6 LDS reads, up to 4 instructions of
// class `other`: 0x200 LDS writes, 0x020 global loads): the reads early (MFMA, two reads, three
// times: the next sub-step starts several MFMAs after the last of them), then MFMA, two others,
// twice, then the remaining MFMAs.
#define PJ_INTERLEAVE(other, n_mfma)                          \
  do {                                                        \
    _Pragma("unroll") for (int i_ = 0; i_ < 3; ++i_) {        \
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);      \
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);      \
    }                                                         \
    _Pragma("unroll") for (int i_ = 0; i_ < 2; ++i_) {        \
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);      \
      __builtin_amdgcn_sched_group_barrier(other, 2, 0);      \
    }                                                         \
    __builtin_amdgcn_sched_group_barrier(0x008, (n_mfma) - 5, 0); \
  } while (0)

// Barrier that publishes a tile loaded straight into the LDS: the wave's own loads have landed
// (vmcnt) and its LDS reads are done (lgkmcnt) before it arrives.
__device__ __forceinline__ void pj_tile_barrier() {
  __asm__ volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <int WM, int WN, int BM, int BN>
__global__ __launch_bounds__(512) void k_project_mfma(ProjectArgs a) {
  typedef ProjTile<WM, WN, BM, BN> G;
  extern __shared__ __align__(16) unsigned char pj_lds[];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int wm = wv / WN, wn = wv % WN;
  const int half = lane >> 5, l32 = lane & 31;

  // Workgroup ids go round robin over the 8 XCDs (each with its own L2): an XCD keeps to
  // its own tiles along one axis of the product so that operand tiles are shared in its L2.
  int tm, tn;
  {
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    if (a.own_n) {
      tn = xcd + 8 * (j / a.n_m);
      tm = j % a.n_m;
    } else {
      tm = xcd + 8 * (j / a.n_n);
      tn = j % a.n_n;
    }
    if (tm >= a.n_m || tn >= a.n_n) return;
  }
  const int M = a.B * a.L, D = a.D;
  const int nheads_qk = a.H + a.Hkv;
  const int nv_qk = PJ_HEADW * nheads_qk;                   // virtual columns before V
  const int n_real = nheads_qk * a.r + a.Hkv * a.dk;
  const int m0 = tm * G::TM, n0 = tn * G::TN;

  // loader: thread -> 16-byte chunk (row ld_row + 64 i, chunk ld_kc) of both operand tiles
  const int ld_row = tid >> 3, ld_kc = tid & 7;
  const int ld_gc = ld_kc ^ ((ld_row >> 1) & 7);           // chunk of the row that lands at LDS chunk ld_kc
  const bf16_t* xp[G::XN];
  const bf16_t* wp[G::WNLD];
#pragma unroll
  for (int i = 0; i < G::XN; ++i) {
    const int row = min(m0 + ld_row + 64 * i, M - 1);
    xp[i] = (const bf16_t*)a.x + (size_t)row * D + 8 * ld_gc;
  }
#pragma unroll
  for (int i = 0; i < G::WNLD; ++i) {
    const int nv = n0 + ld_row + 64 * i;
    int real;
    if (nv < nv_qk) {
      real = (nv >> 5) * a.r + min(nv & 31, a.r - 1);
    } else {
      real = nheads_qk * a.r + (nv - nv_qk);
    }
    wp[i] = (const bf16_t*)a.w + (size_t)min(real, n_real - 1) * D + 8 * ld_gc;
  }
  // The tiles go from global memory straight into the LDS (global_load_lds_dwordx4: lane l of a
  // wave writes its 16 bytes at the wave's LDS base + 16 l): one instruction of a wave fills 8
  // consecutive tile rows, so the swizzle is applied on the global side (lane -> which chunk of
  // the row it fetches).  No staging registers and no LDS write instructions in the loop.
  // The chunks of a step travel in two halves (part 0, part 1) spread over the first sub-steps.
  const int lds_wave = __builtin_amdgcn_readfirstlane(wv) * 8 * PJ_ROWB;   // first of the wave's 8 rows
  auto load_part = [&](int kt, int buf, int part) {
    unsigned char* base = pj_lds + buf * G::STEP + lds_wave;
#pragma unroll
    for (int i = part * (G::XN / 2); i < (part ? G::XN : G::XN / 2); ++i)
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)(xp[i] + (size_t)kt * PJ_TK),
          (__attribute__((address_space(3))) void*)(base + i * 64 * PJ_ROWB), 16, 0, 0);
#pragma unroll
    for (int i = part * (G::WNLD / 2); i < (part ? G::WNLD : G::WNLD / 2); ++i)
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)(wp[i] + (size_t)kt * PJ_TK),
          (__attribute__((address_space(3))) void*)(base + G::XTILE + i * 64 * PJ_ROWB), 16, 0, 0);
  };

  // operand reads: row (32 blk + l32), chunk 2 ks + half, swizzled by the row
  const int sw = (l32 >> 1) & 7;
  int rd_c[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) rd_c[ks] = ((2 * ks + half) ^ sw) << 4;
  const int rd_a = (wm * BM * 32 + l32) * PJ_ROWB;
  const int rd_b = G::XTILE + (wn * BN * 32 + l32) * PJ_ROWB;

  pj_f32x16 acc[BM][BN];
#pragma unroll
  for (int bm = 0; bm < BM; ++bm)
#pragma unroll
    for (int bn = 0; bn < BN; ++bn)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[bm][bn][v] = 0.f;

  // Operand registers are double buffered: the reads of sub-step ks + 1 are issued before
  // the MFMAs of sub-step ks, and the MFMAs of the last sub-step of a step run after the
  // barrier of the next one, behind its first operand reads and its tile writes, so the
  // matrix pipe has work while the LDS is busiest.
  pj_bf16x8 fa[2][BM], fb[2][BN];
  // (the W operands first: the first MFMAs of a sub-step need both of them and one X operand)
  auto read_frags = [&](const unsigned char* buf, int ks, int set) {
#pragma unroll
    for (int bn = 0; bn < BN; ++bn)
      fb[set][bn] = *(const pj_bf16x8*)(buf + rd_b + bn * 32 * PJ_ROWB + rd_c[ks]);
#pragma unroll
    for (int bm = 0; bm < BM; ++bm)
      fa[set][bm] = *(const pj_bf16x8*)(buf + rd_a + bm * 32 * PJ_ROWB + rd_c[ks]);
  };
  auto mfmas = [&](int set) {
#pragma unroll
    for (int bm = 0; bm < BM; ++bm)
#pragma unroll
      for (int bn = 0; bn < BN; ++bn)
        acc[bm][bn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][bm], fb[set][bn], acc[bm][bn], 0, 0, 0);
  };

  // Inside a step the MFMAs of a sub-step are interleaved one by one with the LDS reads of the
  // next sub-step, the LDS writes of the next tile and the global loads of the tile after it
  // (a wave issues in order: a block of 8 tile writes or 8 loads would leave the matrix pipe of
  // its SIMD idle, and both waves of a SIMD reach that block together).  The operand sets
  // start as zeros so that the deferred MFMAs of the first step add nothing.
#pragma unroll
  for (int bm = 0; bm < BM; ++bm)
#pragma unroll
    for (int e = 0; e < 8; ++e) fa[1][bm][e] = (__bf16)0.f;
#pragma unroll
  for (int bn = 0; bn < BN; ++bn)
#pragma unroll
    for (int e = 0; e < 8; ++e) fb[1][bn][e] = (__bf16)0.f;

  const int nk = D / PJ_TK;
  load_part(0, 0, 0);
  load_part(0, 0, 1);
  int kt = 0;
  for (; kt + 1 < nk; ++kt) {
    // the loads of step kt have landed in buffer kt & 1 and every wave has read all it needs of
    // the other buffer
    pj_tile_barrier();
    const unsigned char* buf = pj_lds + (kt & 1) * G::STEP;
    const int nb = (kt + 1) & 1;
    // sub-step 3 of step kt - 1 | operands of sub-step 0, first half of the loads of step kt + 1
    read_frags(buf, 0, 0);
    load_part(kt + 1, nb, 0);
    mfmas(1);
    PJ_INTERLEAVE(0x020, BM * BN);
    __builtin_amdgcn_sched_barrier(0);
    // sub-step 0 | operands of sub-step 1, second half of the loads
    read_frags(buf, 1, 1);
    load_part(kt + 1, nb, 1);
    mfmas(0);
    PJ_INTERLEAVE(0x020, BM * BN);
    __builtin_amdgcn_sched_barrier(0);
    // sub-step 1 | operands of sub-step 2
    read_frags(buf, 2, 0);
    mfmas(1);
    PJ_INTERLEAVE(0x020, BM * BN);
    __builtin_amdgcn_sched_barrier(0);
    // sub-step 2 | operands of sub-step 3
    read_frags(buf, 3, 1);
    mfmas(0);
    PJ_INTERLEAVE(0x020, BM * BN);
    __builtin_amdgcn_sched_barrier(0);
  }
  {                                                        // the last step: nothing left to load
    pj_tile_barrier();
    const unsigned char* buf = pj_lds + (kt & 1) * G::STEP;
    read_frags(buf, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    mfmas(1);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 0; ks < 3; ++ks) {
      read_frags(buf, ks + 1, (ks + 1) & 1);
      __builtin_amdgcn_sched_barrier(0);
      mfmas(ks & 1);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  mfmas(1);

  // Epilogue.  acc[bm][bn][v]: token row m0 + 128 wm + 32 bm + 8 (v/4) + 4 half + v%4, virtual
  // column n0 + 64 wn + 32 bn + l32 (for the <2,4,4,2> geometry).  Every wave rotates its Q_LR / K_LR blocks in registers
  // (the partner of a rotary pair is another lane of the same register), rounds to bfloat16 and
  // lays its 128 x 64 outputs out by rows in its own piece of the LDS, from where whole rows
  // go to memory: 128-byte pieces of V rows, the 2r-byte rows of Q_LR / K_LR (consecutive
  // tokens of a head are adjacent in memory), 64-byte runs along the tokens of a
  // dimension-major K_LR cache.
  __syncthreads();                                         // the operand tiles are dead: LDS becomes staging space
  unsigned char* stg = pj_lds + wv * G::STG_WAVE;
  const int mw = m0 + wm * (BM * 32);                            // first token row of the wave
  const int odd = lane & 1;
  // rotary embedding: the lane's frequency, partner lane and side of the pair are the same in
  // every block (they depend on lane % 32 only)
  const int nv_first = n0 + wn * (BN * 32);
  const bool rot_any = a.rope && nv_first < nv_qk;         // (blocks are ordered: Q_LR / K_LR heads first)
  const int hr = a.r >> 1;
  const bool lower = l32 < hr;
  double inv_freq_rev = 0.0;
  int partner = lane;
  float c1 = 1.f, s1 = 0.f, c8 = 1.f, s8 = 0.f;            // rotations by 1 and by 8 positions
  if (rot_any) {
    const int t = lower ? l32 : l32 - hr;
    inv_freq_rev = exp2((double)min(t, hr - 1) * a.freq_log2) * 0.15915494309189535;
    partner = (lane & 32) | (l32 < a.r ? (lower ? l32 + hr : l32 - hr) : l32);
    rope_cos_sin_fast(1, inv_freq_rev, c1, s1);
    rope_cos_sin_fast(8, inv_freq_rev, c8, s8);
  }
#pragma unroll
  for (int bm = 0; bm < BM; ++bm) {
    // cos / sin of the lane's 16 rows: row 8 j + i of the lane is position l0 + 8 j + i.  One exact
    // evaluation, then the angle-addition formulas (float32: the results are rounded to bfloat16);
    // a block that runs into the next sequence evaluates every row exactly.
    float cs[16], sn[16];
    if (rot_any) {
      const int mb = min(mw + bm * 32 + 4 * half, M - 1);
      const int l0 = mb - mb / a.L * a.L;
      if (l0 + 27 < a.L) {
        rope_cos_sin_fast(a.pos0 + l0, inv_freq_rev, cs[0], sn[0]);
#pragma unroll
        for (int jj = 1; jj < 4; ++jj) {
          cs[4 * jj] = cs[4 * jj - 4] * c8 - sn[4 * jj - 4] * s8;
          sn[4 * jj] = sn[4 * jj - 4] * c8 + cs[4 * jj - 4] * s8;
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          if ((v & 3) == 0) continue;
          cs[v] = cs[v - 1] * c1 - sn[v - 1] * s1;
          sn[v] = sn[v - 1] * c1 + cs[v - 1] * s1;
        }
      } else {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          int l = l0 + 8 * (v >> 2) + (v & 3);
          if (l >= a.L) l -= l / a.L * a.L;
          rope_cos_sin_fast(a.pos0 + l, inv_freq_rev, cs[v], sn[v]);
        }
      }
    }
#pragma unroll
    for (int bn = 0; bn < BN; ++bn) {
      const int nvb = nv_first + bn * 32;                  // first virtual column of the block (wave-uniform)
      const bool rot = a.rope && nvb < nv_qk;
#pragma unroll
      for (int v = 0; v < 16; v += 2) {
        float y[2] = {acc[bm][bn][v], acc[bm][bn][v + 1]};
        if (rot) {
#pragma unroll
          for (int e = 0; e < 2; ++e) {
            const float other = __shfl(y[e], partner, 64);
            y[e] = lower ? y[e] * cs[v + e] - other * sn[v + e] : other * sn[v + e] + y[e] * cs[v + e];
          }
        }
        // columns c, c + 1 of one row share a 32-bit word: the even lane assembles row v, the odd
        // lane row v + 1
        const unsigned u0 = f32_to_bf16_bits(y[0]), u1 = f32_to_bf16_bits(y[1]);
        const unsigned got = __shfl_xor(odd ? u0 : u1, 1, 64);
        const unsigned word = odd ? (got | (u1 << 16)) : (u0 | (got << 16));
        const int row = bm * 32 + 8 * (v >> 2) + 4 * half + (v & 3) + odd;
        *(unsigned*)(stg + row * G::STG_ROW + (bn * 32 + (l32 & ~1)) * 2) = word;
      }
    }
  }
  // (the staging piece is private to the wave: its own LDS accesses complete in order)
  int bw, lw;                                              // sequence and token index of row mw
  {
    const int mc = min(mw, M - 1);
    bw = mc / a.L;
    lw = mc - bw * a.L;
  }
  auto locate = [&](int row, int& b, int& l) {             // token row mw + row -> (sequence, token)
    b = bw;
    l = lw + row;
    if (l >= a.L) {
      const int q = l / a.L;
      b += q;
      l -= q * a.L;
    }
  };
  const int nvw = n0 + wn * (BN * 32);
  constexpr int WCOLS = BN * 32, WROWS = BM * 32, CH = WCOLS / 8;   // columns, rows, 16-byte chunks per row
  const int n_vcols = a.Hkv * a.dk;
  if (nvw >= nv_qk && (nvw - nv_qk) % a.dk + WCOLS <= a.dk) {
    // all blocks belong to one V head: whole pieces of rows (2 * WCOLS bytes)
    const int col = nvw - nv_qk;
    if (col < n_vcols) {
      const int kv = col / a.dk, cc = col - kv * a.dk;
#pragma unroll 4
      for (int idx = lane; idx < WROWS * CH; idx += 64) {
        const int row = idx / CH, ch = idx - row * CH;
        int b, l;
        locate(row, b, l);
        if (mw + row < M) {
          bf16_t* dst = (bf16_t*)a.v + (((size_t)b * a.Hkv + kv) * a.Lmax + a.pos0 + l) * a.dk + cc + 8 * ch;
          *(pj_u32x4*)dst = *(const pj_u32x4*)(stg + row * G::STG_ROW + ch * 16);
        }
      }
    }
  } else {
    for (int bn = 0; bn < BN; ++bn) {
      const int nvb = nvw + bn * 32;
      const unsigned char* sb = stg + bn * 64;
      if (nvb >= nv_qk) {
        // a V block on its own: 64-byte pieces of rows
        const int col = nvb - nv_qk;
        if (col >= n_vcols) continue;
        const int kv = col / a.dk, cc = col - kv * a.dk;
        for (int pass = 0; pass < WROWS / 16; ++pass) {
          const int row = pass * 16 + (lane >> 2), ch = lane & 3;
          int b, l;
          locate(row, b, l);
          if (mw + row < M) {
            bf16_t* dst = (bf16_t*)a.v + (((size_t)b * a.Hkv + kv) * a.Lmax + a.pos0 + l) * a.dk + cc + 8 * ch;
            *(pj_u32x4*)dst = *(const pj_u32x4*)(sb + row * G::STG_ROW + ch * 16);
          }
        }
        continue;
      }
      const int head = nvb >> 5;
      const bool is_q = head < a.H;
      const int hh = is_q ? head : head - a.H, nh = is_q ? a.H : a.Hkv;
      if (!is_q && a.k_dim_major) {
        // runs along the tokens: lane = (token of a 32-row block, parity of the feature)
        for (int bm = 0; bm < BM; ++bm) {
          const int row = bm * 32 + l32;
          int b, l;
          locate(row, b, l);
          if (mw + row >= M) continue;
          bf16_t* dst = (bf16_t*)a.k_lr + ((size_t)b * a.Hkv + hh) * a.r * a.Lmax + a.pos0 + l;
          for (int c = half; c < a.r; c += 2)
            dst[(size_t)c * a.Lmax].bits = *(const uint16_t*)(sb + row * G::STG_ROW + 2 * c);
        }
        continue;
      }
      // rows of r elements; 16 lanes per row, a 32-bit word (or, for odd r, an element) each
      bf16_t* base = (bf16_t*)(is_q ? a.q_lr : a.k_lr);
      const int lrow = is_q ? a.L : a.Lmax, p0 = is_q ? 0 : a.pos0;
      const int j = lane & 15;
      for (int pass = 0; pass < WROWS / 4; ++pass) {
        const int row = pass * 4 + (lane >> 4);
        int b, l;
        locate(row, b, l);
        if (mw + row >= M) continue;
        bf16_t* dst = base + (((size_t)b * nh + hh) * lrow + p0 + l) * a.r;
        if ((a.r & 1) == 0) {
          if (2 * j < a.r) *(unsigned*)(dst + 2 * j) = *(const unsigned*)(sb + row * G::STG_ROW + 4 * j);
        } else {
          for (int c = j; c < a.r; c += 16) dst[c].bits = *(const uint16_t*)(sb + row * G::STG_ROW + 2 * c);
        }
      }
    }
  }
}

// ---- bf16, few token rows (a decode step: one new token per sequence) ---------------------
// With M = B L <= 128 rows the product is bound by one pass over the weights (HBM), not by the
// matrix cores.  One workgroup = one block of 32 virtual columns (a Q_LR / K_LR head, or 32
// features of V) and all rows; its 8 waves split the reduction axis and stream their slices of
// the weight rows and of X straight into MFMA operand registers (no LDS: nothing is reused),
// then add their partial sums through the LDS (project_skinny_finish).
// The end of both skinny kernels: the partial sums of the 8 waves (their slices of the reduction
// axis) are added through the LDS, and every wave finishes 2 MB of the 16 MB result registers:
// rotation, rounding and element stores (with one wave per row block this tail took 5 us of
// the kernel's 19).  acc layout: token row 32 mb + 8 (v/4) + 4 half + v%4, virtual column nvb + l32.
template <int MB>
__device__ __forceinline__ void project_skinny_finish(const ProjectArgs a, const pj_f32x16 (&acc)[MB], float* red,
                                                      int nvb) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int half = lane >> 5, l32 = lane & 31;
  const int M = a.B * a.L;
  const int nheads_qk = a.H + a.Hkv;
  const int nv_qk = PJ_HEADW * nheads_qk;
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int v = 0; v < 16; ++v) red[((wv * MB + mb) * 16 + v) * 64 + lane] = acc[mb][v];
  __syncthreads();
  // the 16 MB registers (row block mb, register v) of the result are dealt to the 8 waves
  constexpr int PER = 2 * MB;
  float y[PER];
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int pi = wv * PER + i;                            // = 16 mb + v
    float sum = 0.f;
#pragma unroll
    for (int w = 0; w < 8; ++w) sum += red[(w * MB * 16 + pi) * 64 + lane];
    y[i] = sum;
  }
  int head, c;
  bool valid;
  if (nvb < nv_qk) {
    head = nvb >> 5;
    c = l32;
    valid = c < a.r;
  } else {
    const int col = nvb - nv_qk + l32;
    head = nheads_qk + col / a.dk;
    c = col % a.dk;
    valid = col < a.Hkv * a.dk;
  }
  const bool rot = a.rope && nvb < nv_qk;
  const int hr = a.r >> 1;
  const bool lower = c < hr;
  double inv_freq_rev = 0.0;
  int partner = lane;
  if (rot) {
    const int t = lower ? c : c - hr;
    inv_freq_rev = exp2((double)min(t, hr - 1) * a.freq_log2) * 0.15915494309189535;
    partner = (lane & 32) | (valid ? (lower ? c + hr : c - hr) : l32);
  }
  bf16_t* dst_base = (bf16_t*)(head < a.H ? a.q_lr : head < nheads_qk ? a.k_lr : a.v);
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int pi = wv * PER + i, mb = pi >> 4, v = pi & 15;
    const int m = mb * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
    const int mc = min(m, M - 1);
    const int b = mc / a.L, l = mc - b * a.L;
    float out = y[i];
    if (rot) {
      const float other = __shfl(out, partner, 64);
      float cs, sn;
      rope_cos_sin_fast(a.pos0 + l, inv_freq_rev, cs, sn);
      out = lower ? out * cs - other * sn : other * sn + out * cs;
    }
    if (valid && m < M) {
      int which;
      const size_t at = project_dest(a, b, l, head, c, which);
      dst_base[at].bits = (uint16_t)f32_to_bf16_bits(out);
    }
  }
}

template <int MB>
__global__ __launch_bounds__(512) void k_project_skinny(ProjectArgs a) {
  extern __shared__ __align__(16) unsigned char pj_lds[];
  float* red = (float*)pj_lds;                              // [8 waves][MB][16][64]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int half = lane >> 5, l32 = lane & 31;
  const int M = a.B * a.L, D = a.D;
  const int nheads_qk = a.H + a.Hkv;
  const int nv_qk = PJ_HEADW * nheads_qk;
  const int n_real = nheads_qk * a.r + a.Hkv * a.dk;
  const int nvb = blockIdx.x * 32;                          // first virtual column of the block
  int real;
  if (nvb < nv_qk) {
    real = (nvb >> 5) * a.r + min(l32, a.r - 1);
  } else {
    real = nheads_qk * a.r + (nvb - nv_qk) + l32;
  }
  const bf16_t* wrow = (const bf16_t*)a.w + (size_t)min(real, n_real - 1) * D + 8 * half;
  const bf16_t* xrow[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
    xrow[mb] = (const bf16_t*)a.x + (size_t)min(mb * 32 + l32, M - 1) * D + 8 * half;

  pj_f32x16 acc[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[mb][v] = 0.f;
  const int nsteps = D / 16, per = (nsteps + 7) / 8;
  const int s0 = wv * per, s1 = min(s0 + per, nsteps);
#pragma unroll 8
  for (int s = s0; s < s1; ++s) {
    const pj_bf16x8 bop = *(const pj_bf16x8*)(wrow + 16 * s);
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const pj_bf16x8 aop = *(const pj_bf16x8*)(xrow[mb] + 16 * s);
      acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop, bop, acc[mb], 0, 0, 0);
    }
  }
  project_skinny_finish<MB>(a, acc, red, nvb);
}

// The same product with both operands staged through the LDS.  Read straight into MFMA operand
// registers, a load touches 32 rows for 32 bytes each (the operand layout wants a lane per row):
// four requests per 128-byte line, for the weights and, from the L2, for X, which every workgroup
// reads whole.  Here a wave loads its slice of the reduction axis in chunks of 64 elements, 8 rows
// x 128 bytes per load (whole lines), writes them to its own LDS region (rows of 128 + 16 bytes:
// conflict-free 16-byte operand reads) and reads its operands from there; the next chunk's loads
// are in flight meanwhile.  No barrier in the loop: the region is private to the wave, and LDS
// operations of a wave execute in order.  Requires D % 512 == 0 (8 waves x whole chunks), MB <= 2
// (LDS: 8 waves x (1 + MB) x 4.5 KB).
constexpr int PJS_ROW = 128 + 16;                           // bytes per staged row (64 elements + pad)
template <int MB>
__global__ __launch_bounds__(512) void k_project_skinny_lds(ProjectArgs a) {
  extern __shared__ __align__(16) unsigned char pj_lds[];
  float* red = (float*)pj_lds;                              // after the loop: [8 waves][MB][16][64]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int half = lane >> 5, l32 = lane & 31;
  const int M = a.B * a.L, D = a.D;
  const int nheads_qk = a.H + a.Hkv;
  const int nv_qk = PJ_HEADW * nheads_qk;
  const int n_real = nheads_qk * a.r + a.Hkv * a.dk;
  const int nvb = blockIdx.x * 32;                          // first virtual column of the block
  constexpr int NX = 4 * MB;                                // X loads per chunk (8 rows each)
  unsigned char* wst = pj_lds + (size_t)wv * (1 + MB) * 32 * PJS_ROW;   // this wave's region: W rows, then X rows
  unsigned char* xst = wst + 32 * PJS_ROW;
  const int lrow = lane >> 3, lpiece = lane & 7;            // load: row lrow + 8 j, 16-byte piece lpiece
  // This wave's slice of the reduction axis, and the chunk it starts with, rotate with the
  // workgroup: rows are D elements apart (a multiple of the channel interleave), so workgroups
  // that walk the axis in step all load from the same few L2 / HBM channels at any one time
  // (a few percent on the LLaMA2-7B width).  The order of a sum does not matter to its parity bound.
  const int kslice = D / 8, k0 = ((wv + (int)blockIdx.x) & 7) * kslice;
  const int ch_rot = (int)(blockIdx.x >> 3);
  const bf16_t* wsrc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int n = lrow + 8 * j;
    const int real = nvb < nv_qk ? (nvb >> 5) * a.r + min(n, a.r - 1) : nheads_qk * a.r + (nvb - nv_qk) + n;
    wsrc[j] = (const bf16_t*)a.w + (size_t)min(real, n_real - 1) * D + k0 + 8 * lpiece;
  }
  const bf16_t* xsrc[NX];
#pragma unroll
  for (int j = 0; j < NX; ++j) xsrc[j] = (const bf16_t*)a.x + (size_t)min(lrow + 8 * j, M - 1) * D + k0 + 8 * lpiece;
  const int st_at = lrow * PJS_ROW + lpiece * 16;           // + 8 j rows
  const int op_at = l32 * PJS_ROW + half * 16;              // + 32 ks (+ 32 mb rows for X)

  pj_f32x16 acc[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[mb][v] = 0.f;
  // NPF chunks in flight per wave (12 KB each with two row blocks): at one, the loop ran at the
  // latency of a load per chunk.  The chunk count of a slice is rounded up to a multiple of NPF;
  // the chunks of the round-up enter the product with a zero weight operand.
  constexpr int NPF = 2;
  pj_u32x4 wr[NPF][4], xr[NPF][NX];
  const int n_chunks = kslice / 64;
  auto load_chunk = [&](int ch, int p) {                   // (beyond the slice: the first chunks again, no
    const int at = 64 * ((ch + ch_rot) % n_chunks);        //  branch around loads)
#pragma unroll
    for (int j = 0; j < 4; ++j) wr[p][j] = *(const pj_u32x4*)(wsrc[j] + at);
#pragma unroll
    for (int j = 0; j < NX; ++j) xr[p][j] = *(const pj_u32x4*)(xsrc[j] + at);
  };
#pragma unroll
  for (int p = 0; p < NPF; ++p) {                           // (in this order: the loop waits for the older set only)
    load_chunk(p, p);
    __builtin_amdgcn_sched_barrier(0);
  }
  for (int ch0 = 0; ch0 < n_chunks; ch0 += NPF) {
#pragma unroll
    for (int p = 0; p < NPF; ++p) {
      const int ch = ch0 + p;
#pragma unroll
      for (int j = 0; j < 4; ++j) *(pj_u32x4*)(wst + st_at + 8 * j * PJS_ROW) = wr[p][j];
#pragma unroll
      for (int j = 0; j < NX; ++j) *(pj_u32x4*)(xst + st_at + 8 * j * PJS_ROW) = xr[p][j];
      // (fences: left alone, the compiler issues these loads after the MFMAs and waits for them
      // before the next set is written, which leaves one chunk in flight)
      __builtin_amdgcn_sched_barrier(0);
      load_chunk(ch + NPF, p);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        pj_u32x4 braw = *(const pj_u32x4*)(wst + op_at + 32 * ks);
        if (ch >= n_chunks) braw = pj_u32x4{0u, 0u, 0u, 0u};      // (a chunk of the round-up: adds nothing)
        const pj_bf16x8 bop = __builtin_bit_cast(pj_bf16x8, braw);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
          const pj_bf16x8 aop = *(const pj_bf16x8*)(xst + op_at + mb * 32 * PJS_ROW + 32 * ks);
          acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop, bop, acc[mb], 0, 0, 0);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  __syncthreads();                                          // every wave is done with its staging region
  project_skinny_finish<MB>(a, acc, red, nvb);
}

}  // namespace lisa
