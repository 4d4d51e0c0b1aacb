// Fused LiSA prefill layer on the matrix cores (bf16 inputs, half scores, float32 softmax).
//
// One workgroup owns 16 query rows of one sequence and a group of GH = NW * HPW heads (NW waves,
// HPW heads per wave).  The alignment FFN couples the heads of a position (Sec. 5.1), while
// softmax and P V are per head (Sec. 2.1 Eq. 1-2), so the waves split the work two ways and swap
// roles inside every tile of 32 keys:
//   stage A (by position): the 32 blocks of 16 positions (one query row, 16 consecutive keys)
//           are dealt to the waves; a wave reads A_{n-1} of ALL heads for its block and runs the
//           FFN on MFMA (mfma_ffn.h), producing y = FFN(A_{n-1}) for the GH heads of the group;
//           y goes to LDS as float32, indexed [head][row][key].
//   stage B (by head): wave w owns heads w*HPW .. w*HPW+HPW-1 of the group.  Per head: low-rank
//           scores A_delta = K_LR Q_LR^T (Eq. 3) by MFMA, A_n = y + A_delta (Eq. 4), half store of
//           A_n for the next layer, online softmax in float32, O^T += V^T P^T by MFMA.
// A_n never leaves registers between the FFN and the softmax.  With more than one head group
// per row block (grid.z > 1) the first FFN layer is recomputed by every group; that buys
// parallelism and registers (the float32 output accumulators of 16 rows x GH heads x 128 must
// fit the register file of one compute unit).
//
// Layout of the per-head products (16x16x32 MFMA, lane = 16 g + c):
//   scores  D[key, row] = sum_t K_LR[key,t] Q_LR[row,t]: A = K_LR (rows = keys), B = Q_LR^T.
//           Two MFMAs cover 32 keys; MFMA u in {0,1} takes keys 8 (m/4) + 4 u + m % 4 for its
//           rows m, so that lane (c = row, g) ends with the 8 consecutive keys 8 g .. 8 g + 7.
//   output  D[d, row] = sum_key V^T[d,key] P^T[key,row]: A = V^T (16 features), B = P^T; the
//           lane's 8 probabilities are exactly its B operand (k = 8 g + e), no data movement.
//   Both leave "row" on the lane index c, where the softmax statistics of that row live.
//
// Inputs are repacked once per call into the workspace: Q_LR and K_LR rows zero-padded from r to
// 32 elements (64-byte rows, aligned 16-byte operand loads) and V regrouped as
// [B,Hkv,Lkp/8,d_k,8] (8 consecutive keys of one feature = one 16-byte load, the 128 features of
// a key chunk contiguous, so the 8 feature blocks of a lane differ by an immediate offset).
//
// Software pipeline of one workgroup (tile t = 32 keys):
//   top of tile t : the A_{n-1} tile t is already in LDS (xs); barrier B1
//   stage A(t)    : reads xs, writes ys; barrier B2
//   stage B(t)    : first writes the A_{n-1} tile t+1 (in registers since stage B(t-1)) into xs and
//                   issues the global loads of tile t+2; then, head by head, consumes the K_LR / V
//                   operand registers and immediately refills them with the operands of the next
//                   head (or of the first head of tile t+1), so every operand load has one head of
//                   work to hide its latency.
#pragma once
#include "kernels_generic.h"
#include "mfma_ffn.h"

namespace lisa {

constexpr int PF_ROWS = 16;       // query rows per workgroup
constexpr int PF_TK = 32;         // keys per tile
constexpr int PF_XS_HEAD = PF_ROWS * PF_TK * 2 + 32;        // bytes per head of the A_{n-1} tile
constexpr int PF_YS_ROW = PF_TK * 4 + 16;                   // bytes per (head,row) of the y tile
constexpr int PF_YS_HEAD = PF_ROWS * PF_YS_ROW + 16;

typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef unsigned int pf_u32x4 __attribute__((ext_vector_type(4)));

struct PrefillArgs {
  const bf16_t* qp;       // [B,H,Lqp,32]       Q_LR padded (Lqp = Lq rounded up to 16)
  const bf16_t* kp;       // [B,Hkv,Lkp,32]     K_LR padded (Lkp = Lk rounded up to 64)
  const bf16_t* vt;       // [B,Hkv,Lkp/8,128,8] V by key chunks
  const half_t* prev;     // [B,H,Lq,Lk]
  const bf16_t* w1;
  const bf16_t* w2;
  half_t* scores;         // [B,H,Lq,Lk] or null
  void* out;              // [B,Lq,H,128] float32 or bf16
  int H, Hkv, Lq, Lk, Lqp, Lkp, F, causal, out_f32;
  float dscale;
  int split;              // key-range splits per row block (1: the kernel writes `out` itself)
  float* part_o;          // [split][B][Lqp][H][128] unnormalised partial outputs (split > 1)
  float* part_ml;         // [split][B][Lqp][H][2]   running maximum, partial sum
};

// Grid-stride, block 256: zero-pads the Q_LR / K_LR rows from r to 32 elements.
__global__ void k_pack_prefill(const bf16_t* __restrict__ q_lr, const bf16_t* __restrict__ k_lr,
                               bf16_t* __restrict__ qp, bf16_t* __restrict__ kp, int B, int H, int Hkv,
                               int Lq, int Lk, int Lqp, int Lkp, int r) {
  const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t nth = (size_t)gridDim.x * blockDim.x;
  const size_t nq = (size_t)B * H * Lqp * 32, nk = (size_t)B * Hkv * Lkp * 32;
  bf16_t z;
  z.bits = 0;
  for (size_t e = tid; e < nq; e += nth) {
    const int t = e & 31;
    const size_t row = e >> 5;
    const int i = row % Lqp;
    const size_t bh = row / Lqp;
    qp[e] = (t < r && i < Lq) ? q_lr[(bh * Lq + i) * r + t] : z;
  }
  for (size_t e = tid; e < nk; e += nth) {
    const int t = e & 31;
    const size_t row = e >> 5;
    const int j = row % Lkp;
    const size_t bh = row / Lkp;
    kp[e] = (t < r && j < Lk) ? k_lr[(bh * Lk + j) * r + t] : z;
  }
}

// vt[bh][j / 8][d][j % 8] = v[bh][j][d] through a 64 x 64 LDS tile (zero for j >= Lk).
// grid (Lkp / 64, dk / 64, B * Hkv), block 256.
__global__ __launch_bounds__(256) void k_regroup_v(const bf16_t* __restrict__ v, bf16_t* __restrict__ vt,
                                                   int Lk, int Lkp, int dk) {
  __shared__ unsigned short tile[64][66];
  const int j0 = blockIdx.x * 64, d0 = blockIdx.y * 64;
  const size_t bh = blockIdx.z;
  for (int idx = threadIdx.x; idx < 64 * 64; idx += 256) {
    const int jl = idx >> 6, dl = idx & 63;
    tile[jl][dl] = (j0 + jl < Lk) ? v[(bh * Lk + j0 + jl) * dk + d0 + dl].bits : (unsigned short)0;
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < 64 * 64; idx += 256) {
    const int e = idx & 7, dl = (idx >> 3) & 63, jc = idx >> 9;
    vt[((bh * (Lkp / 8) + j0 / 8 + jc) * dk + d0 + dl) * 8 + e].bits = tile[8 * jc + e][dl];
  }
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every global
// load and store in flight (workgroup-scope fence), which would drain the operand prefetch of
// the pipeline at every tile; the tiles exchange data through LDS alone.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Butterflies across the four 16-lane rows of a wave with the row-swap instructions of gfx950
// (no LDS crossbar): after both steps every lane 16 g + c holds the reduction over g.
__device__ __forceinline__ float rows_max(float v) {
  const unsigned u = __float_as_uint(v);
  auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);   // rows (0,1) and (2,3) exchanged
  v = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
  const unsigned w = __float_as_uint(v);
  auto q = __builtin_amdgcn_permlane32_swap(w, w, false, false);   // halves exchanged
  return fmaxf(__uint_as_float(q[0]), __uint_as_float(q[1]));
}
__device__ __forceinline__ float rows_sum(float v) {
  const unsigned u = __float_as_uint(v);
  auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  v = __uint_as_float(r[0]) + __uint_as_float(r[1]);
  const unsigned w = __float_as_uint(v);
  auto q = __builtin_amdgcn_permlane32_swap(w, w, false, false);
  return __uint_as_float(q[0]) + __uint_as_float(q[1]);
}

// H = NG * NW * HPW heads in NG groups; NW waves per workgroup, HPW heads per wave; FS hidden
// k-steps of the FFN.  grid (Lqp / 16, B, NG), block NW * 64.  Requires Lk % 8 == 0.
template <int NG, int FS, int HPW, int NW>
__global__ __launch_bounds__(NW * 64) void k_lisa_prefill_fused(PrefillArgs a) {
  constexpr int DK = 128;
  constexpr int THREADS = NW * 64;
  constexpr int GH = NW * HPW;                       // heads of this workgroup's group
  constexpr int H = NG * GH;
  constexpr int HB = (H + 15) / 16;
  constexpr int HBO = (GH + 15) / 16;
  typedef MfmaFfn<HB, FS, HBO> Ffn;
  constexpr int KS = Ffn::KS;
  constexpr int XCH = (H * 64 + THREADS - 1) / THREADS;   // 16-byte chunks of a tile per thread
  constexpr int NBW = ((2 * PF_ROWS + NW - 1) / NW + 1) / 2 * 2;   // position blocks per wave in stage A (even)
  extern __shared__ __align__(16) unsigned char pf_lds[];
  const int Lq = a.Lq, Lk = a.Lk;
  unsigned char* xs = pf_lds;                               // A_{n-1} tile, half
  unsigned char* ys = xs + H * PF_XS_HEAD;                  // y tile of the group, float
  unsigned short* w_s = (unsigned short*)(ys + GH * PF_YS_HEAD);
  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform
  const int c = lane & 15, g = lane >> 4;
  const int b = blockIdx.y;
  const int hg0 = blockIdx.z * GH;                          // first head of the group
  const int unit = gridDim.x - 1 - blockIdx.x;              // long row blocks first
  const int rb = unit / a.split, sp = unit % a.split;       // row block, key-range split
  const int i0 = rb * PF_ROWS;
  const int shift = Lk - Lq;                                // key j visible to row i iff j <= i + shift
  const int group = H / a.Hkv;
  const float LOG2E = 1.4426950408889634f;

  const int i_last = min(i0 + PF_ROWS - 1, Lq - 1);
  const int n_keys = a.causal ? min(Lk, i_last + 1 + shift) : Lk;
  const int n_tiles_all = (n_keys + PF_TK - 1) / PF_TK;
  // this workgroup's share of the key tiles (identical formula in k_prefill_combine)
  const int per_split = (n_tiles_all + a.split - 1) / a.split;
  const int t_begin = sp * per_split;
  const int n_tiles = min(n_tiles_all, t_begin + per_split);   // one past my last tile
  if (t_begin >= n_tiles) return;                            // empty share (short row block)
  // tiles whose 32 keys are visible to all 16 rows (and all 16 rows exist) need no masking
  const int n_full = (i0 + PF_ROWS <= Lq) ? (a.causal ? min(Lk, i0 + 1 + shift) : Lk) / PF_TK : 0;

  Ffn::stage(a.w1, a.w2, H, a.F, w_s, tid, THREADS, hg0, GH);

  // ---- A_{n-1} tile: thread -> XCH chunks (head, row, 8 keys) of 16 bytes ------------------------
  const half_t* xsrc[XCH];       // row start of each chunk's (head, row)
  int xq4[XCH], xdst[XCH];
#pragma unroll
  for (int u = 0; u < XCH; ++u) {
    const int e = tid + u * THREADS;
    const int q4 = e & 3, i = (e >> 2) & 15, h = min(e >> 6, H - 1);
    xsrc[u] = a.prev + (((size_t)b * H + h) * Lq + min(i0 + i, Lq - 1)) * Lk;
    xq4[u] = 8 * q4;
    xdst[u] = (e >> 6) < H ? h * PF_XS_HEAD + i * 64 + q4 * 16 : -1;
  }
  auto load_x = [&](int tile, pf_u32x4 (&xr)[XCH]) {
#pragma unroll
    for (int u = 0; u < XCH; ++u) {
      // keys >= Lk: any in-bounds chunk will do, those positions are masked in stage B
      const int jc = min(tile * PF_TK + xq4[u], Lk - 8);
      xr[u] = *(const pf_u32x4*)(xsrc[u] + jc);
    }
  };
  auto store_x = [&](unsigned char* xs, const pf_u32x4 (&xr)[XCH]) {
#pragma unroll
    for (int u = 0; u < XCH; ++u)
      if (H * 64 % THREADS == 0 || xdst[u] >= 0) *(pf_u32x4*)(xs + xdst[u]) = xr[u];
  };

  // ---- per-head state of stage B ------------------------------------------------------------------
  const int my_row = min(i0 + c, Lq - 1);                   // clamped for loads; stores check i0 + c
  const int vis_row = a.causal ? min(Lk, my_row + 1 + shift) : Lk;   // keys visible to my row
  f32x4 o[HPW][DK / 16];
  float m_run[HPW], l_run[HPW];
  const bf16_t* kbase[HPW];      // K_LR operand rows of this lane, tile 0
  const bf16_t* vbase[HPW];      // V operand chunk of this lane, tile 0
  const bf16_t* qrow[HPW];
  half_t* srow[HPW];             // A_n row of this lane (key 8 g of tile 0)
  const int h_first = hg0 + wv * HPW;
#pragma unroll
  for (int hh = 0; hh < HPW; ++hh) {
    const int h = h_first + hh, kv = h / group;
    m_run[hh] = -INFINITY;
    l_run[hh] = 0.f;
#pragma unroll
    for (int nb = 0; nb < DK / 16; ++nb) o[hh][nb] = f32x4{0.f, 0.f, 0.f, 0.f};
    kbase[hh] = a.kp + (((size_t)b * a.Hkv + kv) * a.Lkp + 8 * (c >> 2) + (c & 3)) * 32 + 8 * g;   // tile 0
    vbase[hh] = a.vt + ((((size_t)b * a.Hkv + kv) * (a.Lkp / 8) + g) * DK + c) * 8;
    qrow[hh] = a.qp + (((size_t)b * H + h) * a.Lqp + i0 + c) * 32 + 8 * g;
    srow[hh] = a.scores ? a.scores + (((size_t)b * H + h) * Lq + my_row) * Lk + 8 * g : nullptr;
  }
  // operand registers of the head that stage B handles next, refilled right after use (keeping
  // a set per head would give each load a whole tile period but does not fit the register file)
  bf16x8 qop, ka, kb, vop[DK / 16];
  qop = *(const bf16x8*)qrow[0];
  {
    const bf16_t* kp0 = kbase[0] + (size_t)t_begin * (PF_TK * 32);
    ka = *(const bf16x8*)kp0;
    kb = *(const bf16x8*)(kp0 + 4 * 32);
    const bf16_t* vp0 = vbase[0] + (size_t)t_begin * (PF_TK / 8 * DK * 8);
#pragma unroll
    for (int nb = 0; nb < DK / 16; ++nb) vop[nb] = *(const bf16x8*)(vp0 + nb * 128);
  }

  // A_{n-1} tile t+1 travels in xr for one whole tile period: loaded at the start of stage B(t-1),
  // written to LDS at the start of stage B(t)
  pf_u32x4 xr[XCH];
  load_x(t_begin, xr);
  store_x(xs, xr);
  load_x(min(t_begin + 1, n_tiles - 1), xr);

  // LDS addresses of stage A (per lane, tile independent)
  int xrd[KS][2];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    // transposing LDS read: lane s = 4 k' + q4 of a 16-lane group passes the address of head k',
    // keys 4 q4 .. 4 q4 + 3; it receives key c of heads k' = 0..3.
    xrd[ks][0] = min(32 * ks + 8 * g + (c >> 2), H - 1) * PF_XS_HEAD + 8 * (c & 3);
    xrd[ks][1] = min(32 * ks + 8 * g + 4 + (c >> 2), H - 1) * PF_XS_HEAD + 8 * (c & 3);
  }

  for (int tile = t_begin; tile < n_tiles; ++tile) {
    const int j0 = tile * PF_TK;
    lds_barrier();                                                       // B1
    {
      // ---- stage A: y = FFN(A_{n-1}) for this wave's blocks of 16 positions --------------------
      // the FFN weights live in registers during stage A only (stage B needs the registers for
      // the output accumulators and the operand prefetch)
      Ffn ffn;
      ffn.fetch(w_s);
      // two blocks of 16 positions at a time, their MFMA chains interleaved
#pragma unroll
      for (int q = 0; q < NBW; q += 2) {
        f16x8 x[2][KS];
        int yoff[2];
#pragma unroll
        for (int n = 0; n < 2; ++n) {
          // block = (row i, key half kh); a wave with an odd share repeats its last block
          const int nb = min(wv + (q + n) * NW, 2 * PF_ROWS - 1);
          const int i = nb >> 1, kh = nb & 1;
          yoff[n] = i * PF_YS_ROW + (16 * kh + c) * 4;
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) {
            const f16x4 lo = __builtin_bit_cast(
                f16x4, __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                           (s16x4 __attribute__((address_space(3)))*)(xs + xrd[ks][0] + i * 64 + 32 * kh)));
            const f16x4 hi = __builtin_bit_cast(
                f16x4, __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                           (s16x4 __attribute__((address_space(3)))*)(xs + xrd[ks][1] + i * 64 + 32 * kh)));
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              if (H % 32 == 0) {
                x[n][ks][e] = lo[e];
                x[n][ks][4 + e] = hi[e];
              } else {
                x[n][ks][e] = 32 * ks + 8 * g + e < H ? lo[e] : (_Float16)0.f;
                x[n][ks][4 + e] = 32 * ks + 8 * g + 4 + e < H ? hi[e] : (_Float16)0.f;
              }
            }
          }
        }
        f32x4 y[2][HBO];
        ffn.template apply<2>(x, y);
#pragma unroll
        for (int n = 0; n < 2; ++n)
#pragma unroll
          for (int hb = 0; hb < HBO; ++hb)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              const int hl = 16 * hb + 4 * g + v;
              if (GH % 16 == 0 || hl < GH) *(float*)(ys + hl * PF_YS_HEAD + yoff[n]) = y[n][hb][v];
            }
      }
    }
    lds_barrier();                                                       // B2

    // ---- stage B: per head scores, softmax, P V ------------------------------------------------
    const int tile_n = min(tile + 1, n_tiles - 1);            // next tile (clamped: loads stay valid)
    // every wave left stage A(tile), the last reader of xs, before B2; stage A(tile+1) reads the
    // new tile after B1
    store_x(xs, xr);
    load_x(min(tile + 2, n_tiles - 1), xr);
    const bool full = tile < n_full;                          // workgroup-uniform
    const int jl = j0 + 8 * g;                                // first of my 8 keys
#pragma unroll
    for (int hh = 0; hh < HPW; ++hh) {
      const int hn = hh + 1 < HPW ? hh + 1 : 0;
      const int t_next = hh + 1 < HPW ? tile : tile_n;
      // low-rank scores for keys j0 + 8 g + e of row c
      const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
      const f32x4 s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, qop, zero, 0, 0, 0);
      const f32x4 s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kb, qop, zero, 0, 0, 0);
      {
        qop = *(const bf16x8*)qrow[hn];
        const bf16_t* kpn = kbase[hn] + (size_t)t_next * (PF_TK * 32);
        ka = *(const bf16x8*)kpn;
        kb = *(const bf16x8*)(kpn + 4 * 32);
      }
      const float* yp = (const float*)(ys + (wv * HPW + hh) * PF_YS_HEAD + c * PF_YS_ROW + 8 * g * 4);
      const f32x4 y0 = *(const f32x4*)yp, y1 = *(const f32x4*)(yp + 4);
      float an[8];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        an[e] = s0[e] * a.dscale + y0[e];
        an[4 + e] = s1[e] * a.dscale + y1[e];
      }
      f16x8 hv;                                 // A_n for the next layer, stored after the MFMAs
#pragma unroll
      for (int e = 0; e < 8; ++e) hv[e] = f32_to_half_sat(an[e]);
      // online softmax, statistics of row c kept by all four lanes 16 g + c; exponentials in
      // base 2: p = 2^(A log2(e) - m log2(e))
      if (!full) {                              // workgroup-uniform: only diagonal / ragged tiles mask
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (jl + e >= vis_row) an[e] = -INFINITY;
      }
      float mx = fmaxf(fmaxf(fmaxf(an[0], an[1]), fmaxf(an[2], an[3])),
                       fmaxf(fmaxf(an[4], an[5]), fmaxf(an[6], an[7])));
      mx = rows_max(mx);
      const float m_new = fmaxf(m_run[hh], mx);
      // every row sees key 0, so m_new is finite from the first tile on
      const float m2 = m_new * LOG2E;
      const float alpha = fast_exp2(m_run[hh] * LOG2E - m2);
      m_run[hh] = m_new;
      float ps = 0.f;
      bf16x8 pop;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float p = fast_exp2(__builtin_fmaf(an[e], LOG2E, -m2));
        ps += p;
        pop[e] = (__bf16)p;                     // hardware round-to-nearest-even conversion
      }
      l_run[hh] = l_run[hh] * alpha + ps;       // partial sum over my keys; groups merged at the end
      if (__any(alpha != 1.f)) {                // wave-uniform: the running maximum rarely moves
#pragma unroll
        for (int nb = 0; nb < DK / 16; ++nb)
#pragma unroll
          for (int v = 0; v < 4; ++v) o[hh][nb][v] *= alpha;
      }
      const bf16_t* vpn = vbase[hn] + (size_t)t_next * (PF_TK / 8 * DK * 8);
#pragma unroll
      for (int nb = 0; nb < DK / 16; ++nb) {
        o[hh][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop[nb], pop, o[hh][nb], 0, 0, 0);
        vop[nb] = *(const bf16x8*)(vpn + nb * 128);
      }
      // stores share the in-order memory counter with loads: issued last, no operand load of
      // this head has to wait behind them
      if (a.scores) {
        half_t* sp = srow[hh] + j0;
        if (full) {
          *(f16x8*)sp = hv;
        } else if (i0 + c < Lq) {
          if (jl + 8 <= vis_row) {
            *(f16x8*)sp = hv;
          } else {
#pragma unroll
            for (int e = 0; e < 8; ++e)
              if (jl + e < vis_row) sp[e] = hv[e];
          }
        }
      }
    }
  }

  // ---- epilogue ----------------------------------------------------------------------------------
  if (a.split > 1) {
    // unnormalised partial (o, m, l) of this key range; k_prefill_combine merges the ranges
#pragma unroll
    for (int hh = 0; hh < HPW; ++hh) {
      const int h = h_first + hh;
      const float l = rows_sum(l_run[hh]);
      const size_t row = (((size_t)sp * gridDim.y + b) * a.Lqp + i0 + c) * H + h;
      if (g == 0) {
        a.part_ml[row * 2] = m_run[hh];
        a.part_ml[row * 2 + 1] = l;
      }
#pragma unroll
      for (int nb = 0; nb < DK / 16; ++nb) {
        const f32x4 acc = o[hh][nb];
        *(float4*)(a.part_o + row * DK + nb * 16 + 4 * g) = make_float4(acc[0], acc[1], acc[2], acc[3]);
      }
    }
    return;
  }
  // O[row][h][d] = o / l
#pragma unroll
  for (int hh = 0; hh < HPW; ++hh) {
    const int h = h_first + hh;
    const float inv = 1.f / rows_sum(l_run[hh]);
    if (i0 + c < Lq) {
      const size_t at = (((size_t)b * Lq + i0 + c) * H + h) * DK + 4 * g;
#pragma unroll
      for (int nb = 0; nb < DK / 16; ++nb) {
        const f32x4 acc = o[hh][nb];
        if (a.out_f32) {
          *(float4*)((float*)a.out + at + nb * 16) =
              make_float4(acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv);
        } else {
          uint2 pk;
          pk.x = f32_to_bf16_bits(acc[0] * inv) | (f32_to_bf16_bits(acc[1] * inv) << 16);
          pk.y = f32_to_bf16_bits(acc[2] * inv) | (f32_to_bf16_bits(acc[3] * inv) << 16);
          *(uint2*)((bf16_t*)a.out + at + nb * 16) = pk;
        }
      }
    }
  }
}

// Merges the key-range partials of k_lisa_prefill_fused: for every (b, row, h)
//   O = sum_s e^{m_s - M} o_s / sum_s e^{m_s - M} l_s,   M = max_s m_s   over the non-empty ranges.
// grid (Lq, B), block 256; thread -> (head, 4 features) pairs.
__global__ __launch_bounds__(256) void k_prefill_combine(PrefillArgs a) {
  constexpr int DK = 128;
  const int i = blockIdx.x, b = blockIdx.y, H = a.H;
  const int rb = i / PF_ROWS;
  const int i_last = min(rb * PF_ROWS + PF_ROWS - 1, a.Lq - 1);
  const int n_keys = a.causal ? min(a.Lk, i_last + 1 + a.Lk - a.Lq) : a.Lk;
  const int n_tiles_all = (n_keys + PF_TK - 1) / PF_TK;
  const int per_split = (n_tiles_all + a.split - 1) / a.split;
  const int n_used = (n_tiles_all + per_split - 1) / per_split;       // non-empty ranges
  for (int e = threadIdx.x; e < H * (DK / 4); e += 256) {
    const int h = e / (DK / 4), d4 = e % (DK / 4);
    float M = -INFINITY;
    for (int s = 0; s < n_used; ++s)
      M = fmaxf(M, a.part_ml[((((size_t)s * gridDim.y + b) * a.Lqp + i) * H + h) * 2]);
    float den = 0.f;
    float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int s = 0; s < n_used; ++s) {
      const size_t row = (((size_t)s * gridDim.y + b) * a.Lqp + i) * H + h;
      const float w = __expf(a.part_ml[row * 2] - M);
      den += w * a.part_ml[row * 2 + 1];
      const float4 po = *(const float4*)(a.part_o + row * DK + 4 * d4);
      num.x += w * po.x;
      num.y += w * po.y;
      num.z += w * po.z;
      num.w += w * po.w;
    }
    const float inv = 1.f / den;
    const size_t at = (((size_t)b * a.Lq + i) * H + h) * DK + 4 * d4;
    if (a.out_f32) {
      *(float4*)((float*)a.out + at) = make_float4(num.x * inv, num.y * inv, num.z * inv, num.w * inv);
    } else {
      uint2 pk;
      pk.x = f32_to_bf16_bits(num.x * inv) | (f32_to_bf16_bits(num.y * inv) << 16);
      pk.y = f32_to_bf16_bits(num.z * inv) | (f32_to_bf16_bits(num.w * inv) << 16);
      *(uint2*)((bf16_t*)a.out + at) = pk;
    }
  }
}

}  // namespace lisa
