// A_n of a LiSA layer in CONCAT form on the matrix cores (bf16 inputs, half scores):
//   A_n[:,i,j] = W2^T ReLU(W1^T [A_{n-1}[:,i,j] ; A_delta[:,i,j]])      (Sec. 5.1, "An overview of
// LiSA": the alignment FFN takes the concatenation, 2h -> F -> h; Sec. 5.3: 64 -> 256 -> 32),
// with A_delta = Q_LR K_LR^T / sqrt(r) (Eq. 3).  The correction goes through the FFN here, so it
// cannot be added per head after a position-wise stage as in the fused ADD kernel; this kernel
// produces the score tensor (half), which the next layer shares and which the softmax / P V
// kernel that follows reads.  49 kflop per position at the paper's widths against 2 + 2 bytes per
// head and position.
//
// One workgroup (8 waves) works on tiles of 16 query rows x 32 keys, a run of them (see the
// kernel).  Per tile:
//   1. the A_{n-1} tile of all heads goes to LDS ([head][row][key], half); wave w computes the
//      A_delta tile of heads w, w + 8, ... with two 16x16x32 MFMAs each (A = K_LR rows, B = Q_LR
//      rows, both read from copies zero-padded to 32 elements per row: k_prepare_prefill) and
//      appends it as heads H .. 2H-1 of the same LDS array;
//   2. every wave runs the FFN (mfma_ffn.h, weights read from their LDS image) on 4 of the 32
//      blocks of 16 positions, the 2H input "heads" fetched with transposing LDS reads;
//   3. the results go to LDS [head][row][key] and leave by heads in whole rows, 64 bytes of half
//      per row and tile: up to 32 heads as half in an array of their own, stored during the FFN of
//      the next tile (two barriers per tile); wider forms as float32 over the input tile, stored
//      before the next tile is staged (four barriers).
// Requires Lk % 8 == 0, r <= 32, H <= 48, F <= 256.
#pragma once
#include <type_traits>
#include "kernels_prefill.h"

namespace lisa {

struct ScoresMfmaArgs {
  const bf16_t* qp;     // [B,H,Lqp,32]   Q_LR rows zero-padded to 32 elements
  const bf16_t* kp;     // [B,Hkv,Lkp,32] K_LR rows likewise
  const half_t* prev;   // [B,H,Lq,Lk] (or tiled, see below)
  const bf16_t* w1;     // [2H,F]
  const bf16_t* w2;     // [F,H]
  half_t* scores;       // [B,H,Lq,Lk]: A_n, which the softmax kernel that follows reads as well
  int B, H, Hkv, Lq, Lk, Lqp, Lkp, F, causal;
  int tiled;            // prev and scores are [B,ceil(Lq/16),ceil(Lk/32),H,16,32] (TILED kernels only)
  long long tiles_b;    // tiles of one batch element: sum over the row groups of scores_mfma_tiles()
  float dscale;
};

constexpr int SM_YS_ROW = PF_TK * 4;                    // bytes per (head,row) of the output tile (float32)
// bytes per head: 16 more than its rows, so that the four heads 4 apart that the lane groups of a
// wave write at once fall into different banks (the tile still fits under the input tile, 2 x 1056
// bytes per head)
constexpr int SM_YS_HEAD = PF_ROWS * SM_YS_ROW + 16;
// the output tile as half in an array of its own (up to 32 heads, see the kernel), padded likewise
constexpr int SM_YH_HEAD = PF_ROWS * PF_TK * 2 + 16;

// Key tiles (PF_TK keys) that hold visible keys of row group rg (PF_ROWS query rows).
__host__ __device__ inline int scores_mfma_tiles(int rg, int Lq, int Lk, int causal) {
  const int i_last = min(rg * PF_ROWS + PF_ROWS - 1, Lq - 1);
  const int n_keys = causal ? min(Lk, i_last + 1 + (Lk - Lq)) : Lk;
  return (n_keys + PF_TK - 1) / PF_TK;
}

// HBI = ceil(2H / 16) input blocks, FS = ceil(F / 32), HBO = ceil(H / 16), ACT: 0 ReLU, 1 SiLU.
// grid (G), block 512, one workgroup per compute unit: the tiles of the causal triangle, in the
// order (batch, row group, key tile), are cut into G equal runs, so that every workgroup has the
// same number of tiles whatever the shape of the triangle (whole row groups or chunks of them
// leave the last workgroups of a grid with up to twice the average), and stages the weights once.
// TILED (up to 32 heads): A_{n-1} and A_n in the tiled score layout, where the tile of a head is one
// contiguous KB (whole lines instead of 16 half lines) and leaves without a visibility test: the
// entries above the diagonal of a tile are unspecified there.
template <int HBI, int FS, int HBO, int ACT = 0, bool TILED = false>
__global__ __launch_bounds__(512) void k_lisa_scores_mfma(ScoresMfmaArgs a) {
  static_assert(!TILED || HBI <= 4, "tiled scores: the pipelined form only");
  typedef MfmaFfn<HBI, FS, HBO, ACT> Ffn;
  constexpr int KS = Ffn::KS, NW = 8, NBW = 4;
  // hidden k-steps alive at a time in the FFN call (4 blocks x SC x 4 registers; two only where
  // the register file has room)
  constexpr int SC = (HBI >= 4 || FS % 2 != 0) ? 1 : 2;
  extern __shared__ __align__(16) unsigned char sm_lds[];
  const int H = a.H, Din = 2 * H, Lq = a.Lq, Lk = a.Lk;
  // PIPE (up to 32 heads, where the LDS has room): the output tile (H heads, half) has an array of
  // its own and leaves during the FFN of the next tile.  Otherwise it takes the place of the input
  // tile (2H heads, half) as float32 and leaves before the next tile is staged.
  constexpr bool PIPE = HBI <= 4;
  const int io_bytes = PIPE ? Din * PF_XS_HEAD + H * SM_YH_HEAD : max(Din * PF_XS_HEAD, H * SM_YS_HEAD);
  unsigned char* xs = sm_lds;
  unsigned char* ys = sm_lds;
  unsigned char* yh = sm_lds + Din * PF_XS_HEAD;
  unsigned short* w_s = (unsigned short*)(sm_lds + ((io_bytes + 15) & ~15));
  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int c = lane & 15, g = lane >> 4;
  const int shift = Lk - Lq;
  const int group = H / a.Hkv;
  const int n_rg = (Lq + PF_ROWS - 1) / PF_ROWS;
  // this workgroup's run of tiles [pos, hi) and where it starts
  const long long total = a.tiles_b * a.B;
  long long pos = total * blockIdx.x / gridDim.x;
  const long long hi = total * (blockIdx.x + 1) / gridDim.x;
  if (pos >= hi) return;
  int b = (int)(pos / a.tiles_b), rg = 0;
  int tile0 = (int)(pos - b * a.tiles_b);
  for (int nt; tile0 >= (nt = scores_mfma_tiles(rg, Lq, Lk, a.causal)); ++rg) tile0 -= nt;

  Ffn::stage(a.w1, a.w2, Din, a.F, w_s, tid, NW * 64, 0, H, H);

  // transposing LDS reads of stage 2 (see the fused prefill kernel): lane 4 k' + q4 of a 16-lane
  // group passes the address of head k', keys 4 q4 .. 4 q4 + 3, and receives key c of heads k' = 0..3
  int xrd[KS][2];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    xrd[ks][0] = min(32 * ks + 8 * g + (c >> 2), Din - 1) * PF_XS_HEAD + 8 * (c & 3);
    xrd[ks][1] = min(32 * ks + 8 * g + 4 + (c >> 2), Din - 1) * PF_XS_HEAD + 8 * (c & 3);
  }
  while (pos < hi) {
  // ---- one row group: tiles [t_first, t_last) of its key tiles -----------------------------------
  const int i0 = rg * PF_ROWS;
  const int t_first = tile0;
  const int t_last = (int)min((long long)scores_mfma_tiles(rg, Lq, Lk, a.causal), tile0 + (hi - pos));
  // A_delta: B operands (Q_LR rows of this wave's heads), resident
  constexpr int HPW = (HBO * 16 + NW - 1) / NW;             // heads per wave (upper bound)
  bf16x8 qop[HPW];
#pragma unroll
  for (int u = 0; u < HPW; ++u) {
    const int h = min(wv + NW * u, H - 1);
    qop[u] = *(const bf16x8*)(a.qp + (((size_t)b * H + h) * a.Lqp + min(i0 + c, Lq - 1)) * 32 + 8 * g);
  }
  const int x_row = min(i0 + (lane >> 2), Lq - 1), xq8 = 8 * (lane & 3);

  // The operands of a tile (this wave's share of the A_{n-1} tile and its K_LR rows) are loaded
  // into registers one tile ahead, during the FFN of the tile before.
  constexpr int XCH = (HBO * 16 + NW - 1) / NW;             // A_{n-1} chunks (heads) per wave
  pf_u32x4 xr[XCH];
  bf16x8 kop[HPW][2];
  // tiled layout: tile (rg, t) of head h at ((b n_rg + rg) n_kt + t) H + h KB, a lane's 16 bytes at
  // 16 lane (row lane / 4, keys 8 (lane % 4) .. + 7: the same share as in the row-major form)
  const int n_kt = (Lk + PF_TK - 1) / PF_TK;
  const size_t tile_stride = (size_t)H * (PF_ROWS * PF_TK);
  const size_t trow = ((size_t)b * n_rg + rg) * n_kt * tile_stride + lane * 8;   // + t tile_stride + h 512
  auto prefetch = [&](int tile) {
    const int j0 = tile * PF_TK;
#pragma unroll
    for (int u = 0; u < XCH; ++u) {
      const int h = min(wv + NW * u, H - 1);
      if (TILED)
        xr[u] = *(const pf_u32x4*)(a.prev + trow + min(tile, n_kt - 1) * tile_stride + h * (PF_ROWS * PF_TK));
      else
        xr[u] = *(const pf_u32x4*)(a.prev + (((size_t)b * H + h) * Lq + x_row) * Lk + min(j0 + xq8, Lk - 8));
    }
#pragma unroll
    for (int u = 0; u < HPW; ++u) {
      const int h = min(wv + NW * u, H - 1);
      const bf16_t* kbase = a.kp + ((size_t)b * a.Hkv + h / group) * a.Lkp * 32 + 8 * g;
#pragma unroll
      for (int half = 0; half < 2; ++half)
        kop[u][half] = *(const bf16x8*)(kbase + (size_t)min(j0 + 16 * half + c, Lk - 1) * 32);
    }
  };
  prefetch(t_first);
  // (the barriers of the tile loop order LDS traffic only: __syncthreads() would also wait for the
  // global stores of the previous tile and for the prefetch)

  auto stage_tile = [&]() {
#pragma unroll
    for (int u = 0; u < XCH; ++u) {
      const int h = wv + NW * u;
      if (h < H) *(pf_u32x4*)(xs + h * PF_XS_HEAD + lane * 16) = xr[u];
    }
#pragma unroll
    for (int u = 0; u < HPW; ++u) {
      const int h = wv + NW * u;
      if (h >= H) break;
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        f32x4 d = {0.f, 0.f, 0.f, 0.f};
        d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop[u][half], qop[u], d, 0, 0, 0);
        // d[v] = A_delta(row c, key 16 half + 4 g + v) / scale
        f16x4 hv;
#pragma unroll
        for (int v = 0; v < 4; ++v) hv[v] = f32_to_half_sat(d[v] * a.dscale);
        *(f16x4*)(xs + (H + h) * PF_XS_HEAD + c * 64 + (16 * half + 4 * g) * 2) = hv;
      }
    }
  };
  auto read_x = [&](f16x8 (&x)[NBW][KS], bool x_all) {     // x_all: 2H fills the k-steps, nothing to zero
#pragma unroll
    for (int n = 0; n < NBW; ++n) {
      const int nb = wv + n * NW;                           // block = (row nb / 2, key half nb % 2)
      const int i = nb >> 1, kh = nb & 1;
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
          x[n][ks][e] = (x_all || 32 * ks + 8 * g + e < Din) ? lo[e] : (_Float16)0.f;
          x[n][ks][4 + e] = (x_all || 32 * ks + 8 * g + 4 + e < Din) ? hi[e] : (_Float16)0.f;
        }
      }
    }
  };

  if constexpr (PIPE) {
    // Two barriers per tile.  Between A and B: the FFN of tile t, and in the shadow of its MFMA
    // groups the loads of tile t + 1 and the stores of A_n of tile t - 1 (from yh).  Between B and
    // A: tile t + 1 goes into xs and the result of tile t into yh.
    const int orow = lane >> 2, och = lane & 3;             // output: 8 keys of a row per lane
    const int gi = i0 + orow;
    const int vis = gi < Lq ? (a.causal ? min(Lk, gi + 1 + shift) : Lk) : 0;
    half_t* const obase = a.scores + (((size_t)b * H + wv) * Lq + min(gi, Lq - 1)) * Lk + 8 * och;
    const size_t ohead = (size_t)NW * Lq * Lk;              // from a head of this wave to its next
    const unsigned char* const yrd = yh + wv * SM_YH_HEAD + orow * (PF_TK * 2) + 16 * och;
    const half_t* const pbase = a.prev + ((size_t)b * H * Lq + x_row) * Lk;
    const size_t phead = (size_t)Lq * Lk;
    f32x4 y[NBW][HBO];
    f16x8 held;
    auto out_read = [&](int u) {
      if (wv + NW * u < H) held = *(const f16x8*)(yrd + u * NW * SM_YH_HEAD);
    };
    auto out_store = [&](int u, int tile) {                 // the lane's 8 keys of key tile `tile`
      if (wv + NW * u >= H) return;
      if (TILED) {
        *(f16x8*)(a.scores + trow + tile * tile_stride + (wv + NW * u) * (PF_ROWS * PF_TK)) = held;
        return;
      }
      const int jc = tile * PF_TK + 8 * och;                // first of the lane's 8 keys
      if (jc >= vis) return;
      half_t* sp = obase + u * ohead + jc - 8 * och;
      if (jc + 8 <= vis) {
        *(f16x8*)sp = held;
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (jc + e < vis) sp[e] = held[e];
      }
    };
    // The result leaves the registers as dwords of two keys: a lane holds one key of the four heads
    // 4 g + v; the lanes of a pair (keys c, c ^ 1) swap halves, after which the even lane has both
    // keys of heads v = 0, 1 and the odd lane those of v = 2, 3 (2-byte LDS writes cost about three
    // times as much).
    const bool odd = c & 1;
    auto write_y = [&]() {
#pragma unroll
      for (int qn = 0; qn < NBW; ++qn) {
        const int nb = wv + qn * NW, i = nb >> 1, kh = nb & 1;
#pragma unroll
        for (int hb = 0; hb < HBO; ++hb) {
          f16x4 hv;
#pragma unroll
          for (int v = 0; v < 4; ++v) hv[v] = f32_to_half_sat(y[qn][hb][v]);
          const uint2 pq = __builtin_bit_cast(uint2, hv);   // (heads v = 0, 1), (heads v = 2, 3) of key c
          const unsigned keep = odd ? pq.y : pq.x;
          const unsigned got = (unsigned)__builtin_amdgcn_update_dpp(0, (int)(odd ? pq.x : pq.y), 0xB1, 0xF, 0xF, true);
          const unsigned first = odd ? got : keep, second = odd ? keep : got;   // keys c & ~1, c | 1
          const int hl = 16 * hb + 4 * g + 2 * (c & 1);
          unsigned char* yp = yh + hl * SM_YH_HEAD + i * (PF_TK * 2) + (16 * kh + (c & ~1)) * 2;
          if (hl < H) *(unsigned*)yp = (first & 0xffffu) | (second << 16);
          if (hl + 1 < H) *(unsigned*)(yp + SM_YH_HEAD) = (first >> 16) | (second & 0xffff0000u);
        }
      }
    };
    constexpr int N_OPS = XCH + 1 + XCH + 2 * HPW;          // read / store pairs of a tile, then the loads of the next
    constexpr int N_GROUPS = (FS / SC) * (2 * SC + HBO);
    constexpr int OPG = (N_OPS + N_GROUPS - 1) / N_GROUPS;
    const bool x_all = Din == 32 * KS;
    // one tile; PEND (a compile-time constant: the first tile of a run has its own copy of the
    // loop body, so that no store of the others sits behind a branch): the result of the tile
    // before is in yh and leaves during this tile's FFN
    auto do_tile = [&](auto pend, int tile) {
      constexpr bool PEND = decltype(pend)::value;
      stage_tile();
      if (PEND) write_y();
      lds_barrier();                                         // A: xs and yh are complete
      f16x8 x[NBW][KS];
      read_x(x, x_all);
      const int jn = (tile + 1) * PF_TK;
      const int xoff = min(jn + xq8, Lk - 8);
      const size_t toff = trow + min(tile + 1, n_kt - 1) * tile_stride;
      int koff[2];
#pragma unroll
      for (int half = 0; half < 2; ++half) koff[half] = min(jn + 16 * half + c, Lk - 1) * 32 + 8 * g;
      // (the loads are not conditional on a next tile: its clamped addresses are in bounds, and a
      // branch around a load makes the compiler wait for every earlier one)
      Ffn::template apply_lds_chunked_ahead<NBW, SC>(w_s, x, y, [&](int gidx) {
#pragma unroll
        for (int k = gidx * OPG; k < (gidx + 1) * OPG && k < N_OPS; ++k) {
          if (k <= XCH) {                                    // stores first: the wait for the loads, at the
            if (PEND) {                                      // next staging, also waits for them
              if (k > 0) out_store(k - 1, tile - 1);
              if (k < XCH) out_read(k);
            }
          } else if (k <= 2 * XCH) {
            const int u = k - XCH - 1, h = min(wv + NW * u, H - 1);
            if (TILED) xr[u] = *(const pf_u32x4*)(a.prev + toff + h * (PF_ROWS * PF_TK));
            else xr[u] = *(const pf_u32x4*)(pbase + h * phead + xoff);
          } else {
            const int u = (k - 2 * XCH - 1) >> 1, half = (k - 2 * XCH - 1) & 1;
            const int h = min(wv + NW * u, H - 1);
            kop[u][half] = *(const bf16x8*)(a.kp + ((size_t)b * a.Hkv + h / group) * a.Lkp * 32 + koff[half]);
          }
        }
      });
      lds_barrier();                                         // B: xs and yh have been read
    };
    do_tile(std::false_type{}, t_first);
    for (int tile = t_first + 1; tile < t_last; ++tile) do_tile(std::true_type{}, tile);
    // the result of the last tile of the run
    write_y();
    lds_barrier();
#pragma unroll
    for (int u = 0; u < XCH; ++u) {
      out_read(u);
      out_store(u, t_last - 1);
    }
  } else
  for (int tile = t_first; tile < t_last; ++tile) {
    const int j0 = tile * PF_TK;
    lds_barrier();                                           // the stores of the previous tile have read ys
    // ---- 1. input tile -----------------------------------------------------------------------
#pragma unroll
    for (int u = 0; u < XCH; ++u) {
      const int h = wv + NW * u;
      if (h < H) *(pf_u32x4*)(xs + h * PF_XS_HEAD + lane * 16) = xr[u];
    }
#pragma unroll
    for (int u = 0; u < HPW; ++u) {
      const int h = wv + NW * u;
      if (h >= H) break;
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        f32x4 d = {0.f, 0.f, 0.f, 0.f};
        d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop[u][half], qop[u], d, 0, 0, 0);
        // d[v] = A_delta(row c, key 16 half + 4 g + v) / scale
        f16x4 hv;
#pragma unroll
        for (int v = 0; v < 4; ++v) hv[v] = f32_to_half_sat(d[v] * a.dscale);
        *(f16x4*)(xs + (H + h) * PF_XS_HEAD + c * 64 + (16 * half + 4 * g) * 2) = hv;
      }
    }
    if (tile + 1 < t_last) prefetch(tile + 1);
    lds_barrier();   
    // ---- 2. FFN over the wave's 4 blocks of 16 positions, two at a time (the operands of four do
    //         not fit the register file next to those of 40 - 48 heads) ---------------------------
    f32x4 y[NBW][HBO];
#pragma unroll
    for (int q = 0; q < NBW; q += 2) {
      f16x8 x[2][KS];
#pragma unroll
      for (int n = 0; n < 2; ++n) {
        const int nb = wv + (q + n) * NW;                   // block = (row nb / 2, key half nb % 2)
        const int i = nb >> 1, kh = nb & 1;
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
            x[n][ks][e] = 32 * ks + 8 * g + e < Din ? lo[e] : (_Float16)0.f;
            x[n][ks][4 + e] = 32 * ks + 8 * g + 4 + e < Din ? hi[e] : (_Float16)0.f;
          }
        }
      }
      f32x4 yq[2][HBO];
      Ffn::template apply_lds_chunked<2, SC>(w_s, x, yq, [](int) {});
#pragma unroll
      for (int n = 0; n < 2; ++n)
#pragma unroll
        for (int hb = 0; hb < HBO; ++hb) y[q + n][hb] = yq[n][hb];
    }
    lds_barrier();                                           // every wave has read the input tile
    // ---- 3. output tile: float32 [head][row][key] over the input tile, then out by heads ---------
#pragma unroll
    for (int qn = 0; qn < NBW; ++qn) {
      const int nb = wv + qn * NW, i = nb >> 1, kh = nb & 1;
#pragma unroll
      for (int hb = 0; hb < HBO; ++hb)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int hl = 16 * hb + 4 * g + v;
          if (hl < H) *(float*)(ys + hl * SM_YS_HEAD + i * SM_YS_ROW + (16 * kh + c) * 4) = y[qn][hb][v];
        }
    }
    lds_barrier();   
    {
      const int row = lane >> 2, ch = lane & 3;             // 8 keys of a row per lane
      const int gi = i0 + row, jc = j0 + 8 * ch;
      const int vis = gi < Lq ? (a.causal ? min(Lk, gi + 1 + shift) : Lk) : 0;
      for (int h = wv; h < H; h += NW) {
        const float4 lo = *(const float4*)(ys + h * SM_YS_HEAD + row * SM_YS_ROW + 32 * ch);
        const float4 hi = *(const float4*)(ys + h * SM_YS_HEAD + row * SM_YS_ROW + 32 * ch + 16);
        const float vals[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
        if (jc >= vis) continue;
        const size_t at = (((size_t)b * H + h) * Lq + gi) * Lk + jc;
        f16x8 hv;
#pragma unroll
        for (int e = 0; e < 8; ++e) hv[e] = f32_to_half_sat(vals[e]);
        if (jc + 8 <= vis) {
          *(f16x8*)(a.scores + at) = hv;
        } else {
#pragma unroll
          for (int e = 0; e < 8; ++e)
            if (jc + e < vis) a.scores[at + e] = hv[e];
        }
      }
    }
  }
  pos += t_last - t_first;
  tile0 = 0;
  if (++rg == n_rg) rg = 0, ++b;
  }
}

// LDS bytes of k_lisa_scores_mfma<HBI, FS, HBO> for H heads.
template <int HBI, int FS, int HBO>
constexpr int scores_mfma_lds(int H) {
  const int io = HBI <= 4 ? 2 * H * PF_XS_HEAD + H * SM_YH_HEAD
                          : (2 * H * PF_XS_HEAD > H * SM_YS_HEAD ? 2 * H * PF_XS_HEAD : H * SM_YS_HEAD);
  return ((io + 15) & ~15) + MfmaFfn<HBI, FS, HBO>::kStageBytes;
}

}  // namespace lisa
