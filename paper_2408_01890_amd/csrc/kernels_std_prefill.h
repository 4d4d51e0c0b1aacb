// Standard attention layer that also emits the shared scores (Sec. 2.1 Eq. 1-2), bf16 on MFMA.
//
// One workgroup = one head and 128 consecutive query rows, one wave per block of 32 rows,
// streaming over 32-key tiles up to the diagonal.  The K tile (and the V tile) of a step is
// loaded once per workgroup into LDS (double buffered, one barrier per tile) and read by the
// four waves as MFMA operands: a fourth of the global loads of a wave-private stream.
// Both products use the 32x32x16 MFMA and keep the query row on the lane index
// (lane = 32 half + r), so the softmax statistics and the probabilities never change lanes:
//   scores  D[key, row] = sum_t K[key,t] Q[row,t]   A = K rows, B = Q^T (8 operands, resident).
//           MFMA row m is given key 16 (m/16) + 8 ((m/4)%2) + 4 ((m/8)%2) + m%4 so that lane
//           (r, half) ends with keys 8 half .. 8 half + 7 and 16 + 8 half .. 16 + 8 half + 7:
//           two 16-byte half stores.
//   output  D[d, row] = sum_key V^T[d,key] P^T[key,row]   A = V by key chunks [L/8][128][8]
//           (k_regroup_v), B = the lane's probabilities as they are.
// A = Q K^T * scale is stored as half; the softmax works on the float32 values.
// A workgroup takes two row groups, the x-th longest and the x-th shortest, so that all
// workgroups stream the same number of tiles (large problems), or one row group (problems with
// fewer than two such workgroups per compute unit: twice the waves in flight).
#pragma once
#include "kernels_prefill.h"

namespace lisa {

typedef float f32x16 __attribute__((ext_vector_type(16)));

struct StdPrefillArgs {
  const bf16_t* q;        // [B,H,Lq,128]
  const bf16_t* k;        // [B,Hkv,Lk,128]
  const bf16_t* vt;       // [B,Hkv,Lkp/8,128,8] or null (scores only)
  half_t* scores;         // [B,H,Lq,Lk] or null
  const void* given;      // GIVEN mode: scores [B,H,Lq,Lk] to take instead of Q K^T (then q, k unused):
                          // float32 (GIVEN = 1) or IEEE half (GIVEN = 2)
  void* out;              // [B,Lq,H,128] or null
  int H, Hkv, Lq, Lk, Lkp, causal, out_f32;
  int pair;               // 1: a workgroup takes two row groups (grid.y = ceil(n_groups / 2)), 0: one
  float scale;
  int tiled;              // scores are written (GIVEN = 2: read) as [B,ceil(Lq/16),ceil(Lk/32),H,16,32]
};

__device__ __forceinline__ float halves_max(float v) {
  const unsigned u = __float_as_uint(v);
  auto q = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(q[0]), __uint_as_float(q[1]));
}
__device__ __forceinline__ float halves_sum(float v) {
  const unsigned u = __float_as_uint(v);
  auto q = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __uint_as_float(q[0]) + __uint_as_float(q[1]);
}

constexpr int SP_ROWS = 32;                 // rows per wave
constexpr int SP_WAVES = 4;
constexpr int SP_GROUP = SP_ROWS * SP_WAVES;   // rows per workgroup pass
constexpr int SP_TK = 32;
constexpr int SP_KROW = 128 * 2 + 16;       // bytes per key row of the K tile in LDS (padded: no bank conflicts)
constexpr int SP_KTILE = SP_TK * SP_KROW;   // 8704
constexpr int SP_VTILE = SP_TK * 128 * 2;   // 8192
constexpr int SP_SROW = 2 * SP_TK * 2 + 16;  // bytes per row of a wave's score staging tile (64 keys, padded)
constexpr int SP_STILE = SP_ROWS * SP_SROW;  // 4608

// LDS bytes: two K tiles, the four staging tiles, two V tiles.
constexpr int std_prefill_head_lds(bool with_v) {
  return 2 * SP_KTILE + SP_WAVES * SP_STILE + (with_v ? 2 * SP_VTILE : 0);
}

// grid (H, pair ? ceil(n_groups / 2) : n_groups, B) with n_groups = ceil(Lq / 128), block 256.  The head is the
// fastest grid index: consecutive workgroups go to different XCDs, so an XCD works on every
// eighth head and its L2 fetches the K / V of those heads only (they are what every row group
// of a head re-reads).
// Requires d_k = 128, Lk % 8 == 0.
// GIVEN: the scores are read from a.given (the A_n that a LiSA scores kernel left there) instead
// of being computed; the rest (masking, online softmax, P V) is the same.
template <bool WITH_V, int GIVEN = 0>
__global__ __launch_bounds__(256, 2) void k_std_prefill(StdPrefillArgs a) {
  constexpr int DK = 128;
  __shared__ __align__(16) unsigned char lds[std_prefill_head_lds(WITH_V)];
  unsigned char* ks_ = lds;
  unsigned char* ss_ = ks_ + 2 * SP_KTILE;              // score staging, one tile per wave
  unsigned char* vs_ = ss_ + SP_WAVES * SP_STILE;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r = lane & 31, half = lane >> 5;
  const int b = blockIdx.z, h = blockIdx.x;
  const int Lq = a.Lq, Lk = a.Lk, H = a.H;
  const int shift = Lk - Lq;
  const int kv = h / (H / a.Hkv);
  const float LOG2E = 1.4426950408889634f;
  const int n_groups = (Lq + SP_GROUP - 1) / SP_GROUP;
  // key of MFMA row m = r (see the header)
  const int key_of_r = 16 * (r >> 4) + 8 * ((r >> 2) & 1) + 4 * ((r >> 3) & 1) + (r & 3);
  const bf16_t* kbase = GIVEN ? nullptr : a.k + ((size_t)b * a.Hkv + kv) * Lk * DK;
  const bf16_t* vbase = WITH_V ? a.vt + ((size_t)b * a.Hkv + kv) * (a.Lkp / 8) * (DK * 8) : nullptr;
  // cooperative tile loads: thread -> two 16-byte chunks of the K tile (key, 8 features) and two
  // of the V tile (contiguous 8 KB)
  const int ck_key = tid >> 4, ck_c = tid & 15;          // chunk u: key ck_key + 16 u
  // operand addresses in LDS
  const int k_rd = key_of_r * SP_KROW + half * 16;       // + 32 ks
  const int v_rd = (half * DK + r) * 16;                 // + (2 s DK + 32 db) 16

  for (int rep = 0; rep < 2; ++rep) {
    const int grp = rep ? (int)blockIdx.y : n_groups - 1 - (int)blockIdx.y;
    if (rep && (!a.pair || grp >= n_groups - 1 - grp)) break;   // (the middle group of an odd count is alone)
    const int i0 = grp * SP_GROUP + wv * SP_ROWS;          // first row of this wave
    const bool have_rows = i0 < Lq;
    const int my_row = min(i0 + r, Lq - 1);
    const int vis_row = a.causal ? min(Lk, my_row + 1 + shift) : Lk;
    const int i_last_w = min(i0 + SP_ROWS - 1, Lq - 1);
    const int n_tiles_w =
        have_rows ? ((a.causal ? min(Lk, i_last_w + 1 + shift) : Lk) + SP_TK - 1) / SP_TK : 0;
    const int i_last_g = min(grp * SP_GROUP + SP_GROUP - 1, Lq - 1);
    const int n_tiles = ((a.causal ? min(Lk, i_last_g + 1 + shift) : Lk) + SP_TK - 1) / SP_TK;
    const int n_full =
        (have_rows && i0 + SP_ROWS <= Lq) ? (a.causal ? min(Lk, i0 + 1 + shift) : Lk) / SP_TK : 0;

    // B operands of the score product: Q[row][16 ks + 8 half + e]
    bf16x8 qop[DK / 16];
    if (!GIVEN) {
      const bf16_t* qp = a.q + (((size_t)b * H + h) * Lq + my_row) * DK + 8 * half;
#pragma unroll
      for (int ks = 0; ks < DK / 16; ++ks) qop[ks] = *(const bf16x8*)(qp + 16 * ks);
    }
    const size_t grow_at = (((size_t)b * H + h) * Lq + my_row) * Lk;
    const float* grow = GIVEN == 1 ? (const float*)a.given + grow_at : nullptr;
    const half_t* grow_h = GIVEN == 2 ? (const half_t*)a.given + grow_at : nullptr;
    const int n_kt = (Lk + SP_TK - 1) / SP_TK;               // tile grid of the tiled score layout
    // (tiled: the H pieces of a tile follow each other, 1 KB each; see k_lisa_prefill_fused)
    const size_t seq_elems = a.tiled ? (size_t)((Lq + 15) / 16) * n_kt * H * (16 * SP_TK) : (size_t)H * Lq * Lk;
    half_t* sbase = a.scores ? a.scores + (size_t)b * seq_elems + (size_t)h * (a.tiled ? (size_t)16 * SP_TK : (size_t)Lq * Lk)
                             : nullptr;
    unsigned char* stg = ss_ + wv * SP_STILE;

    // The K / V tile of a step travels through registers: loaded three tiles ahead into one of two
    // register sets, written to LDS one tile ahead.  Two sets rather than one because loads and
    // stores complete in one order behind one counter, and the score stores below are conditional
    // (uncountable for the compiler): with one set the wait for the tile loads at the top of a step
    // was a wait for everything, the score stores of the step before included; with two the loads
    // of the other set lie between, and only what is older than those has to be complete.
    typedef pf_u32x4 TileRegs[2][2];                       // [K, V][chunk]
    TileRegs regs_a, regs_b;
    auto load_tile = [&](int tile, TileRegs& tr) {
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int j = min(tile * SP_TK + ck_key + 16 * u, Lk - 1);
        if (!GIVEN) tr[0][u] = *(const pf_u32x4*)(kbase + (size_t)j * DK + 8 * ck_c);
        if (WITH_V) tr[1][u] = *(const pf_u32x4*)(vbase + (size_t)tile * (SP_TK / 8 * DK * 8) + (tid + 256 * u) * 8);
      }
    };
    auto store_tile = [&](int buf, const TileRegs& tr) {
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        if (!GIVEN) *(pf_u32x4*)(ks_ + buf * SP_KTILE + (ck_key + 16 * u) * SP_KROW + ck_c * 16) = tr[0][u];
        if (WITH_V) *(pf_u32x4*)(vs_ + buf * SP_VTILE + (tid + 256 * u) * 16) = tr[1][u];
      }
    };
    // GIVEN = 2: the wave's scores of a tile are loaded two tiles ahead (nothing else hides the
    // latency of these loads: there is no score product to wait behind)
    f16x8 gq[2][2];
    // (tiled: row my_row of head h, tile t at (((my_row / 16) n_kt + t) H + h) KB + 64 (my_row % 16) bytes)
    const half_t* grow_t = GIVEN == 2 ? (const half_t*)a.given + (size_t)b * seq_elems +
                                            ((size_t)(my_row >> 4) * n_kt * H + h) * (16 * SP_TK) +
                                            (my_row & 15) * SP_TK + 8 * half
                                      : nullptr;
    auto load_scores = [&](int tile, f16x8 (&dst)[2]) {
#pragma unroll
      for (int u = 0; u < 2; ++u)    // (keys beyond Lk: any in-bounds 8 scores will do, those positions are masked)
        dst[u] = *(const f16x8*)(a.tiled ? grow_t + (size_t)tile * H * (16 * SP_TK) + 16 * u
                                         : grow_h + min(tile * SP_TK + 16 * u + 8 * half, Lk - 8));
    };
    if (rep) __syncthreads();                              // the first pass is done with both buffers
    load_tile(0, regs_a);
    store_tile(0, regs_a);
    load_tile(min(1, n_tiles - 1), regs_a);                // set a: odd tiles, set b: even tiles
    load_tile(min(2, n_tiles - 1), regs_b);
    if (GIVEN == 2) {
      load_scores(0, gq[0]);
      load_scores(min(1, n_tiles - 1), gq[1]);
    }

    f32x16 o[DK / 32];
#pragma unroll
    for (int db = 0; db < DK / 32; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) o[db][v] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    auto step = [&](int tile, TileRegs& tr) {              // tr holds tile + 1
      // tile `tile` is complete in buffer tile & 1, and every wave is done with the other buffer
      lds_barrier();
      store_tile((tile + 1) & 1, tr);
      load_tile(min(tile + 3, n_tiles - 1), tr);
      if (tile >= n_tiles_w) return;                       // beyond this wave's diagonal (wave-uniform)
      const unsigned char* kt = ks_ + (tile & 1) * SP_KTILE;
      const unsigned char* vtl = vs_ + (tile & 1) * SP_VTILE;
      const int j0 = tile * SP_TK;
      // an[8 u + e] = score of key j0 + 16 u + 8 half + e for row r
      float an[16];
      if (GIVEN == 2) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
#pragma unroll
          for (int e = 0; e < 8; ++e) an[8 * u + e] = (float)gq[0][u][e];
          gq[0][u] = gq[1][u];
        }
        load_scores(min(tile + 2, n_tiles - 1), gq[1]);
      } else if (GIVEN == 1) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const float* gp = grow + min(j0 + 16 * u + 8 * half, Lk - 8);
          const float4 lo = *(const float4*)gp, hi = *(const float4*)(gp + 4);
          an[8 * u + 0] = lo.x, an[8 * u + 1] = lo.y, an[8 * u + 2] = lo.z, an[8 * u + 3] = lo.w;
          an[8 * u + 4] = hi.x, an[8 * u + 5] = hi.y, an[8 * u + 6] = hi.z, an[8 * u + 7] = hi.w;
        }
      } else {
        f32x16 acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
        for (int ks = 0; ks < DK / 16; ++ks) {
          const bf16x8 kop = *(const bf16x8*)(kt + k_rd + 32 * ks);
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop, qop[ks], acc, 0, 0, 0);
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) an[v] = acc[v] * a.scale;
      }
      const bool full = tile < n_full;
      const int jl = j0 + 8 * half;
      if (a.scores) {
        // A leaves through the wave's staging tile in whole 128-byte pieces of a row (64 keys =
        // two tiles): 64-byte pieces reach HBM at about half the rate of whole lines
        f16x8 hv0, hv1;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          hv0[e] = f32_to_half_sat(an[e]);
          hv1[e] = f32_to_half_sat(an[8 + e]);
        }
        unsigned char* sl = stg + r * SP_SROW + (tile & 1) * 64 + 16 * half;
        *(f16x8*)sl = hv0;
        *(f16x8*)(sl + 32) = hv1;
        if (a.tiled) {
          // tiled layout: the wave's 32 rows are two row blocks, one 1 KB tile each per step
#pragma unroll
          for (int q = 0; q < 2; ++q) {
            const int rbq = (i0 >> 4) + q;
            if (16 * rbq >= Lq) continue;                      // (wave-uniform)
            const f16x8 hv =
                *(const f16x8*)(stg + (16 * q + (lane >> 2)) * SP_SROW + (tile & 1) * 64 + (lane & 3) * 16);
            // (non-temporal: nobody reads the scores before the whole tensor is written; 2.45 -> 2.14 ms
            // on the LLaMA3-8B shape, and the layer that reads them next is not slower, also where
            // the tensor would fit the last-level cache)
            __builtin_nontemporal_store(__builtin_bit_cast(pf_u32x4, hv),
                                        (pf_u32x4*)((char*)sbase + ((size_t)rbq * n_kt + tile) * H * (16 * SP_TK * 2) + lane * 16));
          }
        } else if ((tile & 1) == 1 || tile == n_tiles_w - 1) {
          const int jc = (tile >> 1) * (2 * SP_TK) + 8 * (lane & 7);
          const bool pair_full = (tile | 1) < n_full;
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int row = 8 * u + (lane >> 3), gi = i0 + row;
            const f16x8 hv = *(const f16x8*)(stg + row * SP_SROW + (lane & 7) * 16);
            const int vis = gi < Lq ? (a.causal ? min(Lk, gi + 1 + shift) : Lk) : 0;
            half_t* sp = sbase + (size_t)min(gi, Lq - 1) * Lk + jc;
            if (pair_full || jc + 8 <= vis) {
              __builtin_nontemporal_store(__builtin_bit_cast(pf_u32x4, hv), (pf_u32x4*)sp);
            } else {
#pragma unroll
              for (int e = 0; e < 8; ++e)
                if (jc + e < vis) sp[e] = hv[e];
            }
          }
        }
      }
      if (WITH_V) {
        if (!full) {
#pragma unroll
          for (int v = 0; v < 16; ++v)
            if (jl + 16 * (v >> 3) + (v & 7) >= vis_row) an[v] = -INFINITY;
        }
        float mx = an[0];
#pragma unroll
        for (int v = 1; v < 16; ++v) mx = fmaxf(mx, an[v]);
        mx = halves_max(mx);
        const float m_new = fmaxf(m_run, mx);
        const float m2 = m_new * LOG2E;
        const float alpha = fast_exp2(m_run * LOG2E - m2);
        m_run = m_new;
        float ps = 0.f;
        bf16x8 pop[2];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float p = fast_exp2(__builtin_fmaf(an[v], LOG2E, -m2));
          ps += p;
          pop[v >> 3][v & 7] = (__bf16)p;
        }
        l_run = l_run * alpha + ps;
        if (__any(alpha != 1.f)) {
#pragma unroll
          for (int db = 0; db < DK / 32; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[db][v] *= alpha;
        }
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
          for (int db = 0; db < DK / 32; ++db) {
            const bf16x8 vop = *(const bf16x8*)(vtl + v_rd + (2 * s * DK + 32 * db) * 16);
            o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop, pop[s], o[db], 0, 0, 0);
          }
      }
    };
    // (everything loaded so far has arrived before the loop is entered: the wait counts inside the
    // loop then follow from the loop's own issue order, not from that of the prologue)
    __builtin_amdgcn_s_waitcnt(0x0F70);                      // vmcnt(0), others untouched
    int tile = 0;
    for (; tile + 1 < n_tiles; tile += 2) {                // (both steps on every path round the loop)
      step(tile, regs_a);
      step(tile + 1, regs_b);
    }
    if (tile < n_tiles) step(tile, regs_a);

    if (WITH_V) {
      // O[row][h][32 db + 8 (v/4) + 4 half + v%4] = o[db][v] / l
      const float inv = 1.f / halves_sum(l_run);
      if (i0 + r < Lq) {
        const size_t at = (((size_t)b * Lq + i0 + r) * H + h) * DK + 4 * half;
#pragma unroll
        for (int db = 0; db < DK / 32; ++db)
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            const float x0 = o[db][4 * q4] * inv, x1 = o[db][4 * q4 + 1] * inv;
            const float x2 = o[db][4 * q4 + 2] * inv, x3 = o[db][4 * q4 + 3] * inv;
            const size_t d = at + 32 * db + 8 * q4;
            if (a.out_f32) {
              *(float4*)((float*)a.out + d) = make_float4(x0, x1, x2, x3);
            } else {
              uint2 pk;
              pk.x = f32_to_bf16_bits(x0) | (f32_to_bf16_bits(x1) << 16);
              pk.y = f32_to_bf16_bits(x2) | (f32_to_bf16_bits(x3) << 16);
              *(uint2*)((bf16_t*)a.out + d) = pk;
            }
          }
      }
    }
  }
}

}  // namespace lisa
