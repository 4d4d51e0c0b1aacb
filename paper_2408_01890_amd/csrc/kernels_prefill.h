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
//   stage A(t)    : reads xs, writes ys; barrier B2.  Between the FFN blocks it issues what does not
//                   depend on this stage: the V operands of the wave's second head for tile t, the
//                   loads of the A_{n-1} tile t+1 and the stores of the pair of A_n tiles that
//                   stage B(t-1) completed.
//   stage B(t)    : head by head, consumes the K_LR / V operand registers and refills them with
//                   the operands of tile t+1 (one register set per head when the register file
//                   allows, else one rotating set refilled for the next head); stages A_n in LDS;
//                   then writes the A_{n-1} tile t+1 into xs.
// What bounds it: a compute unit takes in about 75 GB/s of 16-byte loads from the L2 (measured),
// and a tile moves 192 KB through that pipe (V 128, K_LR 32, A_{n-1} 32); a load that cannot be
// issued blocks its wave, so the loads are spread over both stages rather than issued in bursts.
#pragma once
#include "kernels_generic.h"
#include "mfma_ffn.h"

namespace lisa {

constexpr int PF_ROWS = 16;       // query rows per workgroup
// Neighbouring units of work per chunk: a chunk times the NG head groups fills the 32 compute
// units of one XCD (see the grid of k_lisa_prefill_fused).
constexpr int pf_chunk_units(int ng) { return 32 / ng > 0 ? 32 / ng : 1; }
constexpr int PF_TK = 32;         // keys per tile
constexpr int PF_XS_HEAD = PF_ROWS * PF_TK * 2 + 32;        // bytes per head of the A_{n-1} tile
constexpr int PF_YS_ROW = PF_TK * 4 + 16;                   // bytes per (head,row) of the y tile
constexpr int PF_YS_HEAD = PF_ROWS * PF_YS_ROW + 16;
constexpr int PF_AS_ROW = 2 * PF_TK * 2 + 16;                // bytes per row of the A_n staging tile (64 keys)
constexpr int PF_AS_HEAD = PF_ROWS * PF_AS_ROW;

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
  int split;              // key splits per row block (1: the kernel writes `out` itself)
  float* part_o;          // [split][B][Lqp][H][128] unnormalised partial outputs (split > 1)
  float* part_ml;         // [split][B][Lqp][H][2]   running maximum, partial sum
  int pair;               // workgroup x takes the units (last - x) and x
  int B;                  // sequences
  int tiled;              // prev and scores are [B,ceil(Lq/16),ceil(Lk/32),H,16,32] (1 KB per head and tile)
};

typedef unsigned short pf_u16x8 __attribute__((ext_vector_type(8)));

// One 64-key x 64-feature tile of vt[bh][j / 8][d][j % 8] = v[bh][j][d] (zero for j >= Lk)
// through LDS, 256 threads.  VEC: v is 16-byte aligned and dk % 8 == 0 (row chunks of 8 features
// are read as one 16-byte load); the output is always written as 16-byte chunks.
template <bool VEC>
__device__ __forceinline__ void regroup_v_tile(const bf16_t* __restrict__ v, bf16_t* __restrict__ vt, int Lk,
                                               int Lkp, int dk, int j0, int d0, size_t bh,
                                               unsigned short (*tile)[72]) {
  if (VEC) {
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int id = threadIdx.x + 256 * u, jl = id >> 3, dc = id & 7;
      pf_u16x8 x = {0, 0, 0, 0, 0, 0, 0, 0};
      if (j0 + jl < Lk) x = *(const pf_u16x8*)(v + (bh * Lk + j0 + jl) * dk + d0 + 8 * dc);
      *(pf_u16x8*)&tile[jl][8 * dc] = x;
    }
  } else {
    for (int idx = threadIdx.x; idx < 64 * 64; idx += 256) {
      const int jl = idx >> 6, dl = idx & 63;
      tile[jl][dl] = (j0 + jl < Lk) ? v[(bh * Lk + j0 + jl) * dk + d0 + dl].bits : (unsigned short)0;
    }
  }
  __syncthreads();
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int id = threadIdx.x + 256 * u, jc = id >> 6, dl = id & 63;
    pf_u16x8 x;
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = tile[8 * jc + e][dl];
    *(pf_u16x8*)(vt + ((bh * (Lkp / 8) + j0 / 8 + jc) * dk + d0 + dl) * 8) = x;
  }
}

// grid (Lkp / 64, dk / 64, B * Hkv), block 256.
template <bool VEC>
__global__ __launch_bounds__(256) void k_regroup_v(const bf16_t* __restrict__ v, bf16_t* __restrict__ vt,
                                                   int Lk, int Lkp, int dk) {
  __shared__ __align__(16) unsigned short tile[64][72];
  regroup_v_tile<VEC>(v, vt, Lk, Lkp, dk, blockIdx.x * 64, blockIdx.y * 64, blockIdx.z, tile);
}

// The repacking of one fused prefill call in one launch, block 256:
//   blocks [0, n_v):   V tiles as in k_regroup_v (tile index = x + nx (y + ny z))
//   the rest:          Q_LR and K_LR rows zero-padded from r to 32 elements, one 16-byte chunk of
//                      a padded row per thread (64 rows per block, Q rows first).
template <bool VEC>
__global__ __launch_bounds__(256) void k_prepare_prefill(const bf16_t* __restrict__ q_lr,
                                                         const bf16_t* __restrict__ k_lr,
                                                         const bf16_t* __restrict__ v, bf16_t* __restrict__ qp,
                                                         bf16_t* __restrict__ kp, bf16_t* __restrict__ vt, int B,
                                                         int H, int Hkv, int Lq, int Lk, int Lqp, int Lkp,
                                                         int r, int dk) {
  __shared__ __align__(16) unsigned short tile[64][72];
  const int nx = Lkp / 64, ny = dk / 64;
  const int n_v = nx * ny * B * Hkv;
  int blk = blockIdx.x;
  if (blk < n_v) {
    const int x = blk % nx, y = blk / nx % ny, z = blk / (nx * ny);
    regroup_v_tile<VEC>(v, vt, Lk, Lkp, dk, x * 64, y * 64, z, tile);
    return;
  }
  blk -= n_v;
  const size_t q_rows = (size_t)B * H * Lqp, k_rows = (size_t)B * Hkv * Lkp;
  const size_t row = (size_t)blk * 64 + (threadIdx.x >> 2);
  const int t0 = 8 * (threadIdx.x & 3);
  const bf16_t* src = nullptr;
  bf16_t* dst;
  if (row < q_rows) {
    const int i = row % Lqp;
    const size_t bh = row / Lqp;
    if (i < Lq) src = q_lr + (bh * Lq + i) * r;
    dst = qp + row * 32 + t0;
  } else if (row < q_rows + k_rows) {
    const size_t rk = row - q_rows;
    const int j = rk % Lkp;
    const size_t bh = rk / Lkp;
    if (j < Lk) src = k_lr + (bh * Lk + j) * r;
    dst = kp + rk * 32 + t0;
  } else {
    return;
  }
  pf_u16x8 x;
#pragma unroll
  for (int e = 0; e < 8; ++e) x[e] = (src && t0 + e < r) ? src[t0 + e].bits : (unsigned short)0;
  *(pf_u16x8*)dst = x;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every global
// load and store in flight (workgroup-scope fence), which would drain the operand prefetch of
// the pipeline at every tile; the tiles exchange data through LDS alone.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Maxima as single instructions.  fmaxf makes the compiler quiet every operand it cannot prove
// canonical (a copy through v_max x, x: 8 of them per head and tile in the softmax); the scores
// are never signalling NaNs, so the plain instructions are used.
__device__ __forceinline__ float max2_raw(float a, float b) {
  float r;
  asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ float max3_raw(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}
// Butterflies across the four 16-lane rows of a wave with the row-swap instructions of gfx950
// (no LDS crossbar): after both steps every lane 16 g + c holds the reduction over g.
// Returns max(m, reduction of v).
__device__ __forceinline__ float rows_max(float v, float m) {
  const unsigned u = __float_as_uint(v);
  auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);   // rows (0,1) and (2,3) exchanged
  v = max2_raw(__uint_as_float(r[0]), __uint_as_float(r[1]));
  const unsigned w = __float_as_uint(v);
  auto q = __builtin_amdgcn_permlane32_swap(w, w, false, false);   // halves exchanged
  return max3_raw(m, __uint_as_float(q[0]), __uint_as_float(q[1]));
}
__device__ __forceinline__ float rows_sum(float v) {
  const unsigned u = __float_as_uint(v);
  auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  v = __uint_as_float(r[0]) + __uint_as_float(r[1]);
  const unsigned w = __float_as_uint(v);
  auto q = __builtin_amdgcn_permlane32_swap(w, w, false, false);
  return __uint_as_float(q[0]) + __uint_as_float(q[1]);
}

// Access at a wave-uniform base plus a per-lane 32-bit byte offset: the form that one global
// load or store with a scalar base register pair and a vector offset covers, so that no lane
// keeps 64-bit pointers.
template <class T>
__device__ __forceinline__ T ld_uv(const void* ubase, unsigned voff, int imm = 0) {
  return *(const T*)((const char*)ubase + imm + voff);
}
template <class T>
__device__ __forceinline__ void st_uv(void* ubase, unsigned voff, T v) {
  *(T*)((char*)ubase + voff) = v;
}
// The same for the A_{n-1} and A_n streams, kept apart because cache hints were tried on them:
// non-temporal loads stop the head groups of a row block from sharing the A_{n-1} tile in the L2
// (fetch 36.9 GB instead of 22.9 GB on the LLaMA3-8B shape), non-temporal stores of row-major
// scores change nothing (21.4 GB, same time); plain accesses are what is used here.  (The stores of
// tiled scores, which do not come through these helpers, are non-temporal.)
template <class T>
__device__ __forceinline__ T ld_uv_stream(const void* ubase, unsigned voff) {
  return *(const T*)((const char*)ubase + voff);
}
template <class T>
__device__ __forceinline__ void st_uv_stream(void* ubase, unsigned voff, T v) {
  *(T*)((char*)ubase + voff) = v;
}
// H = NG * NW * HPW heads in NG groups; NW waves per workgroup, HPW heads per wave; FS hidden
// k-steps of the FFN; RS slices of 16 query rows per workgroup (RS > 1 needs HPW = 1).
//
// Row slices.  A workgroup owns R = 16 RS query rows.  The K_LR / V operands of a tile of 32 keys
// are loaded once and used for all RS slices, one slice per step: a step is what the pipeline
// above calls a tile (stage A on the A_{n-1} piece of 16 rows x 32 keys, stage B for the same
// rows), and the steps of a tile run through its slices in order.  What a compute unit fetches
// per position for K_LR and V falls with 1 / RS, and so does what leaves the L2: row blocks do not
// share their K_LR / V tiles in the L2 in practice (the streams of A_{n-1} and A_n flush it within
// a few tiles; measured fetch = one K_LR / V tile per workgroup and tile), so HBM traffic is
// Hkv * 320 / R bytes per position on top of the 4 H bytes of the two score tensors.
// A slice is skipped in the tiles that none of its rows can see (beyond its own diagonal).
//
// A unit of work is (row block of R rows, key split); units are numbered by length.
// Grid: one dimension.  Workgroup ids go round robin over the 8 XCDs, each with its own L2 and 32
// compute units.  The ids of one XCD are dealt in chunks of 32 / NG neighbouring units of one
// sequence times NG head groups: the workgroups that fill one XCD start together and carry nearly
// the same number of tiles, so they walk the keys side by side.  The NG head groups of a row block
// then find the A_{n-1} tile, and the row blocks of a head group the K_LR / V tiles, in the L2
// after the first of them has fetched it from HBM.  With a.pair the workgroup takes the units (last - x) and x, a
// long and a short one, so that all workgroups carry the same number of tiles and stage the FFN
// weights once.
// Requires Lk % 8 == 0.
// SHG > 0: every SHG consecutive heads of a wave share one key/value head (grouped KV heads, H / Hkv
// a multiple of SHG, HPW a multiple of SHG): one set of K_LR / V operands per tile serves all of
// them, and every such set is refilled behind its last head with the next tile's operands.  With
// NG = 1 and 32 heads (XSTG below) the whole layer of a row block runs in one workgroup: the FFN is
// computed once, the A_{n-1} tile is read once, and a wave issues 10 operand loads per tile and
// key/value head for four query heads.
// FTRIM: F <= 32 FS - 16, the last 16 hidden units are padding and their products are left out
// (the 40 -> 80 -> 40 network of the LLaMA2-13B shape: 10 instead of 12 MFMAs of the first layer).
template <int NG, int FS, int HPW, int NW, int ACT = 0, int RS = 1, int SHG = 0, bool FTRIM = false>
__global__ __launch_bounds__(NW * 64) void k_lisa_prefill_fused(PrefillArgs a) {
  static_assert(RS == 1 || HPW == 1, "row slices: one head per wave");
  // XSTG: the A_{n-1} piece is double buffered by tile parity and the buffers double as the staging
  // tiles of A_n (a wave loads the A_{n-1} rows of its own heads, so it alone touches those parts
  // between the barriers): the 32 heads' own staging tiles would not fit the LDS.
  constexpr bool SHKV = SHG > 0;
  static_assert(!SHKV || HPW % SHG == 0, "whole key/value head groups per wave");
  constexpr bool XSTG = NG == 1 && HPW * NW == 32;
  static_assert(!XSTG || RS == 1, "one row slice with all heads in one workgroup");
  constexpr int DK = 128;
  constexpr int THREADS = NW * 64;
  constexpr int GH = NW * HPW;                       // heads of this workgroup's group
  constexpr int H = NG * GH;
  constexpr int R = PF_ROWS * RS;                    // query rows of this workgroup
  constexpr int HB = (H + 15) / 16;
  constexpr int HBO = (GH + 15) / 16;
  typedef MfmaFfn<HB, FS, HBO, ACT> Ffn;
  constexpr int KS = Ffn::KS;
  constexpr int XCH = NG * HPW;                      // A_{n-1} chunks per lane: heads wv + NW u
  constexpr int NBW = ((2 * PF_ROWS + NW - 1) / NW + 1) / 2 * 2;   // position blocks per wave in stage A (even)
  extern __shared__ __align__(16) unsigned char pf_lds[];
  const int Lq = a.Lq, Lk = a.Lk;
  unsigned char* xs = pf_lds;                               // A_{n-1} piece, half
  unsigned char* ys = xs + (XSTG ? 2 : 1) * H * PF_XS_HEAD; // y piece of the group, float
  unsigned short* w_s = (unsigned short*)(ys + GH * PF_YS_HEAD);
  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform
  unsigned char* as_ = (unsigned char*)w_s + Ffn::kStageBytes + wv * (HPW * RS) * PF_AS_HEAD;   // this wave's A_n staging
  const int c = lane & 15, g = lane >> 4;
  const int shift = Lk - Lq;                                // key j visible to row i iff j <= i + shift
  const int group = H / a.Hkv;
  const float LOG2E = 1.4426950408889634f;
  const int n_units = (Lq + R - 1) / R * a.split;
  // workgroup id -> (XCD, chunk of PF_CHUNK(NG) neighbouring slots of one sequence, slot in the chunk, head group)
  const int n_slots = a.pair ? (n_units + 1) / 2 : n_units;
  int slot, b, grp;
  {
    constexpr int CHU = pf_chunk_units(NG);
    const int i = blockIdx.x, x = i & 7, j = i >> 3;
    grp = j % NG;
    const int jj = j / NG;                                   // position among this XCD's workgroups
    const int chunk = (jj / CHU) * 8 + x;                    // chunks go round robin over the XCDs, long first
    const int n_chunks = (n_slots + CHU - 1) / CHU;
    if (chunk >= n_chunks * a.B) return;
    b = chunk % a.B;
    slot = (chunk / a.B) * CHU + jj % CHU;
    if (slot >= n_slots) return;
  }
  const int hg0 = grp * GH;                                 // first head of the group
  const int h_first = hg0 + wv * HPW;

  Ffn::stage(a.w1, a.w2, H, a.F, w_s, tid, THREADS, hg0, GH);
  // One head per wave, or two with shared operands, leave registers for the FFN weights: fetched
  // once per workgroup instead of read from LDS, each read followed by a wait, by every block
  // pair (5 % on the LLaMA3-8B shape once the score tensors are tiled; nothing before that, when
  // the layer waited for HBM).
  constexpr bool WREG = (HPW == 1 || (SHKV && HPW == 2)) && RS == 1 && NW <= 8 && (Ffn::FB * Ffn::KS + HBO * FS) <= 8;
  // blocks of 16 positions whose MFMA chains are interleaved in stage A (one at a time where the
  // accumulators of four row slices leave no registers for a second chain)
  constexpr int NBLK = RS >= 4 ? 1 : 2;
  Ffn ffn;
  if (WREG) {
    __syncthreads();
    ffn.fetch(w_s);
  }

  // score tensors.  Row-major: head h of sequence b starts at (b H + h) Lq Lk.  Tiled: tile (rb, kt)
  // of sequence b holds the H pieces of 16 rows x 32 keys one after the other, 1 KB each -- what a
  // workgroup reads per step is one run of H KB, in one page of the address translation (with a
  // tensor per head the 32 + 16 pieces of a step lay in as many pages and every step missed in the
  // translation cache of the compute unit for most of them: 36 misses per step).
  const int n_rb = (Lq + PF_ROWS - 1) / PF_ROWS, n_kt = (Lk + PF_TK - 1) / PF_TK;
  constexpr int TILE_ELEMS = PF_ROWS * PF_TK;
  const size_t head_elems = a.tiled ? (size_t)TILE_ELEMS : (size_t)Lq * Lk;                 // head stride
  const size_t seq_elems = a.tiled ? (size_t)n_rb * n_kt * H * TILE_ELEMS : (size_t)H * Lq * Lk;
  const size_t tile_stride = (size_t)H * TILE_ELEMS;        // tiled: elements from one (rb, kt) to the next
  // wave-uniform bases of this wave's heads (scalar registers)
  const bf16_t* k_base[HPW];     // K_LR rows of the head's key/value head
  const bf16_t* v_base[HPW];     // V chunks of it
  half_t* s_base[HPW];           // A_n of the head
#pragma unroll
  for (int hh = 0; hh < HPW; ++hh) {
    const int h = h_first + hh, kv = h / group;
    k_base[hh] = a.kp + ((size_t)b * a.Hkv + kv) * a.Lkp * 32;
    v_base[hh] = a.vt + ((size_t)b * a.Hkv + kv) * (a.Lkp / 8) * (DK * 8);
    s_base[hh] = a.scores ? a.scores + (size_t)b * seq_elems + (size_t)h * head_elems : nullptr;
  }
  const half_t* x_base[XCH];     // A_{n-1} of head wv + NW u (XSTG: of the wave's own heads)
#pragma unroll
  for (int u = 0; u < XCH; ++u)
    x_base[u] = a.prev + (size_t)b * seq_elems + (size_t)(XSTG ? wv * HPW + u : wv + NW * u) * head_elems;
  // per-lane byte offsets, the same for every head
  const unsigned k_off = ((8 * (c >> 2) + (c & 3)) * 32 + 8 * g) * 2;   // MFMA row c -> key 8 (c/4) + c%4 (+4)
  const unsigned v_off = (g * DK + c) * 16;                             // key chunk g, feature c (+16 nb)
  const int xq8 = 8 * (lane & 3);                                       // A_{n-1} chunk: row lane/4, 8 keys
  const int xdst = (XSTG ? wv * HPW : wv) * PF_XS_HEAD + lane * 16;     // + u NW PF_XS_HEAD (XSTG: + u PF_XS_HEAD)

  // LDS addresses of stage A (per lane, step independent)
  int xrd[KS][2];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    // transposing LDS read: lane s = 4 k' + q4 of a 16-lane group passes the address of head k',
    // keys 4 q4 .. 4 q4 + 3; it receives key c of heads k' = 0..3.
    xrd[ks][0] = min(32 * ks + 8 * g + (c >> 2), H - 1) * PF_XS_HEAD + 8 * (c & 3);
    xrd[ks][1] = min(32 * ks + 8 * g + 4 + (c >> 2), H - 1) * PF_XS_HEAD + 8 * (c & 3);
  }

  for (int rep = 0; rep < 2; ++rep) {
    int unit;
    if (a.pair) {
      unit = rep ? slot : n_units - 1 - slot;
      if (rep && unit >= n_units - 1 - unit) break;         // the middle unit of an odd count is alone
    } else {
      if (rep) break;
      unit = n_units - 1 - slot;                             // long units first
    }
    // Row block and key split.  The key tiles are dealt in pairs (64 keys = one 128-byte line of a
    // score row): split sp takes the pairs sp, sp + split, ...; the longer share comes later in
    // the unit numbering.
    const int rb = unit / a.split, sp = a.split - 1 - unit % a.split;
    const int i0 = rb * R;
    const int i_last = min(i0 + R - 1, Lq - 1);
    // (a slice without rows, in the last row block of a ragged Lq, runs on copies of row Lq - 1 and
    // stores nothing: "last slice of a tile" stays a compile-time property, and with it the place
    // where the tile's operands are refilled -- a load behind a run-time branch would make every
    // later wait for an older load a wait for everything)
    constexpr int rs_last = RS - 1;
    const int n_keys = a.causal ? min(Lk, i_last + 1 + shift) : Lk;
    const int n_tiles_all = (n_keys + PF_TK - 1) / PF_TK;
    const int n_mine = n_tiles_all / (2 * a.split) * 2 + min(max(n_tiles_all % (2 * a.split) - 2 * sp, 0), 2);
    if (n_mine == 0) continue;                                 // empty share (short row block)
    // The first unit of a workgroup walks its tiles upwards, the second one downwards.
    auto tile_at = [&](int it) {
      const int k = rep ? n_mine - 1 - it : it;
      return 2 * (sp + a.split * (k >> 1)) + (k & 1);
    };
    const int t_begin = tile_at(0);
    // first slice of which some row sees a key of the tile (the slices after it do too)
    auto rs_min = [&](int tile) {
      int r0 = 0;
      if (RS > 1 && a.causal) {
#pragma unroll
        for (int rs = 0; rs + 1 < RS; ++rs)
          if (tile * PF_TK > min(i0 + PF_ROWS * rs + PF_ROWS - 1, Lq - 1) + shift) r0 = rs + 1;
      }
      return min(r0, rs_last);
    };
    // tiles of slice rs whose 32 keys are visible to all its 16 rows (and all 16 rows exist) need no masking
    auto n_full_of = [&](int rs) {
      const int f = i0 + PF_ROWS * rs;
      return (f + PF_ROWS <= Lq) ? (a.causal ? min(Lk, f + 1 + shift) : Lk) / PF_TK : 0;
    };
    // last tile that slice rs takes part in
    auto last_tile_of = [&](int rs) {
      const int l = min(i0 + PF_ROWS * rs + PF_ROWS - 1, Lq - 1);
      return (a.causal ? min(Lk, l + 1 + shift) - 1 : Lk - 1) / PF_TK;
    };

    // ---- A_{n-1} piece: lane -> XCH chunks (head wv + NW u, row lane / 4, 8 keys) of 16 bytes ------
    // Row-major scores: the piece of a head is 16 half lines (64 bytes of 16 rows).  The L2 fetches
    // whole 128-byte lines, and the other half of each is wanted one tile later, by when the line
    // has usually left the L2 again: A_{n-1} was measured to come from HBM 2.5 times (22 GB on the
    // LLaMA3-8B shape at L = 8192; a 4-byte load of the other half issued next to each piece, to have
    // it fetched once, changed little).  Tiled scores: the piece is 1 KB of consecutive memory.
    auto load_x = [&](int tile, int rs, pf_u32x4 (&xr)[XCH]) {
      unsigned off;
      size_t at = 0;                                          // wave-uniform element offset of the tile
      if (a.tiled) {
        at = ((size_t)min((i0 >> 4) + rs, n_rb - 1) * n_kt + tile) * tile_stride;
        off = lane * 16;
      } else {
        const unsigned x_row = (unsigned)min(i0 + PF_ROWS * rs + (lane >> 2), Lq - 1) * Lk * 2;
        // keys >= Lk: any in-bounds chunk will do, those positions are masked in stage B
        off = x_row + 2 * min(tile * PF_TK + xq8, Lk - 8);
      }
#pragma unroll
      for (int u = 0; u < XCH; ++u) xr[u] = ld_uv_stream<pf_u32x4>(x_base[u] + at, off);
    };
    auto store_x = [&](const pf_u32x4 (&xr)[XCH], int tile) {   // XSTG: into the buffer of the tile's parity
      unsigned char* dst = xs + (XSTG ? (tile & 1) * (H * PF_XS_HEAD) : 0) + xdst;
#pragma unroll
      for (int u = 0; u < XCH; ++u) *(pf_u32x4*)(dst + u * ((XSTG ? 1 : NW) * PF_XS_HEAD)) = xr[u];
    };

    // ---- per-head, per-slice state of stage B ---------------------------------------------------------
    // A_n leaves through LDS in whole 128-byte pieces of a row (64 keys = two tiles): lane ->
    // rows lane / 8 and lane / 8 + 8 of the slice, keys 8 (lane % 8) .. + 7 of the pair of tiles
    f32x4 o[HPW * RS][DK / 16];
    float m_run[HPW * RS], l_run[HPW * RS];
    // PERSIST: every head keeps its own operand registers; each is refilled right after its use
    // with the same head's next tile, so the load has a whole tile period to arrive.  Otherwise
    // (register file too small) one rotating set, refilled for the head that stage B handles next.
    constexpr bool PERSIST = (HPW <= 2 && NW <= 8) || SHKV;
    constexpr int SH = SHKV ? SHG : 1;                         // heads per operand set
    constexpr int NSET = PERSIST ? HPW / SH : 1;
    // SPREAD: the V operands of the second head are loaded during stage A of their own tile
    // instead of right after their use: the compute unit's load pipe, which every wave fills at
    // the same time in stage B, then also works during stage A.
    constexpr bool SPREAD = PERSIST && HPW == 2 && !SHKV;
    // QRES: the Q_LR operands of all slices stay in registers; with many slices the accumulators
    // need that room and the operand of a step is loaded at the start of its stage A instead
    constexpr bool QRES = RS <= 2;
    bf16x8 qop[QRES ? HPW * RS : HPW], ka[NSET], kb[NSET], vop[NSET][DK / 16];
    const bf16_t* q_head = a.qp + ((size_t)b * H + h_first) * a.Lqp * 32;   // + hh Lqp 32
#pragma unroll
    for (int hh = 0; hh < HPW; ++hh) {
#pragma unroll
      for (int rs = 0; rs < RS; ++rs) {
        m_run[hh * RS + rs] = -INFINITY;
        l_run[hh * RS + rs] = 0.f;
#pragma unroll
        for (int nb = 0; nb < DK / 16; ++nb) o[hh * RS + rs][nb] = f32x4{0.f, 0.f, 0.f, 0.f};
        const int qrow = min(i0 + PF_ROWS * rs + c, a.Lqp - 1);
        if (QRES) qop[hh * RS + rs] = *(const bf16x8*)(q_head + ((size_t)hh * a.Lqp + qrow) * 32 + 8 * g);
      }
      if (hh >= NSET) continue;                                // (hh here numbers the operand sets)
      const bf16_t* kt = k_base[hh * SH] + (size_t)t_begin * (PF_TK * 32);
      ka[hh] = ld_uv<bf16x8>(kt, k_off);
      kb[hh] = ld_uv<bf16x8>(kt, k_off, 4 * 32 * 2);
      if (SPREAD && hh == 1) continue;
      const bf16_t* vt = v_base[hh * SH] + (size_t)t_begin * (PF_TK / 8 * DK * 8);
#pragma unroll
      for (int nb = 0; nb < DK / 16; ++nb) vop[hh][nb] = ld_uv<bf16x8>(vt, v_off, nb * 256);
    }

    // The A_{n-1} piece of the next step travels in xr through stage B: loaded during stage A,
    // written to LDS at the end of stage B.  (With the tile already in the L2 the layer runs 8 %
    // faster at L = 8192 and 20 % faster at L = 2048, so the load from HBM is not fully covered;
    // a second register set, loaded two tiles ahead, gained 4 % with one head per wave and cost
    // more than that in spilled registers with two: loads complete in order, so the younger
    // K_LR / V loads wait for it anyway.)
    pf_u32x4 xr[XCH];
    load_x(t_begin, rs_min(t_begin), xr);
    store_x(xr, t_begin);
    // Stores of a staged pair of A_n tiles (head hh, slice rs of this wave); pending[rs] = last
    // tile of a pair whose stores are still to be issued.  They go out during stage A of the
    // slice's next step: all waves of a workgroup run the same stage at the same time, stage B is
    // where the operand loads crowd the load / store pipe of the compute unit and stage A is where
    // it has room.
    int pending[RS];
#pragma unroll
    for (int rs = 0; rs < RS; ++rs) pending[rs] = -1;
    auto flush_scores = [&](int tile, int hh, int rs) {
      const int jp = (tile >> 1) * (2 * PF_TK);               // first key of the pair
      const bool pair_full = (tile | 1) < n_full_of(rs);      // workgroup-uniform
      const int jc = jp + 8 * (lane & 7);
      half_t* st = s_base[hh] + jp;
      if (a.tiled) {
        // each staged tile of the pair is 1 KB of consecutive memory: lane -> row lane / 4, 16
        // bytes; what lies above the diagonal inside a stored tile is unspecified
        if (i0 + PF_ROWS * rs >= Lq) return;                 // (a slice without rows)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const int tl = (tile & ~1) + u;
          if (tl > last_tile_of(rs)) continue;                // the last pair of a row block may be half
          const unsigned char* sp =
              XSTG ? xs + u * (H * PF_XS_HEAD) + (wv * HPW + hh) * PF_XS_HEAD + (lane >> 2) * (2 * PF_TK) + (lane & 3) * 16
                   : as_ + (hh * RS + rs) * PF_AS_HEAD + (lane >> 2) * PF_AS_ROW + u * 64 + (lane & 3) * 16;
          const size_t at = ((size_t)((i0 >> 4) + rs) * n_kt + tl) * tile_stride;   // wave-uniform
          st_uv_stream<f16x8>(s_base[hh] + at, lane * 16, *(const f16x8*)sp);
        }
        return;
      }
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int gi = i0 + PF_ROWS * rs + (lane >> 3) + 8 * u;
        const unsigned a_off = ((unsigned)min(gi, Lq - 1) * Lk + 8 * (lane & 7)) * 2;
        const int a_vis = gi < Lq ? (a.causal ? min(Lk, gi + 1 + shift) : Lk) : 0;
        // XSTG: keys 0..31 of the pair lie in the even buffer, 32..63 in the odd one
        const unsigned char* sp =
            XSTG ? xs + ((lane >> 2) & 1) * (H * PF_XS_HEAD) + (wv * HPW + hh) * PF_XS_HEAD +
                       ((lane >> 3) + 8 * u) * (2 * PF_TK) + (lane & 3) * 16
                 : as_ + (hh * RS + rs) * PF_AS_HEAD + ((lane >> 3) + 8 * u) * PF_AS_ROW + (lane & 7) * 16;
        if (pair_full || jc + 8 <= a_vis) {
          st_uv_stream<f16x8>(st, a_off, *(const f16x8*)sp);
        } else if (jc < a_vis) {
          // a piece that straddles the row's last visible key (diagonal tiles only): the entries
          // beyond it keep what memory holds -- read, merge, write back; every piece has one writer.
          // (Element-wise stores kept eight addresses per piece alive across the whole tile loop.)
          const f16x8 old = ld_uv<f16x8>(st, a_off);
          f16x8 hv = *(const f16x8*)sp;
          int rel = a_vis - jc;                   // kept inside this branch: the eight compares
          asm volatile("" : "+v"(rel));           // were hoisted into every pass of the tile loop
#pragma unroll
          for (int e = 1; e < 8; ++e)
            if (e >= rel) hv[e] = old[e];
          st_uv<f16x8>(st, a_off, hv);
        }
      }
    };

    // Everything loaded so far has arrived before the loop is entered: the wait counts inside the
    // loop then follow from the loop's own issue order alone (a load pending on entry would cap
    // them at what the first pass needs and drain the prefetch on every pass).
    __builtin_amdgcn_s_waitcnt(0x0F70);                       // vmcnt(0), others untouched
    for (int it = 0; it < n_mine; ++it) {
      const int tile = tile_at(it);
      const int j0 = tile * PF_TK;
      const int tile_n = tile_at(min(it + 1, n_mine - 1));      // next tile (clamped: loads stay valid)
      const int rs_first = rs_min(tile), rs_first_n = rs_min(tile_n);
#pragma unroll
      for (int rs = 0; rs < RS; ++rs) {
      if (RS > 1 && rs < rs_first) continue;                   // workgroup-uniform: no row of the slice sees the tile
      const bool last_slice = RS == 1 || rs == rs_last;        // the tile's operands are used up after this step
      // the step after this one: the next slice of the tile, else the first slice of the next tile
      const int x_tile = last_slice ? tile_n : tile, x_rs = last_slice ? rs_first_n : rs + 1;
      unsigned char* xs_t = xs + (XSTG ? (tile & 1) * (H * PF_XS_HEAD) : 0);   // this tile's A_{n-1} buffer
      lds_barrier();                                                       // B1
      if (!QRES) {
        const unsigned qoff = ((unsigned)min(i0 + PF_ROWS * rs + c, a.Lqp - 1) * 32 + 8 * g) * 2;
#pragma unroll
        for (int hh = 0; hh < HPW; ++hh) qop[hh] = ld_uv<bf16x8>(q_head + (size_t)hh * a.Lqp * 32, qoff);
      }
      // ---- stage A: y = FFN(A_{n-1}) for this wave's blocks of 16 positions ----------------------
      // two blocks of 16 positions at a time, their MFMA chains interleaved; the weights are read
      // from LDS as the products need them (stage B keeps the register file)
#pragma unroll
      for (int q = 0; q < NBW; q += NBLK) {
        if (!XSTG && pending[rs] >= 0) {
          // heads of this wave dealt over the block pairs
#pragma unroll
          for (int hh = q / NBLK; hh < HPW; hh += NBW / NBLK) flush_scores(pending[rs], hh, rs);
        }
        if (q + NBLK >= NBW) load_x(x_tile, x_rs, xr);
        if (SPREAD) {
          constexpr int PER = (DK / 16 + NBW / NBLK - 1) / (NBW / NBLK);    // V loads per block group
          const bf16_t* vt = v_base[HPW - 1] + (size_t)tile * (PF_TK / 8 * DK * 8);
#pragma unroll
          for (int nb = q / NBLK * PER; nb < min(q / NBLK * PER + PER, DK / 16); ++nb)
            vop[NSET - 1][nb] = ld_uv<bf16x8>(vt, v_off, nb * 256);
        }
        f16x8 x[NBLK][KS];
        int yoff[NBLK];
#pragma unroll
        for (int n = 0; n < NBLK; ++n) {
          // block = (row i, key half kh); a wave with an odd share repeats its last block
          const int nb = min(wv + (q + n) * NW, 2 * PF_ROWS - 1);
          const int i = nb >> 1, kh = nb & 1;
          yoff[n] = i * PF_YS_ROW + (16 * kh + c) * 4;
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) {
            const f16x4 lo = __builtin_bit_cast(
                f16x4, __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                           (s16x4 __attribute__((address_space(3)))*)(xs_t + xrd[ks][0] + i * 64 + 32 * kh)));
            const f16x4 hi = __builtin_bit_cast(
                f16x4, __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                           (s16x4 __attribute__((address_space(3)))*)(xs_t + xrd[ks][1] + i * 64 + 32 * kh)));
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
        f32x4 y[NBLK][HBO];
        if (WREG) ffn.template apply<NBLK>(x, y);
        else Ffn::template apply_lds<NBLK, FTRIM>(w_s, x, y);
#pragma unroll
        for (int n = 0; n < NBLK; ++n)
#pragma unroll
          for (int hb = 0; hb < HBO; ++hb)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              const int hl = 16 * hb + 4 * g + v;
              if (GH % 16 == 0 || hl < GH) *(float*)(ys + hl * PF_YS_HEAD + yoff[n]) = y[n][hb][v];
            }
      }
      pending[rs] = -1;
      lds_barrier();                                                       // B2

      // ---- stage B: per head scores, softmax, P V ------------------------------------------------
      const bool full = tile < n_full_of(rs);                   // workgroup-uniform
      const int jl = j0 + 8 * g;                                // first of my 8 keys
      const int my_row = min(i0 + PF_ROWS * rs + c, Lq - 1);    // clamped; stores check the row itself
      const int vis_row = a.causal ? min(Lk, my_row + 1 + shift) : Lk;   // keys visible to my row
#pragma unroll
      for (int hh = 0; hh < HPW; ++hh) {
        const int sl = hh * RS + rs;                                   // accumulator slot
        if (HPW * RS > 2) __builtin_amdgcn_sched_barrier(0);           // keep the heads' chains apart: registers
        // low-rank scores for keys j0 + 8 g + e of row c
        const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
        const int hs = PERSIST ? hh / SH : 0;                          // operand set in use
        const int hn = PERSIST ? hh / SH * SH : (hh + 1 < HPW ? hh + 1 : 0);   // head it is refilled for
        const int t_next = PERSIST || hh + 1 == HPW ? tile_n : tile;
        // (shared operands are refilled behind the last head that uses them)
        const bool refill = (RS == 1 || last_slice) && (hh + 1) % SH == 0;   // compile time
        const bf16x8 qo = qop[QRES ? sl : hh];
        const f32x4 s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[hs], qo, zero, 0, 0, 0);
        const f32x4 s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kb[hs], qo, zero, 0, 0, 0);
        if (refill) {
          const bf16_t* kt = k_base[hn] + (size_t)t_next * (PF_TK * 32);
          ka[hs] = ld_uv<bf16x8>(kt, k_off);
          kb[hs] = ld_uv<bf16x8>(kt, k_off, 4 * 32 * 2);
        }
        const float* yp = (const float*)(ys + (wv * HPW + hh) * PF_YS_HEAD + c * PF_YS_ROW + 8 * g * 4);
        const f32x4 y0 = *(const f32x4*)yp, y1 = *(const f32x4*)(yp + 4);
        float an[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          an[e] = s0[e] * a.dscale + y0[e];
          an[4 + e] = s1[e] * a.dscale + y1[e];
        }
        // A_n for the next layer: into this wave's staging tile, stored at the end of the stage
        if (a.scores) {
          f16x8 hv;
#pragma unroll
          for (int e = 0; e < 8; ++e) hv[e] = f32_to_half_sat(an[e]);
          if (a.tiled && !XSTG) {
            // tiled scores: the lane's 8 keys of row c are 16 bytes of the head's KB and leave from
            // the registers (through the staging tile, which row-major scores need to pair two
            // tiles into whole lines, the layer took 1 - 3 % longer)
            if (i0 + PF_ROWS * rs < Lq) {
              const size_t at = ((size_t)((i0 >> 4) + rs) * n_kt + tile) * tile_stride;   // wave-uniform
              // (a non-temporal store: 1 - 6 % on the three benchmark shapes)
              __builtin_nontemporal_store(__builtin_bit_cast(pf_u32x4, hv),
                                          (pf_u32x4*)((char*)(s_base[hh] + at) + (unsigned)(c * 64 + g * 16)));
            }
          } else if (XSTG) *(f16x8*)(xs_t + (wv * HPW + hh) * PF_XS_HEAD + c * (2 * PF_TK) + g * 16) = hv;
          else *(f16x8*)(as_ + sl * PF_AS_HEAD + c * PF_AS_ROW + (tile & 1) * 64 + g * 16) = hv;
        }
        // online softmax, statistics of row c kept by all four lanes 16 g + c; exponentials in
        // base 2: p = 2^(A log2(e) - m log2(e))
        if (!full) {                              // workgroup-uniform: only diagonal / ragged tiles mask
          int rel = vis_row - jl;                 // the compares stay inside the branch
          asm volatile("" : "+v"(rel));
#pragma unroll
          for (int e = 0; e < 8; ++e)
            if (e >= rel) an[e] = -INFINITY;
        }
        const float mx = max2_raw(max3_raw(max3_raw(max3_raw(an[0], an[1], an[2]), an[3], an[4]), an[5], an[6]), an[7]);
        const float m_new = rows_max(mx, m_run[sl]);
        // A row may have seen no key yet: a key share, a walk downwards from the diagonal, or a
        // slice at its own diagonal can meet a tile that lies wholly beyond the row's last visible
        // key.  The exponent is then taken against 0 instead of -inf, so alpha and every p are
        // exactly 0 and the row's state stays (m = -inf, l = 0, o = 0).
        const float m2 = (m_new == -INFINITY ? 0.f : m_new) * LOG2E;
        const float alpha = fast_exp2(m_run[sl] * LOG2E - m2);
        m_run[sl] = m_new;
        float ps = 0.f;
        bf16x8 pop;
        // SPREAD: the V operands of the first head for the next tile are loaded here, one load
        // per exponential of the second head (its registers are free since the first head's P V)
        const bf16_t* v0n = v_base[0] + (size_t)tile_n * (PF_TK / 8 * DK * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          if (SPREAD && hh == 1) vop[0][e] = ld_uv<bf16x8>(v0n, v_off, e * 256);
          const float p = fast_exp2(__builtin_fmaf(an[e], LOG2E, -m2));
          ps += p;
          pop[e] = (__bf16)p;                     // hardware round-to-nearest-even conversion
          if (SPREAD && hh == 1) __builtin_amdgcn_sched_barrier(0);
        }
        l_run[sl] = l_run[sl] * alpha + ps;       // partial sum over my keys; groups merged at the end
        if (__any(alpha != 1.f)) {                // wave-uniform: the running maximum rarely moves
#pragma unroll
          for (int nb = 0; nb < DK / 16; ++nb)
#pragma unroll
            for (int v = 0; v < 4; ++v) o[sl][nb][v] *= alpha;
        }
        const bf16_t* vt = v_base[hn] + (size_t)t_next * (PF_TK / 8 * DK * 8);
#pragma unroll
        for (int nb = 0; nb < DK / 16; ++nb) {
          o[sl][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop[hs][nb], pop, o[sl][nb], 0, 0, 0);
          if (!SPREAD && refill) vop[hs][nb] = ld_uv<bf16x8>(vt, v_off, nb * 256);
        }
      }
      // A_n is written once both tiles of a pair are staged (64-byte pieces of a line reach HBM at
      // half the rate of whole lines): after the odd tile when walking upwards (or after the
      // slice's last tile, which may have no partner), after the even tile when walking downwards.
      if (a.scores && (XSTG || !a.tiled) && (rep ? (tile & 1) == 0 : ((tile & 1) == 1 || tile >= last_tile_of(rs)))) pending[rs] = tile;
      if (XSTG && pending[rs] >= 0) {
        // the pair sits in the two A_{n-1} buffers, which the next pieces are about to overwrite
#pragma unroll
        for (int hh = 0; hh < HPW; ++hh) flush_scores(pending[rs], hh, rs);
        pending[rs] = -1;
      }
      // every wave left stage A of this step, the last reader of xs, before B2; stage A of the
      // next step reads the new piece after B1
      store_x(xr, x_tile);
      }
    }
#pragma unroll
    for (int rs = 0; rs < RS; ++rs) {
      if (pending[rs] >= 0) {
#pragma unroll
        for (int hh = 0; hh < HPW; ++hh) flush_scores(pending[rs], hh, rs);
      }
    }

    // ---- epilogue ----------------------------------------------------------------------------------
    if (a.split > 1) {
      // unnormalised partial (o, m, l) of this key share; k_prefill_combine merges the shares
      // (RS = 1 only: the host never splits the keys of wider row blocks)
#pragma unroll
      for (int hh = 0; hh < HPW; ++hh) {
        const int h = h_first + hh;
        const float l = rows_sum(l_run[hh * RS]);
        const size_t row = (((size_t)sp * a.B + b) * a.Lqp + i0 + c) * H + h;
        if (g == 0) {
          a.part_ml[row * 2] = m_run[hh * RS];
          a.part_ml[row * 2 + 1] = l;
        }
#pragma unroll
        for (int nb = 0; nb < DK / 16; ++nb) {
          const f32x4 acc = o[hh * RS][nb];
          *(float4*)(a.part_o + row * DK + nb * 16 + 4 * g) = make_float4(acc[0], acc[1], acc[2], acc[3]);
        }
      }
      continue;
    }
    // O[row][h][d] = o / l
#pragma unroll
    for (int hh = 0; hh < HPW; ++hh) {
#pragma unroll
      for (int rs = 0; rs < RS; ++rs) {
        const int h = h_first + hh, sl = hh * RS + rs;
        const float inv = 1.f / rows_sum(l_run[sl]);
        const int row = i0 + PF_ROWS * rs + c;
        if (row < Lq) {
          const size_t at = (((size_t)b * Lq + row) * H + h) * DK + 4 * g;
#pragma unroll
          for (int nb = 0; nb < DK / 16; ++nb) {
            const f32x4 acc = o[sl][nb];
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
  }
}


// Merges the key-split partials of k_lisa_prefill_fused: for every (b, row, h)
//   O = sum_s e^{m_s - M} o_s / sum_s e^{m_s - M} l_s,   M = max_s m_s   over the non-empty shares.
// grid (Lq, B), block 256; thread -> (head, 4 features) pairs.
__global__ __launch_bounds__(256) void k_prefill_combine(PrefillArgs a) {
  constexpr int DK = 128;
  const int i = blockIdx.x, b = blockIdx.y, H = a.H;
  const int rb = i / PF_ROWS;
  const int i_last = min(rb * PF_ROWS + PF_ROWS - 1, a.Lq - 1);
  const int n_keys = a.causal ? min(a.Lk, i_last + 1 + a.Lk - a.Lq) : a.Lk;
  const int n_tiles_all = (n_keys + PF_TK - 1) / PF_TK;
  const int n_used = min(a.split, (n_tiles_all + 1) / 2);             // non-empty shares (tile pairs)
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
