/*
 * lisa.h -- C ABI of the LiSA attention-layer library for AMD MI355X (gfx950).
 *
 * LiSA (cross-layer attention sharing) replaces the full-rank Q K^T of a layer by
 *   (1) the previous layer's pre-softmax scores A_{n-1}, re-aligned across heads by a
 *       small feed-forward network applied over the head axis at every (query, key)
 *       position (Sec. 5.1, "Learn to share attention weights"),
 *   (2) a low-rank correction A_delta = Q_LR K_LR^T / sqrt(r) (Sec. 5.1, Eq. 3),
 *   (3) Integrate(A_align, A_delta) (Eq. 4), followed by the usual softmax and P V of
 *       Sec. 2.1, Eq. 1-2.
 * A standard-attention entry point that emits the shared score tensor A (the bracketed
 * term of Eq. 2) is included, because a LiSA layer needs a producer for A_{n-1}.
 *
 * General rules for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller, valid on the device that
 *     is current when the call is made.  The descriptor pointer is a HOST pointer.  The
 *     library never allocates, frees or retains device memory.  (The one exception is the
 *     optional stage timing, lisa_profile_*, which creates HIP events and a host-side list.)
 *   - Calls only enqueue work on `hip_stream` (a hipStream_t cast to void*, NULL = the
 *     default stream) and return without synchronising.  Re-entrant; no state is shared between
 *     threads.  Per calling thread the library keeps diagnostics only: the text of the last HIP
 *     error, the name of the last kernel family, the stage-timing records and the test
 *     overrides of lisa_tune_set(), none of which a call needs.
 *   - Return value: 0 (LISA_OK) or a negative lisa_status.  All argument validation is
 *     done on the host before any HIP call, so a rejected call has touched nothing.
 *   - Tensors are dense, row-major, innermost index last, base pointers 16-byte aligned.
 *   - Element types: `dtype` is the type of Q, K, V, Q_LR, K_LR, W1, W2 and of the
 *     attention output O (float32 instead when out_f32 = 1: the accumulators are float32
 *     and rounding O to bfloat16 alone costs up to 2^-9 of each element).  Score tensors
 *     (A_{n-1}, A_n) use the *score type*:
 *     float32 when dtype = LISA_F32, IEEE binary16 (half) when dtype = LISA_BF16 -- the
 *     2-byte score element assumed by the memory analysis of Sec. 5.2, chosen as half
 *     because the softmax that consumes A needs absolute, not relative, precision.
 *   - Visibility: with causal = 1 query row i (0-based, of Lq) sees key j (of Lk) iff
 *     j <= i + (Lk - Lq); with causal = 0 every key is visible.  Score entries of
 *     invisible keys are never used and never written (a kernel may load a few of them inside
 *     an aligned 16-byte chunk of an allocated row and discard them).
 *   - Grouped KV heads: query head h uses KV head h / (H / Hkv).
 */
#ifndef LISA_H_
#define LISA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { LISA_F32 = 0, LISA_BF16 = 1 } lisa_dtype;

/* Integrate() of Eq. 4.  ADD:    A_n = FFN(A_{n-1}) + A_delta, FFN input width Din = H.
 *                        CONCAT: A_n = FFN([A_{n-1} ; A_delta]), Din = 2H, rows 0..H-1 of W1
 *                                act on A_{n-1} and rows H..2H-1 on A_delta (Sec. 5.1,
 *                                "An overview of LiSA"). */
/*                        Two variants without the alignment FFN (w1, w2, F are ignored):
 *                        PLUS:   A_n = A_{n-1} + A_delta (LiSA_plus for models pre-trained with
 *                                shared attention, Sec. 5.5);
 *                        SHARE:  A_n = A_{n-1}, the direct sharing the method starts from (DS,
 *                                Sec. 4; q_lr, k_lr, r are ignored as well).
 * MFMA kernels exist for ADD (fused prefill, split-context decode) and for CONCAT (scores kernel
 * + softmax / P V kernel in prefill, split-context decode), each with ReLU or SiLU.  A
 * single layer, PLUS and SHARE are served by them too (y = W^T x equals the two-layer ReLU
 * network [W,-W] then [I;-I], built in the workspace; SHARE with an all-zero correction).  Other
 * combinations and shapes run on the generic kernels. */
typedef enum { LISA_MIX_ADD = 0, LISA_MIX_CONCAT = 1, LISA_MIX_PLUS = 2, LISA_MIX_SHARE = 3 } lisa_mix;

/* The alignment FFN (Sec. 5.3 "Model configuration": two layers with ReLU; Sec. 5.7 ablates
 * SiLU, x * sigmoid(x), and a single layer).  SINGLE: A_align = W1^T x with W1 [Din,H]; F must
 * equal H and w2 is ignored. */
typedef enum { LISA_ACT_RELU = 0, LISA_ACT_SILU = 1, LISA_ACT_SINGLE = 2 } lisa_act;

typedef enum {
  LISA_OK = 0,
  LISA_ERR_NULL = -1,        /* a required pointer is NULL                              */
  LISA_ERR_SHAPE = -2,       /* a dimension is non-positive or inconsistent             */
  LISA_ERR_UNSUPPORTED = -3, /* valid request outside what the kernels implement        */
  LISA_ERR_ALIGN = -4,       /* a base pointer is not 16-byte aligned                   */
  LISA_ERR_WORKSPACE = -5,   /* workspace missing or smaller than lisa_workspace_bytes  */
  LISA_ERR_HIP = -6,         /* a HIP launch failed; see lisa_last_hip_error()          */
  LISA_ERR_SCRATCH = -7      /* lisa_attn_decode_static: needs more than the static scratch */
} lisa_status;

typedef enum {
  LISA_WS_PREFILL = 0, LISA_WS_DECODE = 1, LISA_WS_STD = 2, LISA_WS_LAYER = 3, LISA_WS_LAYER_DECODE = 4,
  LISA_WS_KD = 5
} lisa_ws_kind;

/* Problem descriptor (host memory, plain data, zero-initialise then fill). */
typedef struct lisa_desc {
  int32_t dtype;            /* lisa_dtype                                                     */
  int32_t B;                /* sequences in the batch                                         */
  int32_t H;                /* query heads (h of Sec. 2.1)                                    */
  int32_t Hkv;              /* key/value heads, divides H                                     */
  int32_t Lq;               /* query rows in this call (decode: 1)                            */
  int32_t Lk;               /* keys attended (decode: cached context + the new token)         */
  int32_t d_k;              /* head dimension of V (and of Q, K in std_attn_scores)           */
  int32_t r;                /* per-head low-rank dimension of Q_LR, K_LR (Eq. 3)              */
  int32_t F;                /* hidden width of the head-alignment FFN                         */
  int32_t mix;              /* lisa_mix                                                       */
  int32_t act;              /* lisa_act                                                       */
  float delta_scale;        /* scale of A_delta; 0 selects 1/sqrt(r)   (Eq. 3)                */
  float std_scale;          /* scale of the standard scores; 0 selects 1/sqrt(d_k) (Eq. 2)    */
  int32_t causal;           /* 1 causal, 0 full visibility                                    */
  int32_t write_scores;     /* lisa_*: 1 = emit A_n for the next layer                        */
  int32_t kcache_dim_major; /* decode: K_LR cache is [B,Hkv,r,Lmax] (1) or [B,Hkv,Lmax,r] (0) */
  int32_t Lmax;             /* decode: capacity of the caches along the key axis, >= Lk       */
  int32_t out_f32;          /* 1: the attention output O is written as float32 whatever dtype */
  int32_t score_tiled;      /* prefill score tensors: 0 = [B,H,Lq,Lk]; 1 = tiles, see below    */
} lisa_desc;

/*
 * Tiled score layout (score_tiled = 1; prefill calls of the bf16 matrix-core kernels only, other
 * requests return LISA_ERR_UNSUPPORTED).  A score tensor is then
 *     [B, ceil(Lq / 16), ceil(Lk / 32), H, 16, 32]     (lisa_scores_elems() elements)
 * i.e. tile (rb, kt) holds, head after head, rows 16 rb .. 16 rb + 15 and keys 32 kt .. 32 kt + 31 of
 * every head as 1 KB of consecutive memory each: what a workgroup of the LiSA layer reads per
 * step is one run of H KB.  In [B,H,Lq,Lk] the piece of a head is 16 separate half lines, each
 * fetched from HBM as a whole line and again one step later for its other half, and the pieces of
 * the H heads lie in H pages of the address translation; tiled, the layer moves a third fewer
 * bytes.
 * The standard layer writes this layout, the LiSA layer reads and writes it: the fused ADD kernels,
 * and the CONCAT form on the matrix cores up to 32 heads with d_k = 128 (its scores kernel reads
 * and writes tiles, the softmax / P V kernel behind it reads them).  Entries of a stored
 * tile that lie above the diagonal, beyond row Lq - 1 or beyond key Lk - 1 are unspecified; tiles
 * wholly above the diagonal are neither written nor read.
 */
#define LISA_SCORE_TILE_ROWS 16
#define LISA_SCORE_TILE_KEYS 32
/* Elements of one prefill score tensor of the descriptor in its layout (0 on a NULL descriptor). */
size_t lisa_scores_elems(const lisa_desc* desc);

/*
 * lisa_attn_prefill -- one LiSA attention layer over Lq query rows (Sec. 5.1, Eq. 3-4,
 * then Sec. 2.1 Eq. 1-2 without W^O).
 *   q_lr        [B,H,Lq,r]     in   low-rank queries  H W^Q_LR, split in heads
 *   k_lr        [B,Hkv,Lk,r]   in   low-rank keys     H W^K_LR
 *   v           [B,Hkv,Lk,d_k] in   values
 *   scores_prev [B,H,Lq,Lk]    in   A_{n-1}, score type
 *   w1 [Din,F], w2 [F,H]       in   FFN weights (no bias), dtype; NULL where the variant
 *                                   (lisa_mix, lisa_act) does not use them
 *   out         [B,Lq,H,d_k]   out  concatenated heads softmax(A_n) V, dtype
 *   scores_out  [B,H,Lq,Lk]    out  A_n, score type; required iff write_scores = 1; must not
 *                                   alias scores_prev
 *   workspace                  scratch of at least lisa_workspace_bytes(desc, LISA_WS_PREFILL)
 *                              bytes (may be NULL when that is 0); contents undefined after.
 *                              The fused kernels keep A_n in float32 registers up to the
 *                              softmax and the generic kernels stage it here as float32; the
 *                              matrix-core kernels of the CONCAT form pass it between their two
 *                              launches in the score type (the rounding its inputs carry).
 */
int lisa_attn_prefill(const lisa_desc* desc, const void* q_lr, const void* k_lr, const void* v,
                      const void* scores_prev, const void* w1, const void* w2, void* out,
                      void* scores_out, void* workspace, size_t workspace_bytes,
                      void* hip_stream);

/*
 * lisa_attn_decode -- the same layer for one new token per sequence against the caches
 * (Sec. 2.2 prefilling/decoding stages; Sec. 5.2: the cache holds K_LR instead of K).
 * Requires Lq = 1 and Lk <= Lmax.
 *   q_lr           [B,H,r]          in
 *   k_lr_new       [B,Hkv,r]        in   or NULL; when given it is stored at key index Lk-1
 *   v_new          [B,Hkv,d_k]      in   or NULL; likewise (both or neither)
 *   k_lr_cache     [B,Hkv,Lmax,r] or [B,Hkv,r,Lmax]   in/out (only index Lk-1 is written)
 *   v_cache        [B,Hkv,Lmax,d_k]                   in/out (only index Lk-1 is written)
 *   score_row_prev [B,H,Lk]         in   A_{n-1} row of the new token, score type
 *   out            [B,H,d_k]        out
 *   score_row_out  [B,H,Lk]         out  required iff write_scores = 1 (the "small weight
 *                                        matrix" of h*l elements in Sec. 5.2)
 */
int lisa_attn_decode(const lisa_desc* desc, const void* q_lr, const void* k_lr_new,
                     const void* v_new, void* k_lr_cache, void* v_cache,
                     const void* score_row_prev, const void* w1, const void* w2, void* out,
                     void* score_row_out, void* workspace, size_t workspace_bytes,
                     void* hip_stream);

/*
 * lisa_attn_decode_static -- lisa_attn_decode for callers that cannot allocate device memory and
 * have no workspace to hand over: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, same kernels and same results as lisa_attn_decode,
 * without the workspace: the partial results of the split-context kernels (and the operands that
 * the variants without a two-layer FFN synthesise) live in a buffer of LISA_STATIC_SCRATCH_BYTES
 * bytes that is part of the library's code object, one copy per GPU, held until the process ends.
 *   - The call makes no hipMalloc / hipFree and uses no allocating library routine; stage timing
 *     (lisa_profile_*) is off inside it.  The first call on a device resolves the address of that
 *     device's copy of the buffer (hipGetSymbolAddress); make that first call outside any capture.
 *   - A problem whose lisa_workspace_bytes(desc, LISA_WS_DECODE) exceeds LISA_STATIC_SCRATCH_BYTES
 *     is rejected with LISA_ERR_SCRATCH before any HIP call (B * ceil(Lk / 128) * H <= 32263 units
 *     at d_k = 128: e.g. 30 sequences of 32 heads at 4097 keys).
 *   - All calls on one GPU share that GPU's buffer and it keeps the last call's contents; every
 *     kernel writes what it later reads, so nothing needs clearing between calls.  Calls that can
 *     overlap on one GPU (different streams, or graphs replayed concurrently) race on it: the
 *     caller orders them.
 */
#define LISA_STATIC_SCRATCH_BYTES (16u << 20)
int lisa_attn_decode_static(const lisa_desc* desc, const void* q_lr, const void* k_lr_new,
                            const void* v_new, void* k_lr_cache, void* v_cache,
                            const void* score_row_prev, const void* w1, const void* w2, void* out,
                            void* score_row_out, void* hip_stream);

/*
 * lisa_decode_stack -- one decode step through the attention layers of a model in which some
 * layers share attention (Sec. 5.1, "Selecting layers to implement LiSA" and its table of
 * configurations; Sec. 4 for direct sharing): every layer is a standard layer, a LiSA layer or a
 * direct-sharing layer.  A sharing layer takes A_{n-1} from the layer in front of it, so the first
 * layer must be standard.  The score row travels from layer to layer inside the workspace; a
 * layer emits its row only if the next layer shares it (or the caller gives it a place).
 *   desc     the LiSA layers' descriptor (Lq = 1, Lk, Lmax, r, F, mix, act, kcache_dim_major, ...);
 *            standard layers use its B, H, Hkv, Lk, Lmax, d_k, std_scale, out_f32; write_scores is
 *            ignored.  mix must not be LISA_MIX_SHARE.
 *   layers   HOST array of n_layers entries, in layer order; device pointers inside:
 *     kind       LISA_LAYER_STD | LISA_LAYER_LISA | LISA_LAYER_SHARE
 *     q          STD: q [B,H,d_k]; LISA: q_lr [B,H,r]; SHARE: unused
 *     k_cache    STD: K cache [B,Hkv,Lmax,d_k]; LISA: K_LR cache (layout as in lisa_attn_decode);
 *                SHARE: unused.  The caches already hold the new token (index Lk-1).
 *     v_cache    [B,Hkv,Lmax,d_k]
 *     w1, w2     LISA: FFN weights as in lisa_attn_decode
 *     out        [B,H,d_k]  out  the layer's attention output
 *     score_row  [B,H,Lk]   out  or NULL: where to keep this layer's A_n (score type)
 *   workspace    at least lisa_stack_workspace_bytes(desc) bytes
 * All layers are enqueued on hip_stream in order; the call returns after the last launch.  The
 * partial results of a layer (split over the cached keys) are combined into its `out` by the
 * workgroups of the next layer's launch, the last layer's by a launch of their own: a layer's
 * `out` is complete when the call's work on the stream is, not before.
 */
typedef enum { LISA_LAYER_STD = 0, LISA_LAYER_LISA = 1, LISA_LAYER_SHARE = 2 } lisa_layer_kind;
typedef struct lisa_stack_layer {
  int32_t kind;      /* lisa_layer_kind */
  int32_t reserved;  /* 0 */
  const void* q;
  void* k_cache;
  void* v_cache;
  const void* w1;
  const void* w2;
  void* out;
  void* score_row;
} lisa_stack_layer;
int lisa_decode_stack(const lisa_desc* desc, const lisa_stack_layer* layers, int32_t n_layers,
                      void* workspace, size_t workspace_bytes, void* hip_stream);
/* Scratch bytes of lisa_decode_stack for this descriptor (two score rows + twice the largest layer). */
size_t lisa_stack_workspace_bytes(const lisa_desc* desc);

/*
 * std_attn_scores -- standard scaled dot-product attention (Sec. 2.1 Eq. 1-2) that also
 * emits the pre-softmax scores A = Q K^T * std_scale shared with the following LiSA layer.
 *   q [B,H,Lq,d_k], k [B,Hkv,Lk,d_k]   in
 *   v [B,Hkv,Lk,d_k]                   in   or NULL (then `out` must be NULL too)
 *   scores_out [B,H,Lq,Lk]             out  A, score type; or NULL when only `out` is wanted
 *   out [B,Lq,H,d_k]                   out  or NULL
 * With Lq = 1 and Lmax >= Lk this is the decode step of a standard layer: k and v are then
 * caches [B,Hkv,Lmax,d_k] of which the first Lk keys are attended (Lmax = 0: dense, Lk keys).
 * Lmax > 0 with Lq > 1, or 0 < Lmax < Lk, is LISA_ERR_SHAPE.
 */
int std_attn_scores(const lisa_desc* desc, const void* q, const void* k, const void* v,
                    void* scores_out, void* out, void* workspace, size_t workspace_bytes,
                    void* hip_stream);

/*
 * lisa_cache_fill -- hand-over from prefill to decode: a LiSA layer keeps K_LR instead of K
 * for the decoding stage (Sec. 5.2; Sec. 2.2 for the two stages).  Copies the K_LR and V rows of
 * the first Lk tokens into the caches, in the layouts lisa_attn_decode reads.
 * Uses dtype, B, Hkv, Lk, r, d_k, kcache_dim_major and Lmax (>= Lk) of the descriptor.
 *   k_lr        [B,Hkv,Lk,r]     in
 *   v           [B,Hkv,Lk,d_k]   in
 *   k_lr_cache  [B,Hkv,Lmax,r] or [B,Hkv,r,Lmax]   out (key indices 0 .. Lk-1 are written)
 *   v_cache     [B,Hkv,Lmax,d_k]                   out (likewise)
 * No workspace.  Byte copies: the caches hold exactly the input values.  B, Hkv and B * Hkv at
 * most 65535.
 */
int lisa_cache_fill(const lisa_desc* desc, const void* k_lr, const void* v, void* k_lr_cache,
                    void* v_cache, void* hip_stream);

/* Descriptor of lisa_project_qkv (host memory, plain data, zero-initialise then fill). */
typedef struct lisa_proj_desc {
  int32_t dtype;            /* lisa_dtype of X, W and of the three outputs                     */
  int32_t B;                /* sequences                                                       */
  int32_t L;                /* new tokens per sequence in this call                            */
  int32_t d_model;          /* width d of the hidden states                                    */
  int32_t H;                /* query heads                                                     */
  int32_t Hkv;              /* key/value heads                                                 */
  int32_t r;                /* per-head low-rank dimension (Eq. 3); even when rope_theta > 0   */
  int32_t d_k;              /* head dimension of V                                             */
  int32_t Lmax;             /* token capacity of k_lr and v, >= pos0 + L; 0 selects pos0 + L   */
  int32_t pos0;             /* position of the first new token: token l is written at key
                               index pos0 + l and rotated by the angle of position pos0 + l   */
  int32_t kcache_dim_major; /* k_lr is [B,Hkv,r,Lmax] (1) or [B,Hkv,Lmax,r] (0)                */
  float rope_theta;         /* base of the rotary position embedding; 0 = none                 */
} lisa_proj_desc;

/*
 * lisa_project_qkv -- front end of a LiSA layer: the low-rank queries and keys
 * Q_LR = X W^Q_LR, K_LR = X W^K_LR (the two factors of Eq. 3) and the values V = X W^V
 * (Sec. 2.1 Eq. 1) in one product, split in heads and written where lisa_attn_prefill (dense
 * tensors: pos0 = 0, Lmax = L or 0, kcache_dim_major = 0) or lisa_attn_decode (the caches,
 * Sec. 5.2) read them.  The paper's LLaMA models (Sec. 5.3) rotate queries and keys by
 * position; with rope_theta > 0 every Q_LR / K_LR head y of the token at position p becomes
 *   (y[t] cos a - y[t+r/2] sin a,  y[t] sin a + y[t+r/2] cos a),  a = p * rope_theta^(-2t/r),
 * for t < r/2, before it is rounded and stored (the cache holds rotated K_LR).
 *   x     [B,L,d_model]                          in
 *   w     [H*r + Hkv*r + Hkv*d_k, d_model]       in   one row per output feature: the columns
 *                                                     of W^Q_LR (head-major), then of W^K_LR,
 *                                                     then of W^V
 *   q_lr  [B,H,L,r]                              out
 *   k_lr  [B,Hkv,Lmax,r] or [B,Hkv,r,Lmax]       out  key indices pos0 .. pos0+L-1 are written
 *   v     [B,Hkv,Lmax,d_k]                       out  likewise
 * No workspace.  Accumulation is float32 (float64 for LISA_F32 inputs).
 */
int lisa_project_qkv(const lisa_proj_desc* desc, const void* x, const void* w, void* q_lr,
                     void* k_lr, void* v, void* hip_stream);

/*
 * lisa_layer_prefill -- a whole LiSA attention layer from the hidden states: lisa_project_qkv
 * (Eq. 3's factors H W^Q_LR, H W^K_LR and V = H W^V, rotated by position when rope_theta > 0)
 * followed by lisa_attn_prefill (Sec. 5.1, Eq. 3-4; Sec. 2.1 Eq. 1-2 without W^O) on the same
 * stream.  A fresh prefill: requires Lq = Lk; positions 0 .. Lq-1.
 *   x [B,Lq,d_model], w_qkv [H*r + Hkv*r + Hkv*d_k, d_model]   in   as in lisa_project_qkv
 *   scores_prev, w1, w2, out, scores_out                        as in lisa_attn_prefill
 *   workspace   at least lisa_workspace_bytes(desc, LISA_WS_LAYER) bytes: the prefill workspace
 *               followed by Q_LR, K_LR and V, which can be read there after the call
 *               (offsets lisa_layer_offsets()).
 */
int lisa_layer_prefill(const lisa_desc* desc, int32_t d_model, float rope_theta, const void* x,
                       const void* w_qkv, const void* scores_prev, const void* w1, const void* w2,
                       void* out, void* scores_out, void* workspace, size_t workspace_bytes,
                       void* hip_stream);

/*
 * lisa_layer_decode -- the decode step of a whole LiSA layer from the hidden state of the new
 * token of every sequence: lisa_project_qkv for one token at position Lk-1 (its rotated K_LR row
 * and its V row go straight into the caches, Sec. 5.2) followed by lisa_attn_decode.
 * Requires Lq = 1 and Lk <= Lmax.
 *   x [B,d_model], w_qkv [H*r + Hkv*r + Hkv*d_k, d_model]     in   as in lisa_project_qkv
 *   k_lr_cache, v_cache                                        in/out (only index Lk-1 is written)
 *   score_row_prev, w1, w2, out, score_row_out                 as in lisa_attn_decode
 *   workspace   at least lisa_workspace_bytes(desc, LISA_WS_LAYER_DECODE) bytes (the decode
 *               workspace followed by Q_LR [B,H,r])
 */
int lisa_layer_decode(const lisa_desc* desc, int32_t d_model, float rope_theta, const void* x,
                      const void* w_qkv, void* k_lr_cache, void* v_cache, const void* score_row_prev,
                      const void* w1, const void* w2, void* out, void* score_row_out, void* workspace,
                      size_t workspace_bytes, void* hip_stream);

/* Host-only helpers (no HIP call). */

/* Byte offsets of Q_LR [B,H,Lq,r], K_LR [B,Hkv,Lq,r] and V [B,Hkv,Lq,d_k] inside the workspace of
 * lisa_layer_prefill; returns 0 or a negative lisa_status. */
int lisa_layer_offsets(const lisa_desc* desc, size_t* q_lr_off, size_t* k_lr_off, size_t* v_off);

/*
 * lisa_kd_huber -- regression term of the knowledge-distillation loss for one LiSA layer
 * (Sec. 5.1 "Training strategy": L_KD = 1/|S| sum_{n in S} L_delta(A_n, A_n^*); App. C.1 "Huber
 * loss function": L_delta(a, b) = (a - b)^2 / 2 where |a - b| <= delta, delta (|a - b| - delta / 2)
 * otherwise).  The paper states no reduction over the entries; this library takes the mean over
 * the entries a query row can see (all entries when causal = 0), of all heads and sequences.
 *   scores   in   A_n of the student, score type, [B,H,Lq,Lk] or tiled (desc->score_tiled)
 *   teacher  in   A_n^* of the teacher, same type and layout
 *   delta         threshold of the loss, > 0 (the paper uses 1)
 *   weight, accumulate   out[0] = (accumulate ? out[0] : 0) + weight * mean: the |S| layers of a
 *                 model are |S| calls with weight 1 / |S|, the first with accumulate = 0
 *   out      out  2 doubles on the device: out[0] as above, out[1] = this layer's mean
 *   workspace     at least lisa_workspace_bytes(desc, LISA_WS_KD) bytes (partial sums, added in a
 *                 fixed order: the result does not depend on scheduling)
 * Uses dtype, B, H, Lq, Lk, causal and score_tiled of the descriptor (tiled: LISA_BF16 only).
 * Errors: LISA_ERR_NULL, LISA_ERR_SHAPE (delta <= 0 or not finite, weight not finite, bad
 * dimensions), LISA_ERR_ALIGN (16-byte), LISA_ERR_WORKSPACE, LISA_ERR_UNSUPPORTED, LISA_ERR_HIP.
 */
int lisa_kd_huber(const lisa_desc* desc, const void* scores, const void* teacher, float delta,
                  float weight, int accumulate, double* out, void* workspace,
                  size_t workspace_bytes, void* hip_stream);

/* Scratch bytes the given entry point (lisa_ws_kind) needs for this descriptor. */
size_t lisa_workspace_bytes(const lisa_desc* desc, int which);
/* Bytes of one score tensor of the descriptor in the score type and in its layout (Sec. 5.2:
 * h*l*l*2 per sequence in prefill, h*l*2 per sequence in decode; tiled: whole tiles). */
size_t lisa_scores_bytes(const lisa_desc* desc);
/* Bytes per score element: 4 (LISA_F32) or 2 (LISA_BF16). */
size_t lisa_score_elem_bytes(const lisa_desc* desc);
/* Bytes of key cache saved by storing K_LR instead of K in n_lisa_layers layers
 * (Sec. 5.2: |S| * h * l * (d_k - r) * element size, per sequence, times B). */
size_t lisa_kcache_saved_bytes(const lisa_desc* desc, int n_lisa_layers);
/* LISA_OK if the three entry points accept this descriptor, else the status they return. */
int lisa_supported(const lisa_desc* desc);
/* Static, human-readable text for a lisa_status. */
const char* lisa_strerror(int status);
/* hipGetErrorString of the last failed launch seen by this thread ("" if none). */
const char* lisa_last_hip_error(void);
/* Name of the kernel family the last successful call on this thread dispatched to
 * ("generic", "mfma_fused", "mfma_std", "decode_split", "cache_fill", "project_generic",
 * "project_mfma", "project_skinny", "mfma_scores"); for tests and
 * benchmark reports. */
const char* lisa_last_path(void);

/*
 * Geometry overrides for tests (per calling thread; nothing in production needs them).  The
 * dispatch picks head grouping, key splits and tile widths from the problem size; a test that
 * must cover the other instantiation on a small problem forces it here.  value < 0 restores the
 * library's own choice.  An override changes what lisa_workspace_bytes() returns: set it before
 * the size query and leave it until the call it is meant for has been made.
 *   LISA_TUNE_PREFILL_GROUPS  head groups of the fused prefill kernel (H = 16: 1 or 2; H = 32: 2 or 4)
 *   LISA_TUNE_PREFILL_SPLIT   key splits per row block: 1, 2 or 4 (other values are ignored)
 *   LISA_TUNE_PREFILL_PAIR    1: a workgroup takes a long and a short unit, 0: one unit
 *   LISA_TUNE_STD_PAIR        the same for the standard layer's prefill kernel
 *   LISA_TUNE_PROJECT_TN      tile width of the projection kernel: 192 or 256
 *   LISA_TUNE_PREFILL_SLICES  slices of 16 query rows per workgroup of the fused prefill kernel:
 *                             1, 2 or 4 (where the shape has them: ReLU, 33..96 hidden units)
 * Returns LISA_OK, or LISA_ERR_SHAPE for an unknown knob.
 */
typedef enum {
  LISA_TUNE_PREFILL_GROUPS = 0, LISA_TUNE_PREFILL_SPLIT = 1, LISA_TUNE_PREFILL_PAIR = 2,
  LISA_TUNE_STD_PAIR = 3, LISA_TUNE_PROJECT_TN = 4, LISA_TUNE_PREFILL_SLICES = 5, LISA_TUNE_COUNT = 6
} lisa_tune_knob;
int lisa_tune_set(int knob, int value);

/*
 * Reference kernels for benchmarks (diagnostic; nothing of the method is computed).  The caller times
 * them with events on the stream it passes; bench.py reports their rates next to the roofline
 * fractions of the library's kernels, as what a plain kernel reaches on the chip at hand.
 *   lisa_probe_hbm_read   reads `bytes` bytes (device memory, 16-byte aligned; a multiple of 16 is
 *                         read) once with 8 loads of 16 bytes in flight per lane and writes nothing.
 *                         `sink`: 16 bytes of device memory that stay untouched (they keep the loads
 *                         alive for the compiler).  Use a buffer larger than the last-level cache.
 *   lisa_probe_hbm_write  writes floor(bytes / 16) 16-byte pieces of `dst` (device memory, 16-byte
 *                         aligned) once with non-temporal stores: piece i becomes the four 32-bit
 *                         words {seed, i mod 2^32, i / 2^32, ~seed}.
 *   lisa_probe_mfma       `workgroups` workgroups of four waves, each wave `iters` rounds of
 *                         independent MFMAs on constant operands: shape 0 = 8 x 16x16x32 f16 per round
 *                         (the shape of the library's FFNs), 1 = 4 x 32x32x16 f16 (the same
 *                         2 x 65536 flop per wave and round).  `sink` as above (4 bytes used).
 * Return LISA_OK, LISA_ERR_NULL / LISA_ERR_ALIGN / LISA_ERR_SHAPE (checked before the launch) or
 * LISA_ERR_HIP.
 */
int lisa_probe_hbm_read(const void* src, size_t bytes, void* sink, void* hip_stream);
int lisa_probe_hbm_write(void* dst, size_t bytes, unsigned seed, void* hip_stream);
int lisa_probe_mfma(int shape, int iters, int workgroups, void* sink, void* hip_stream);

/*
 * Stage timing for benchmarks (diagnostic, per calling thread, off by default).  While
 * enabled, every entry point brackets each kernel it launches with HIP events recorded on
 * the call's own stream; nothing is synchronised until lisa_profile_collect().
 *   lisa_profile_enable(1)  start (drops earlier records);  lisa_profile_enable(0)  stop.
 *   lisa_profile_collect    waits for the recorded events, sums them per stage name and
 *                           fills up to max_stages entries; returns the number of stages
 *                           (or a negative lisa_status) and clears the records.
 * At most 16384 kernel launches are recorded between two collects; later ones are skipped.
 */
typedef struct lisa_stage_time {
  const char* name; /* static string: kernel (stage) name      */
  int32_t launches; /* launches recorded under that name       */
  float total_ms;   /* sum of their event-to-event durations   */
} lisa_stage_time;
int lisa_profile_enable(int on);
int lisa_profile_collect(lisa_stage_time* out, int max_stages);

#ifdef __cplusplus
}
#endif
#endif /* LISA_H_ */
