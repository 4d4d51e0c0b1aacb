// C ABI of the LiSA attention-layer library: argument validation (host only, before any
// HIP call), workspace accounting and kernel dispatch.  See include/lisa.h for the contract.
#include "../../include/lisa.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <cstdlib>
#include <mutex>

#include "kernels_decode.h"
#include "kernels_kd.h"
#include "kernels_generic.h"
#include "kernels_prefill.h"
#include "kernels_probe.h"
#include "kernels_project.h"
#include "kernels_scores_mfma.h"
#include "kernels_std_prefill.h"

using namespace lisa;

namespace {

thread_local char g_hip_err[256] = "";
thread_local const char* g_path = "";
// lisa_tune_set(): geometry overrides of the calling thread, -1 = the library's own choice
thread_local int g_tune[LISA_TUNE_COUNT] = {-1, -1, -1, -1, -1, -1};

// ---- static scratch of lisa_attn_decode_static ------------------------------------------
// Device memory that exists from the moment the code object is loaded on a GPU until the process
// ends: one copy per GPU, each at its own address.  In host code the array's name is only a
// handle for hipGetSymbolAddress; kernels receive the resolved address as an ordinary argument.
static __device__ __align__(256) unsigned char scratch[LISA_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

// Address of this GPU's copy of `scratch` (resolved once per device, with that device current).
int static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return LISA_ERR_HIP;
  if (dev < 0 || dev >= kMaxDevices) return LISA_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      snprintf(g_hip_err, sizeof(g_hip_err), "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
      return LISA_ERR_HIP;
    }
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return LISA_OK;
}

inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Limits of the kernels in this library (see lisa_supported()).
constexpr int kMaxHeadDim = 256;      // k_softmax_v: 8 rows * d_k outputs over 256 threads * 8
constexpr int kMaxRank = 256;
constexpr int kMaxFfnRows = 640;      // (Din + F + H) * 64 floats of LDS <= 160 KB
constexpr int kMaxGridYZ = 65535;

// Which operands a descriptor's variant uses (see lisa_mix / lisa_act).
inline bool has_ffn(const lisa_desc* d) { return d->mix == LISA_MIX_ADD || d->mix == LISA_MIX_CONCAT; }
inline bool has_w2(const lisa_desc* d) { return has_ffn(d) && d->act != LISA_ACT_SINGLE; }
inline bool has_delta(const lisa_desc* d) { return d->mix != LISA_MIX_SHARE; }

int check_common(const lisa_desc* d) {
  if (!d) return LISA_ERR_NULL;
  if (d->dtype != LISA_F32 && d->dtype != LISA_BF16) return LISA_ERR_UNSUPPORTED;
  if (d->B <= 0 || d->H <= 0 || d->Hkv <= 0 || d->Lq <= 0 || d->Lk <= 0 || d->d_k <= 0)
    return LISA_ERR_SHAPE;
  if (d->H % d->Hkv != 0) return LISA_ERR_SHAPE;
  if (d->causal != 0 && d->causal != 1) return LISA_ERR_SHAPE;
  if (d->out_f32 != 0 && d->out_f32 != 1) return LISA_ERR_SHAPE;
  if (d->score_tiled != 0 && d->score_tiled != 1) return LISA_ERR_SHAPE;
  if (d->causal && d->Lk < d->Lq) return LISA_ERR_SHAPE;
  if (d->d_k > kMaxHeadDim) return LISA_ERR_UNSUPPORTED;
  if (d->B > kMaxGridYZ || d->Lq > kMaxGridYZ || (long long)d->B * d->H > kMaxGridYZ)
    return LISA_ERR_UNSUPPORTED;
  if (d->std_scale < 0.f || !std::isfinite(d->std_scale)) return LISA_ERR_SHAPE;
  return LISA_OK;
}

int check_lisa(const lisa_desc* d) {
  int rc = check_common(d);
  if (rc) return rc;
  if (d->mix < LISA_MIX_ADD || d->mix > LISA_MIX_SHARE) return LISA_ERR_UNSUPPORTED;
  if (d->act < LISA_ACT_RELU || d->act > LISA_ACT_SINGLE) return LISA_ERR_UNSUPPORTED;
  if (has_delta(d) && d->r <= 0) return LISA_ERR_SHAPE;
  if (d->r < 0 || d->F < 0) return LISA_ERR_SHAPE;
  if (has_ffn(d) && (d->act == LISA_ACT_SINGLE ? d->F != d->H : d->F <= 0)) return LISA_ERR_SHAPE;
  if (d->write_scores != 0 && d->write_scores != 1) return LISA_ERR_SHAPE;
  if (d->delta_scale < 0.f || !std::isfinite(d->delta_scale)) return LISA_ERR_SHAPE;
  if (d->r > kMaxRank) return LISA_ERR_UNSUPPORTED;
  const int Din = d->mix == LISA_MIX_CONCAT ? 2 * d->H : d->H;
  if (Din + d->F + d->H > kMaxFfnRows) return LISA_ERR_UNSUPPORTED;
  return LISA_OK;
}

int check_decode(const lisa_desc* d) {
  int rc = check_lisa(d);
  if (rc) return rc;
  if (d->Lq != 1) return LISA_ERR_SHAPE;
  if (d->Lmax < d->Lk) return LISA_ERR_SHAPE;
  if (d->kcache_dim_major != 0 && d->kcache_dim_major != 1) return LISA_ERR_SHAPE;
  if (d->score_tiled) return LISA_ERR_UNSUPPORTED;          // a decode step hands over score rows
  return LISA_OK;
}

size_t score_elem(const lisa_desc* d) { return d->dtype == LISA_F32 ? 4 : 2; }

size_t scores_elems(const lisa_desc* d) {
  if (d->score_tiled)
    return (size_t)d->B * d->H * ((d->Lq + PF_ROWS - 1) / PF_ROWS) * ((d->Lk + PF_TK - 1) / PF_TK) * (PF_ROWS * PF_TK);
  return (size_t)d->B * d->H * d->Lq * d->Lk;
}
size_t scores_bytes(const lisa_desc* d) { return scores_elems(d) * score_elem(d); }

// float32 copy of the score tensor that the generic softmax kernel reads
size_t exact_bytes(const lisa_desc* d) {
  return round_up((size_t)d->B * d->H * d->Lq * d->Lk * sizeof(float), 256);
}

int hip_fail(hipError_t e) {
  snprintf(g_hip_err, sizeof(g_hip_err), "%s", hipGetErrorString(e));
  return LISA_ERR_HIP;
}

int check_launch() {
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? LISA_OK : hip_fail(e);
}

float pick_scale(float given, int n) { return given > 0.f ? given : 1.0f / std::sqrt((float)n); }

// ---- optional stage timing (lisa_profile_*) -------------------------------------------
struct ProfRec {
  const char* name;
  hipEvent_t beg, end;
};
constexpr size_t kMaxProfRecs = 16384;
thread_local bool g_prof_on = false;
thread_local std::vector<ProfRec> g_prof_recs;
thread_local std::vector<hipEvent_t> g_prof_pool;

hipEvent_t prof_event() {
  if (!g_prof_pool.empty()) {
    hipEvent_t e = g_prof_pool.back();
    g_prof_pool.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

// Brackets the launches made while it is alive with two events on their stream.
struct StageScope {
  hipStream_t st;
  ProfRec rec{nullptr, nullptr, nullptr};
  StageScope(const char* name, hipStream_t s) : st(s) {
    if (!g_prof_on || g_prof_recs.size() >= kMaxProfRecs) return;
    rec.beg = prof_event();
    rec.end = prof_event();
    if (!rec.beg || !rec.end) { rec.beg = rec.end = nullptr; return; }
    rec.name = name;
    (void)hipEventRecord(rec.beg, st);
  }
  ~StageScope() {
    if (!rec.name) return;
    (void)hipEventRecord(rec.end, st);
    g_prof_recs.push_back(rec);
  }
};

// ---- generic launches ----------------------------------------------------------------
template <typename T, typename S>
int launch_std_scores(const lisa_desc* d, const void* q, const void* k, KeyStrides ks, void* scores,
                      float* exact, hipStream_t st) {
  dim3 grid((d->Lk + 63) / 64, (d->Lq + 63) / 64, d->B * d->H);
  StageScope prof("k_std_scores", st);
  k_std_scores<T, S><<<grid, 256, 0, st>>>((const T*)q, (const T*)k, ks, (S*)scores, exact, d->H, d->Hkv,
                                           d->Lq, d->Lk, d->d_k, pick_scale(d->std_scale, d->d_k),
                                           d->causal);
  return check_launch();
}

// CONCAT with the two-layer ReLU FFN on the matrix cores (dense prefill tensors only).
constexpr int kComputeUnits = 256;   // MI355X

bool scores_mfma_ok(const lisa_desc* d) {
  if (d->dtype != LISA_BF16 || d->mix != LISA_MIX_CONCAT) return false;
  if (d->act != LISA_ACT_RELU && d->act != LISA_ACT_SILU) return false;
  if (d->Lq == 1) return false;                            // decode rows: the generic kernel (strided caches)
  if (d->H > 48 || d->F > 256 || d->r > 32 || d->Lk % 8 != 0) return false;
  return (long long)d->Lq * d->Lk < (1LL << 31);
}

template <int HBI, int FS, int HBO, bool TILED = false>
int launch_scores_mfma_t(const lisa_desc* d, const ScoresMfmaArgs& a, hipStream_t st) {
  const int lds = scores_mfma_lds<HBI, FS, HBO>(d->H);
  auto kern = d->act == LISA_ACT_SILU ? k_lisa_scores_mfma<HBI, FS, HBO, 1, TILED>
                                      : k_lisa_scores_mfma<HBI, FS, HBO, 0, TILED>;
  hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (e != hipSuccess) return hip_fail(e);
  // one workgroup per compute unit, each with an equal run of the tiles
  const long long total = a.tiles_b * a.B;
  dim3 grid((unsigned)std::min<long long>(total, kComputeUnits));
  StageScope prof("k_lisa_scores_mfma", st);
  kern<<<grid, 512, lds, st>>>(a);
  return check_launch();
}

// Workspace of the CONCAT pipeline: A_n in the score type when the caller does not ask for it (the
// softmax kernel reads it from there), the padded low-rank operands, V by key chunks.
struct ConcatWs {
  size_t qp, kp, vt, total;
  int Lqp, Lkp;
};
bool std_prefill_fast_ok(const lisa_desc* d);
// The CONCAT pipeline on tiled score tensors: the pipelined scores kernel (up to 32 heads) followed
// by the matrix-core softmax kernel, which then reads tiles.
bool concat_tiled_ok(const lisa_desc* d) { return scores_mfma_ok(d) && d->H <= 32 && std_prefill_fast_ok(d); }
ConcatWs concat_ws(const lisa_desc* d) {
  ConcatWs w;
  w.Lqp = (d->Lq + PF_ROWS - 1) / PF_ROWS * PF_ROWS;
  w.Lkp = (d->Lk + 63) / 64 * 64;
  w.qp = round_up(scores_bytes(d), 256);                   // (2-byte scores, in the layout of the call)
  w.kp = w.qp + round_up((size_t)d->B * d->H * w.Lqp * 32 * 2, 256);
  w.vt = w.kp + round_up((size_t)d->B * d->Hkv * w.Lkp * 32 * 2, 256);
  w.total = w.vt + (std_prefill_fast_ok(d) ? round_up((size_t)d->B * d->Hkv * d->d_k * w.Lkp * 2, 256) : 0);
  return w;
}

int launch_scores_mfma(const lisa_desc* d, const void* q_lr, const void* k_lr, const void* v, const void* prev,
                       const void* w1, const void* w2, void* scores, void* workspace, hipStream_t st) {
  const ConcatWs w = concat_ws(d);
  char* ws = (char*)workspace;
  {
    // V is regrouped in the same launch when the MFMA softmax kernel follows (d_k = 128)
    const bool with_v = std_prefill_fast_ok(d);
    const int dk = with_v ? d->d_k : 0;
    StageScope prof("k_prepare_prefill", st);
    const size_t rows = (size_t)d->B * d->H * w.Lqp + (size_t)d->B * d->Hkv * w.Lkp;
    const size_t blocks = (size_t)(w.Lkp / 64) * (dk / 64) * d->B * d->Hkv + (rows + 63) / 64;
    const bool vec = (uintptr_t)v % 16 == 0;
    auto kern = vec ? k_prepare_prefill<true> : k_prepare_prefill<false>;
    kern<<<(unsigned)blocks, 256, 0, st>>>((const bf16_t*)q_lr, (const bf16_t*)k_lr, (const bf16_t*)v,
                                          (bf16_t*)(ws + w.qp), (bf16_t*)(ws + w.kp), (bf16_t*)(ws + w.vt),
                                          d->B, d->H, d->Hkv, d->Lq, d->Lk, w.Lqp, w.Lkp, d->r, dk);
    int rc = check_launch();
    if (rc) return rc;
  }
  ScoresMfmaArgs a{};
  a.qp = (const bf16_t*)(ws + w.qp);
  a.kp = (const bf16_t*)(ws + w.kp);
  a.prev = (const half_t*)prev;
  a.w1 = (const bf16_t*)w1;
  a.w2 = (const bf16_t*)w2;
  a.scores = (half_t*)scores;
  a.B = d->B;
  a.H = d->H;
  a.Hkv = d->Hkv;
  a.Lq = d->Lq;
  a.Lk = d->Lk;
  a.tiles_b = 0;
  for (int rg = 0; rg < (d->Lq + PF_ROWS - 1) / PF_ROWS; ++rg)
    a.tiles_b += scores_mfma_tiles(rg, d->Lq, d->Lk, d->causal);
  a.Lqp = w.Lqp;
  a.Lkp = w.Lkp;
  a.F = d->F;
  a.causal = d->causal;
  a.dscale = pick_scale(d->delta_scale, d->r);
  a.tiled = d->score_tiled;
  const bool wide = d->F > 128;
  if (d->score_tiled) {                                      // (concat_tiled_ok: up to 32 heads)
    if (d->H <= 16)
      return wide ? launch_scores_mfma_t<2, 8, 1, true>(d, a, st) : launch_scores_mfma_t<2, 4, 1, true>(d, a, st);
    return wide ? launch_scores_mfma_t<4, 8, 2, true>(d, a, st) : launch_scores_mfma_t<4, 4, 2, true>(d, a, st);
  }
  if (d->H <= 16) return wide ? launch_scores_mfma_t<2, 8, 1>(d, a, st) : launch_scores_mfma_t<2, 4, 1>(d, a, st);
  if (d->H <= 32) return wide ? launch_scores_mfma_t<4, 8, 2>(d, a, st) : launch_scores_mfma_t<4, 4, 2>(d, a, st);
  return wide ? launch_scores_mfma_t<6, 8, 3>(d, a, st) : launch_scores_mfma_t<6, 4, 3>(d, a, st);
}

template <typename T, typename S>
int launch_lisa_scores(const lisa_desc* d, const void* q_lr, const void* k_lr, KeyStrides ks,
                       const void* prev, const void* w1, const void* w2, void* scores,
                       float* exact, hipStream_t st) {
  const int Din = d->mix == LISA_MIX_CONCAT ? 2 * d->H : d->H;
  const size_t lds = has_ffn(d) ? (size_t)(Din + d->F + d->H) * 64 * sizeof(float) : 0;
  auto kern = k_lisa_scores<T, S>;
  if (lds > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)lds);
    if (e != hipSuccess) return hip_fail(e);
  }
  dim3 grid((d->Lk + 63) / 64, d->Lq, d->B);
  StageScope prof("k_lisa_scores", st);
  kern<<<grid, 256, lds, st>>>((const T*)q_lr, (const T*)k_lr, ks, (const S*)prev, (const T*)w1,
                               (const T*)w2, (S*)scores, exact, d->H, d->Hkv, d->Lq, d->Lk, d->r, d->F,
                               d->mix, d->act, has_delta(d) ? pick_scale(d->delta_scale, d->r) : 0.f,
                               d->causal);
  return check_launch();
}

template <typename T, typename S = float>
int launch_softmax_v(const lisa_desc* d, const S* scores, const void* v, KeyStrides vs, void* out,
                     hipStream_t st) {
  dim3 grid((d->Lq + 7) / 8, d->H, d->B);
  const long long sh = d->d_k, si = (long long)d->H * d->d_k, sb = si * d->Lq;
  StageScope prof("k_softmax_v", st);
  if (d->out_f32)
    k_softmax_v<T, S, float><<<grid, 256, 0, st>>>(scores, (const T*)v, vs, (float*)out, sb, si, sh, d->H,
                                                   d->Hkv, d->Lq, d->Lk, d->d_k, d->causal);
  else
    k_softmax_v<T, S, T><<<grid, 256, 0, st>>>(scores, (const T*)v, vs, (T*)out, sb, si, sh, d->H, d->Hkv,
                                               d->Lq, d->Lk, d->d_k, d->causal);
  return check_launch();
}

KeyStrides dense_keys(const lisa_desc* d, int len, int width) {
  KeyStrides s;
  s.t = 1;
  s.j = width;
  s.h = (long long)len * width;
  s.b = s.h * d->Hkv;
  return s;
}

KeyStrides dim_major_keys(const lisa_desc* d, int len, int width) {
  KeyStrides s;
  s.j = 1;
  s.t = len;
  s.h = (long long)len * width;
  s.b = s.h * d->Hkv;
  return s;
}

bool std_prefill_fast_ok(const lisa_desc* d);
size_t std_prefill_ws(const lisa_desc* d);
int run_softmax_given_fast(const lisa_desc* d, const void* given, bool given_half, const void* v, void* out,
                           void* vt_ws, hipStream_t st);

template <typename T, typename S>
int run_lisa(const lisa_desc* d, const void* q_lr, const void* k_lr, KeyStrides ks, const void* v,
             KeyStrides vs, const void* prev, const void* w1, const void* w2, void* out,
             void* scores, float* exact, hipStream_t st) {
  const bool mfma = scores_mfma_ok(d);
  if (mfma) {
    // A_n exists as the IEEE-half tensor that the next layer shares, and the softmax reads that
    // tensor: a float32 copy would triple the bytes this pipeline writes.  The rounding, |A_n| 2^-11,
    // is the size of what the module's inputs already carry (A_{n-1} is stored as half, and A_delta
    // enters the FFN as a half MFMA operand).
    void* an = scores ? scores : (void*)exact;
    int rc = launch_scores_mfma(d, q_lr, k_lr, v, prev, w1, w2, an, exact, st);
    if (rc) return rc;
    if (std_prefill_fast_ok(d))
      rc = run_softmax_given_fast(d, an, true, nullptr, out, (char*)exact + concat_ws(d).vt, st);
    else
      rc = launch_softmax_v<T, half_t>(d, (const half_t*)an, v, vs, out, st);
    if (rc == LISA_OK) g_path = "mfma_scores";
    return rc;
  }
  // Generic kernels: the softmax reads the unrounded float32 A_n from the workspace.
  int rc = launch_lisa_scores<T, S>(d, q_lr, k_lr, ks, prev, w1, w2, scores, exact, st);
  if (rc) return rc;
  // softmax and P V from the float32 scores: on the matrix cores where the standard layer's kernel
  // fits (it then reads the scores instead of computing Q K^T), else the generic kernel
  if (std_prefill_fast_ok(d))
    rc = run_softmax_given_fast(d, exact, false, v, out, (char*)exact + exact_bytes(d), st);
  else
    rc = launch_softmax_v<T>(d, exact, v, vs, out, st);
  if (rc == LISA_OK) g_path = "generic";
  return rc;
}

// ---- split-context decode (bf16) -----------------------------------------------------
// Shapes the decode kernels are instantiated for.
bool decode_fast_ok(const lisa_desc* d, bool lisa_layer) {
  if (d->dtype != LISA_BF16 || d->Lq != 1) return false;
  if (d->d_k != 64 && d->d_k != 128) return false;
  if (d->H > 64) return false;
  if (lisa_layer) {
    if (d->mix == LISA_MIX_SHARE) return true;             // direct sharing: the previous row as it stands
    if (d->mix == LISA_MIX_CONCAT)                         // the instantiated CONCAT shapes
      return (d->act == LISA_ACT_RELU || d->act == LISA_ACT_SILU) && d->H <= 48 && d->F <= 256 && d->r <= 64;
    if (d->mix != LISA_MIX_ADD || (d->act != LISA_ACT_RELU && d->act != LISA_ACT_SILU)) return false;
    if (d->F > 128 || d->r > 64) return false;
  }
  return true;
}

int decode_chunks(const lisa_desc* d) { return (d->Lk + DEC_CK - 1) / DEC_CK; }

size_t decode_fast_bytes(const lisa_desc* d) {
  const size_t units = (size_t)d->B * decode_chunks(d) * d->H;
  return round_up(units * d->d_k * sizeof(float), 256) + round_up(units * 2 * sizeof(float), 256);
}

// A decode stack leaves the combine of a layer to the launch of the layer behind it (its workgroups
// take the units when their own work is done, see k_decode_part): per calling thread, set only inside lisa_decode_stack.
struct DeferredCombine {
  bool on = false, pending = false;
  const float* o = nullptr;
  const float* ml = nullptr;
  void* out = nullptr;
  int H = 0, B = 0, n_chunk = 0, dk = 0, out_f32 = 0;
  long fast_calls = 0;
};
thread_local DeferredCombine g_dc;

int launch_combine(const float* part_o, const float* part_ml, void* out, int H, int B, int n_chunk, int dk,
                   int out_f32, hipStream_t st) {
  dim3 grid(H, B);
  StageScope prof("k_decode_combine", st);
  if (dk == 128) {
    if (out_f32) k_decode_combine<float, 128><<<grid, 256, 0, st>>>(part_o, part_ml, (float*)out, H, n_chunk);
    else k_decode_combine<bf16_t, 128><<<grid, 256, 0, st>>>(part_o, part_ml, (bf16_t*)out, H, n_chunk);
  } else {
    if (out_f32) k_decode_combine<float, 64><<<grid, 256, 0, st>>>(part_o, part_ml, (float*)out, H, n_chunk);
    else k_decode_combine<bf16_t, 64><<<grid, 256, 0, st>>>(part_o, part_ml, (bf16_t*)out, H, n_chunk);
  }
  return check_launch();
}

// The combine that a stack still owes, as a launch of its own.
int flush_deferred_combine(hipStream_t st) {
  if (!g_dc.pending) return LISA_OK;
  g_dc.pending = false;
  return launch_combine(g_dc.o, g_dc.ml, g_dc.out, g_dc.H, g_dc.B, g_dc.n_chunk, g_dc.dk, g_dc.out_f32, st);
}

template <int LISA_MODE, int HB, int FS, int ACT = 0>
int launch_decode_part_dk(const lisa_desc* d, const DecodeArgs& a, size_t lds, hipStream_t st) {
  dim3 grid(a.n_chunk, d->B);
  if (a.cmb_units > 0) lds = std::max<size_t>(lds, 4608);   // (the combine units use the same LDS)
  auto kern = d->d_k == 128 ? k_decode_part<LISA_MODE, HB, FS, 128, ACT> : k_decode_part<LISA_MODE, HB, FS, 64, ACT>;
  if (lds > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)lds);
    if (e != hipSuccess) return hip_fail(e);
  }
  StageScope prof(LISA_MODE == 3 ? "k_decode_part_share" : LISA_MODE ? "k_decode_part_lisa" : "k_decode_part_std", st);
  kern<<<grid, DEC_THREADS, lds, st>>>(a);
  return check_launch();
}

// CONCAT form: HBI blocks of 16 FFN inputs (2H of them), hidden width by thirds of the range
template <int HBI, int ACT>
int launch_decode_concat_act(const lisa_desc* d, const DecodeArgs& a, size_t lds, hipStream_t st) {
  if (d->F <= 64) return launch_decode_part_dk<2, HBI, 2, ACT>(d, a, lds, st);
  if (d->F <= 128) return launch_decode_part_dk<2, HBI, 4, ACT>(d, a, lds, st);
  return launch_decode_part_dk<2, HBI, 8, ACT>(d, a, lds, st);
}
template <int HBI>
int launch_decode_concat_fs(const lisa_desc* d, const DecodeArgs& a, size_t lds, hipStream_t st) {
  return d->act == LISA_ACT_SILU ? launch_decode_concat_act<HBI, 1>(d, a, lds, st)
                                 : launch_decode_concat_act<HBI, 0>(d, a, lds, st);
}

template <int HB, int ACT>
int launch_decode_lisa_act(const lisa_desc* d, const DecodeArgs& a, size_t lds, hipStream_t st) {
  switch ((d->F + 31) / 32) {
    case 1: return launch_decode_part_dk<1, HB, 1, ACT>(d, a, lds, st);
    case 2: return launch_decode_part_dk<1, HB, 2, ACT>(d, a, lds, st);
    case 3: return launch_decode_part_dk<1, HB, 3, ACT>(d, a, lds, st);
    default: return launch_decode_part_dk<1, HB, 4, ACT>(d, a, lds, st);
  }
}
template <int HB>
int launch_decode_lisa_fs(const lisa_desc* d, const DecodeArgs& a, size_t lds, hipStream_t st) {
  return d->act == LISA_ACT_SILU ? launch_decode_lisa_act<HB, 1>(d, a, lds, st)
                                 : launch_decode_lisa_act<HB, 0>(d, a, lds, st);
}

int run_decode_fast(const lisa_desc* d, bool lisa_layer, DecodeArgs a, void* out, void* workspace,
                    hipStream_t st) {
  const size_t units = (size_t)d->B * decode_chunks(d) * d->H;
  a.part_o = (float*)workspace;
  a.part_ml = (float*)((char*)workspace + round_up(units * d->d_k * sizeof(float), 256));
  a.H = d->H;
  a.Hkv = d->Hkv;
  a.Lk = d->Lk;
  a.r = d->r;
  a.F = d->F;
  a.n_chunk = decode_chunks(d);
  a.B = d->B;
  a.cmb_units = 0;
  if (g_dc.on) {
    ++g_dc.fast_calls;
    if (g_dc.pending && g_dc.dk == d->d_k && (long long)g_dc.H * g_dc.B < (1 << 24)) {
      a.cmb_o = g_dc.o;
      a.cmb_ml = g_dc.ml;
      a.cmb_out = g_dc.out;
      a.cmb_units = g_dc.H * g_dc.B;
      a.cmb_H = g_dc.H;
      a.cmb_nchunk = g_dc.n_chunk;
      a.cmb_out_f32 = g_dc.out_f32;
      g_dc.pending = false;
    } else {
      int frc = flush_deferred_combine(st);
      if (frc) return frc;
    }
  }
  size_t lds = (size_t)d->H * DEC_CK * sizeof(float);
  int rc;
  if (lisa_layer && d->mix == LISA_MIX_SHARE) {
    a.scale = 0.f;
    rc = launch_decode_part_dk<3, 1, 1>(d, a, lds, st);
  } else if (lisa_layer && d->mix == LISA_MIX_CONCAT) {
    const int hbi = d->H <= 16 ? 2 : d->H <= 32 ? 4 : 6, fs = d->F <= 64 ? 2 : d->F <= 128 ? 4 : 8;
    const int ks1 = (hbi + 1) / 2, hbo = (hbi + 1) / 2;
    lds += (size_t)((d->H * d->r + 3) & ~3) * sizeof(float) + (size_t)(2 * fs * ks1 + hbo * fs) * 1024;
    a.scale = pick_scale(d->delta_scale, d->r);
    rc = hbi == 2   ? launch_decode_concat_fs<2>(d, a, lds, st)
         : hbi == 4 ? launch_decode_concat_fs<4>(d, a, lds, st)
                    : launch_decode_concat_fs<6>(d, a, lds, st);
  } else if (lisa_layer) {
    // + q_lr [H][r] as float + the FFN weights in MFMA operand order (mfma_ffn.h: kStageBytes)
    const int hb = (d->H + 15) / 16, fs = (d->F + 31) / 32, ks1 = (hb + 1) / 2;
    lds += (size_t)((d->H * d->r + 3) & ~3) * sizeof(float) + (size_t)(2 * fs * ks1 + hb * fs) * 1024;
    a.scale = pick_scale(d->delta_scale, d->r);
    switch ((d->H + 15) / 16) {
      case 1: rc = launch_decode_lisa_fs<1>(d, a, lds, st); break;
      case 2: rc = launch_decode_lisa_fs<2>(d, a, lds, st); break;
      case 3: rc = launch_decode_lisa_fs<3>(d, a, lds, st); break;
      default: rc = launch_decode_lisa_fs<4>(d, a, lds, st); break;
    }
  } else {
    a.scale = pick_scale(d->std_scale, d->d_k);
    rc = launch_decode_part_dk<0, 1, 1>(d, a, lds, st);
  }
  if (rc) return rc;
  if (g_dc.on) {                                             // left to the next layer's launch (or the stack's end)
    g_dc.pending = true;
    g_dc.o = a.part_o;
    g_dc.ml = a.part_ml;
    g_dc.out = out;
    g_dc.H = d->H;
    g_dc.B = d->B;
    g_dc.n_chunk = a.n_chunk;
    g_dc.dk = d->d_k;
    g_dc.out_f32 = d->out_f32;
  } else {
    rc = launch_combine(a.part_o, a.part_ml, out, d->H, d->B, a.n_chunk, d->d_k, d->out_f32, st);
  }
  if (rc == LISA_OK) g_path = "decode_split";
  return rc;
}

// ---- fused MFMA prefill (bf16) ---------------------------------------------------------
// Head counts the fused kernel is instantiated for: H -> (waves, heads per wave, head groups).
bool prefill_fused_ok(const lisa_desc* d) {
  if (d->dtype != LISA_BF16 || d->d_k != 128) return false;
  if (d->mix != LISA_MIX_ADD || (d->act != LISA_ACT_RELU && d->act != LISA_ACT_SILU)) return false;
  if (d->Lk % 8 != 0 || d->F > 128 || d->r > 32) return false;   // 16-byte aligned score rows
  // 32-bit byte offsets inside one head's scores (tiled: rows and keys rounded up to whole tiles)
  if ((long long)(d->Lq + PF_ROWS) * (d->Lk + PF_TK) >= (1LL << 31)) return false;
  return d->H == 8 || d->H == 16 || d->H == 24 || d->H == 32 || d->H == 40;
}


// Geometry of the fused prefill launch: row slices per workgroup (R = 16 * slices query rows), head
// groups, key splits, paired units.
//   slices  A workgroup of R rows fetches each K_LR / V tile once for all its rows: 4 slices where
//           the problem still gives every compute unit several units of work (>= 1024 units), which
//           needs one head per wave (groups of 8 heads); ReLU layers with 33..96 hidden units.
//   groups  H = 32 (16) runs as two (one) groups of 16 heads, two heads per wave, or as four (two)
//           groups of 8, one head per wave: the first FFN layer is computed once more per extra
//           group, but there are more units (no key splits, partial results and combine passes on
//           small problems) and row slices become possible.
//   split   small problems have too few units to fill the chip and their longest unit (the last
//           row block) sets the run time: the key tiles of a row block are dealt to 2 or 4 units.
//   pair    two units (a long and a short one) per workgroup once that still leaves two workgroups
//           per compute unit: equal work per workgroup, FFN weights staged once for both.
struct PrefillGeom {
  int slices, groups, split, pair;
};

bool prefill_slices_ok(const lisa_desc* d) {
  return d->act == LISA_ACT_RELU && d->F > 32 && d->F <= 96 && (d->H == 8 || d->H == 16 || d->H == 32 || d->H == 40);
}

PrefillGeom prefill_geom(const lisa_desc* d) {
  PrefillGeom g{1, 1, 1, 0};
  const long long blocks16 = (long long)((d->Lq + PF_ROWS - 1) / PF_ROWS) * d->B;
  const int few = d->H == 40 ? 5 : d->H == 32 ? 2 : 1;      // groups of 16 heads (H = 40, 8: of 8)
  const int many = d->H / 8;
  const bool two_forms = d->H == 32 || d->H == 16;
  // H = 32 with key/value heads shared by (a multiple of) four query heads can keep the whole layer
  // of a row block in one workgroup, a wave per group of four heads.  It is correct and tested but
  // never chosen: its 128 accumulator registers per lane leave the compiler 50 short (spills), and
  // it measured 11.8 ms against 7.6 ms for two groups of 16 on the LLaMA3-8B shape at L = 8192.
  const bool whole_ok = d->H == 32 && (d->H / d->Hkv) % 4 == 0;
  const bool large = blocks16 * few >= 2 * kComputeUnits;
  if (prefill_slices_ok(d)) {
    // two slices where the problem still gives every compute unit several units of work; not where
    // groups of 16 heads, two per wave, are the alternative (measured with two slices against two
    // groups: 10.2 / 7.6 ms on the LLaMA3-8B shape, where the pair of heads shares its operands;
    // 2.8 / 2.5 ms on LLaMA2-7B heads at B = 4, L = 4096; on the LLaMA2-13B shape, which has no
    // such form, 8.5 ms with two slices against 9.3 ms with one).  Four slices exist and are
    // tested, but their 128 accumulators spill: 16 - 20 ms on the same shapes.
    if (!(two_forms && large) && (long long)((d->Lq + 31) / 32) * d->B * many >= 4 * kComputeUnits) g.slices = 2;
    const int forced = g_tune[LISA_TUNE_PREFILL_SLICES];
    if (forced == 1 || forced == 2 || forced == 4) g.slices = forced;
  }
  const int want = g_tune[LISA_TUNE_PREFILL_GROUPS];
  if (d->H == 24) g.groups = 1;
  else if (whole_ok && g.slices == 1 && want == 1) g.groups = 1;
  else if (!two_forms || g.slices > 1) g.groups = many;
  else if (want >= 0) g.groups = want == many ? many : few;
  // SiLU costs two quarter-rate instructions per hidden unit, once more per extra group: measured
  // 0.27 ms with two groups (and a key split) against 0.32 ms with four on the LLaMA2-7B shape.
  else if (d->act == LISA_ACT_SILU) g.groups = few;
  else g.groups = large ? few : many;
  const long long units = (long long)((d->Lq + 16 * g.slices - 1) / (16 * g.slices)) * d->B * g.groups;
  if (g.slices == 1) {
    const int tiles_max = (d->Lk + PF_TK - 1) / PF_TK;
    while (g.split < 4 && units * g.split < 2 * kComputeUnits && tiles_max / (2 * g.split) >= 4) g.split *= 2;
    const int forced = g_tune[LISA_TUNE_PREFILL_SPLIT];
    if (forced == 1 || forced == 2 || forced == 4) g.split = forced;
  }
  g.pair = units * g.split >= 2 * kComputeUnits;
  if (g_tune[LISA_TUNE_PREFILL_PAIR] >= 0) g.pair = g_tune[LISA_TUNE_PREFILL_PAIR] != 0;
  return g;
}

struct PrefillWs {
  size_t qp, kp, vt, part_o, part_ml, total;   // byte offsets in the workspace
  int Lqp, Lkp;
  PrefillGeom geom;
};

PrefillWs prefill_fused_ws(const lisa_desc* d) {
  PrefillWs w;
  w.Lqp = (d->Lq + PF_ROWS - 1) / PF_ROWS * PF_ROWS;
  w.Lkp = (d->Lk + 63) / 64 * 64;
  w.qp = 0;
  w.kp = w.qp + round_up((size_t)d->B * d->H * w.Lqp * 32 * 2, 256);
  w.vt = w.kp + round_up((size_t)d->B * d->Hkv * w.Lkp * 32 * 2, 256);
  w.part_o = w.vt + round_up((size_t)d->B * d->Hkv * d->d_k * w.Lkp * 2, 256);
  w.geom = prefill_geom(d);
  const size_t rows = w.geom.split > 1 ? (size_t)w.geom.split * d->B * w.Lqp * d->H : 0;
  w.part_ml = w.part_o + round_up(rows * d->d_k * sizeof(float), 256);
  w.total = w.part_ml + round_up(rows * 2 * sizeof(float), 256);
  return w;
}

template <int NG, int FS, int HPW, int NW, int ACT, int RS, int SHG = 0, bool FTRIM = false>
int launch_prefill_fused_t(const lisa_desc* d, const PrefillArgs& a, hipStream_t st) {
  constexpr int GH = NW * HPW, H = NG * GH;
  typedef MfmaFfn<(H + 15) / 16, FS, (GH + 15) / 16> Ffn;
  // (all heads in one workgroup: the A_{n-1} piece is double buffered and doubles as A_n staging)
  constexpr bool XSTG = NG == 1 && HPW == 4;
  constexpr size_t lds = XSTG ? (size_t)2 * H * PF_XS_HEAD + (size_t)GH * PF_YS_HEAD + Ffn::kStageBytes
                              : (size_t)H * PF_XS_HEAD + (size_t)GH * PF_YS_HEAD + Ffn::kStageBytes +
                                    (size_t)GH * RS * PF_AS_HEAD;
  static_assert(lds <= 160 * 1024, "LDS of one compute unit");
  auto kern = k_lisa_prefill_fused<NG, FS, HPW, NW, ACT, RS, SHG, FTRIM>;
  hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)lds);
  if (e != hipSuccess) return hip_fail(e);
  const long long units = (long long)((a.Lq + PF_ROWS * RS - 1) / (PF_ROWS * RS)) * a.split;
  constexpr int CHU = pf_chunk_units(NG);                    // neighbouring units per chunk
  const long long chunks = ((a.pair ? (units + 1) / 2 : units) + CHU - 1) / CHU * a.B;
  const long long wgs = (chunks + 7) / 8 * 8 * CHU * NG;
  if (wgs > 0x7fffffffLL) return LISA_ERR_UNSUPPORTED;
  StageScope prof("k_lisa_prefill_fused", st);
  kern<<<dim3((unsigned)wgs), NW * 64, lds, st>>>(a);
  return check_launch();
}

template <int NG, int HPW, int NW, int ACT, int RS, int SHG = 0>
int launch_prefill_fused_act(const lisa_desc* d, const PrefillArgs& a, hipStream_t st) {
  if (RS > 1) {                                              // row slices: 33..96 hidden units (prefill_slices_ok)
    if ((d->F + 31) / 32 == 2) return launch_prefill_fused_t<NG, 2, HPW, NW, ACT, RS, SHG>(d, a, st);
    // (two slices, 65..80 hidden units: the last block of 16 is padding)
    if (RS == 2 && d->F <= 80) return launch_prefill_fused_t<NG, 3, HPW, NW, ACT, RS, SHG, true>(d, a, st);
    return launch_prefill_fused_t<NG, 3, HPW, NW, ACT, RS, SHG>(d, a, st);
  }
  switch ((d->F + 31) / 32) {
    case 1: return launch_prefill_fused_t<NG, 1, HPW, NW, ACT, 1, SHG>(d, a, st);
    case 2: return launch_prefill_fused_t<NG, 2, HPW, NW, ACT, 1, SHG>(d, a, st);
    case 3: return launch_prefill_fused_t<NG, 3, HPW, NW, ACT, 1, SHG>(d, a, st);
    default: return launch_prefill_fused_t<NG, 4, HPW, NW, ACT, 1, SHG>(d, a, st);
  }
}
template <int NG, int HPW, int NW>
int launch_prefill_fused_fs(const lisa_desc* d, const PrefillArgs& a, int slices, hipStream_t st) {
  if (HPW == 1 && slices == 4) return launch_prefill_fused_act<NG, 1, NW, 0, 4>(d, a, st);
  if (HPW == 1 && slices == 2) return launch_prefill_fused_act<NG, 1, NW, 0, 2>(d, a, st);
  // the heads of a wave share their key/value head: one operand set for all of them
  constexpr int HS = HPW == 3 ? 2 : HPW;                     // (no shared form of the 24-head kernel)
  if (HPW > 1 && HPW != 3 && (d->H / d->Hkv) % HPW == 0)
    return d->act == LISA_ACT_SILU ? launch_prefill_fused_act<NG, HS, NW, 1, 1, HS>(d, a, st)
                                   : launch_prefill_fused_act<NG, HS, NW, 0, 1, HS>(d, a, st);
  return d->act == LISA_ACT_SILU ? launch_prefill_fused_act<NG, HPW, NW, 1, 1>(d, a, st)
                                 : launch_prefill_fused_act<NG, HPW, NW, 0, 1>(d, a, st);
}

int run_prefill_fused(const lisa_desc* d, const void* q_lr, const void* k_lr, const void* v,
                      const void* prev, const void* w1, const void* w2, void* out, void* scores,
                      void* workspace, hipStream_t st) {
  const PrefillWs w = prefill_fused_ws(d);
  const PrefillGeom& geo = w.geom;
  char* ws = (char*)workspace;
  PrefillArgs a{};
  a.qp = (const bf16_t*)(ws + w.qp);
  a.kp = (const bf16_t*)(ws + w.kp);
  a.vt = (const bf16_t*)(ws + w.vt);
  a.prev = (const half_t*)prev;
  a.w1 = (const bf16_t*)w1;
  a.w2 = (const bf16_t*)w2;
  a.scores = (half_t*)scores;
  a.out = out;
  a.B = d->B;
  a.H = d->H;
  a.Hkv = d->Hkv;
  a.Lq = d->Lq;
  a.Lk = d->Lk;
  a.Lqp = w.Lqp;
  a.Lkp = w.Lkp;
  a.F = d->F;
  a.causal = d->causal;
  a.out_f32 = d->out_f32;
  a.tiled = d->score_tiled;
  a.dscale = pick_scale(d->delta_scale, d->r);
  a.split = geo.split;
  a.pair = geo.pair;
  a.part_o = (float*)(ws + w.part_o);
  a.part_ml = (float*)(ws + w.part_ml);
  {
    StageScope prof("k_prepare_prefill", st);
    const size_t rows = (size_t)d->B * d->H * w.Lqp + (size_t)d->B * d->Hkv * w.Lkp;
    const size_t blocks = (size_t)(w.Lkp / 64) * (d->d_k / 64) * d->B * d->Hkv + (rows + 63) / 64;
    const bool vec = (uintptr_t)v % 16 == 0;
    auto kern = vec ? k_prepare_prefill<true> : k_prepare_prefill<false>;
    kern<<<(unsigned)blocks, 256, 0, st>>>((const bf16_t*)q_lr, (const bf16_t*)k_lr, (const bf16_t*)v,
                                          (bf16_t*)(ws + w.qp), (bf16_t*)(ws + w.kp), (bf16_t*)(ws + w.vt),
                                          d->B, d->H, d->Hkv, d->Lq, d->Lk, w.Lqp, w.Lkp, d->r, d->d_k);
    int rc = check_launch();
    if (rc) return rc;
  }
  int rc;
  switch (d->H) {
    case 8: rc = launch_prefill_fused_fs<1, 1, 8>(d, a, geo.slices, st); break;    // one group of 8 heads
    case 16:                                                            // one group of 16 or two of 8
      rc = geo.groups == 2 ? launch_prefill_fused_fs<2, 1, 8>(d, a, geo.slices, st)
                           : launch_prefill_fused_fs<1, 2, 8>(d, a, 1, st);
      break;
    case 24: rc = launch_prefill_fused_fs<1, 3, 8>(d, a, 1, st); break;   // one group of 24
    case 32:                                                   // two groups of 16, four of 8, or all 32 heads
      rc = geo.groups == 4   ? launch_prefill_fused_fs<4, 1, 8>(d, a, geo.slices, st)
           : geo.groups == 1 ? launch_prefill_fused_fs<1, 4, 8>(d, a, 1, st)
                             : launch_prefill_fused_fs<2, 2, 8>(d, a, 1, st);
      break;
    default: rc = launch_prefill_fused_fs<5, 1, 8>(d, a, geo.slices, st); break;   // H = 40: five groups of 8
  }
  if (rc == LISA_OK && a.split > 1) {
    dim3 grid(d->Lq, d->B);
    StageScope prof("k_prefill_combine", st);
    k_prefill_combine<<<grid, 256, 0, st>>>(a);
    rc = check_launch();
  }
  if (rc == LISA_OK) g_path = "mfma_fused";
  return rc;
}

// ---- standard layer, prefill, MFMA (bf16) ---------------------------------------------
bool std_prefill_fast_ok(const lisa_desc* d) {
  return d->dtype == LISA_BF16 && d->d_k == 128 && d->Lk % 8 == 0 && d->Lq > 1;
}

size_t std_prefill_ws(const lisa_desc* d) {   // V by key chunks
  const size_t Lkp = (size_t)(d->Lk + 63) / 64 * 64;
  return round_up((size_t)d->B * d->Hkv * d->d_k * Lkp * 2, 256);
}

// softmax(A) V for scores A that are already in memory, float32 or IEEE half (k_std_prefill in
// GIVEN mode).
int run_softmax_given_fast(const lisa_desc* d, const void* given, bool given_half, const void* v, void* out,
                           void* vt_ws, hipStream_t st) {
  StdPrefillArgs a{};
  a.vt = (const bf16_t*)vt_ws;
  a.given = given;
  a.out = out;
  a.H = d->H;
  a.Hkv = d->Hkv;
  a.Lq = d->Lq;
  a.Lk = d->Lk;
  a.Lkp = (d->Lk + 63) / 64 * 64;
  a.causal = d->causal;
  a.out_f32 = d->out_f32;
  a.scale = 1.f;
  a.tiled = given_half ? d->score_tiled : 0;
  if (v) {                                                   // (null: vt_ws already holds the regrouped V)
    dim3 grid(a.Lkp / 64, d->d_k / 64, d->B * d->Hkv);
    StageScope prof("k_regroup_v", st);
    if ((uintptr_t)v % 16 == 0)
      k_regroup_v<true><<<grid, 256, 0, st>>>((const bf16_t*)v, (bf16_t*)vt_ws, d->Lk, a.Lkp, d->d_k);
    else
      k_regroup_v<false><<<grid, 256, 0, st>>>((const bf16_t*)v, (bf16_t*)vt_ws, d->Lk, a.Lkp, d->d_k);
    int rc = check_launch();
    if (rc) return rc;
  }
  const int n_groups = (d->Lq + SP_GROUP - 1) / SP_GROUP;
  a.pair = 0;
  dim3 grid(d->H, n_groups, d->B);
  StageScope prof("k_softmax_v_mfma", st);
  if (given_half)
    k_std_prefill<true, 2><<<grid, 256, 0, st>>>(a);
  else
    k_std_prefill<true, 1><<<grid, 256, 0, st>>>(a);
  return check_launch();
}

int run_std_prefill_fast(const lisa_desc* d, const void* q, const void* k, const void* v, void* scores,
                         void* out, void* workspace, hipStream_t st) {
  StdPrefillArgs a{};
  a.q = (const bf16_t*)q;
  a.k = (const bf16_t*)k;
  a.vt = (const bf16_t*)workspace;
  a.scores = (half_t*)scores;
  a.out = out;
  a.H = d->H;
  a.Hkv = d->Hkv;
  a.Lq = d->Lq;
  a.Lk = d->Lk;
  a.Lkp = (d->Lk + 63) / 64 * 64;
  a.causal = d->causal;
  a.out_f32 = d->out_f32;
  a.tiled = d->score_tiled;
  a.scale = pick_scale(d->std_scale, d->d_k);
  if (out) {
    dim3 grid(a.Lkp / 64, d->d_k / 64, d->B * d->Hkv);
    StageScope prof("k_regroup_v", st);
    if ((uintptr_t)v % 16 == 0)
      k_regroup_v<true><<<grid, 256, 0, st>>>((const bf16_t*)v, (bf16_t*)workspace, d->Lk, a.Lkp, d->d_k);
    else
      k_regroup_v<false><<<grid, 256, 0, st>>>((const bf16_t*)v, (bf16_t*)workspace, d->Lk, a.Lkp, d->d_k);
    int rc = check_launch();
    if (rc) return rc;
  }
  const int n_groups = (d->Lq + SP_GROUP - 1) / SP_GROUP;
  // One row group per workgroup, long ones first: the dispatcher evens out the rest.  (The kernel
  // can also take the x-th longest and the x-th shortest row group in one workgroup, equal work
  // for all; measured equal on the LLaMA2-13B shape at L = 4096, 3 - 7 % slower at L = 8192 with
  // grouped keys and 10 % slower at L = 2048, where it leaves one workgroup per compute unit.)
  a.pair = 0;
  if (g_tune[LISA_TUNE_STD_PAIR] >= 0) a.pair = g_tune[LISA_TUNE_STD_PAIR] != 0;   // tests force either
  dim3 grid(d->H, a.pair ? (n_groups + 1) / 2 : n_groups, d->B);
  StageScope prof("k_std_prefill", st);
  if (out)
    k_std_prefill<true><<<grid, 256, 0, st>>>(a);
  else
    k_std_prefill<false><<<grid, 256, 0, st>>>(a);
  int rc = check_launch();
  if (rc == LISA_OK) g_path = "mfma_std";
  return rc;
}

}  // namespace

extern "C" {

int lisa_cache_fill(const lisa_desc* d, const void* k_lr, const void* v, void* k_lr_cache, void* v_cache,
                    void* hip_stream) {
  if (!d || !k_lr || !v || !k_lr_cache || !v_cache) return LISA_ERR_NULL;
  if (d->dtype != LISA_F32 && d->dtype != LISA_BF16) return LISA_ERR_UNSUPPORTED;
  if (d->B < 1 || d->Hkv < 1 || d->Lk < 1 || d->r < 1 || d->d_k < 1 || d->Lmax < d->Lk) return LISA_ERR_SHAPE;
  if (d->kcache_dim_major != 0 && d->kcache_dim_major != 1) return LISA_ERR_SHAPE;
  if (d->kcache_dim_major && d->r > 128) return LISA_ERR_UNSUPPORTED;
  // grid limits: (B, Hkv) and B * Hkv are grid.z / grid.y indices, a row of Lk * width elements
  // is covered by 1024 elements per block along grid.x
  if (d->B > kMaxGridYZ || d->Hkv > kMaxGridYZ || (long long)d->B * d->Hkv > kMaxGridYZ)
    return LISA_ERR_UNSUPPORTED;
  if (d->r > kMaxRank || d->d_k > kMaxHeadDim) return LISA_ERR_UNSUPPORTED;
  const void* ptrs[] = {k_lr, v, k_lr_cache, v_cache};
  for (const void* p : ptrs)
    if (!aligned16(p)) return LISA_ERR_ALIGN;
  hipStream_t st = (hipStream_t)hip_stream;
  const int rows = d->B * d->Hkv;
  auto fill_rows = [&](const void* src, void* dst, int row_elems) {
    dim3 grid((unsigned)(((size_t)d->Lk * row_elems + 1023) / 1024), rows);
    if (d->dtype == LISA_F32)
      k_cache_fill_rows<float><<<grid, 256, 0, st>>>((const float*)src, (float*)dst, d->Lk, row_elems, d->Lmax);
    else
      k_cache_fill_rows<bf16_t><<<grid, 256, 0, st>>>((const bf16_t*)src, (bf16_t*)dst, d->Lk, row_elems, d->Lmax);
    return check_launch();
  };
  int rc;
  if (d->kcache_dim_major) {
    dim3 grid((d->Lk + 63) / 64, d->Hkv, d->B);
    if (d->dtype == LISA_F32)
      k_kcache_fill_dim_major<float><<<grid, 256, 0, st>>>((const float*)k_lr, (float*)k_lr_cache, d->Hkv, d->Lk,
                                                          d->r, d->Lmax);
    else
      k_kcache_fill_dim_major<bf16_t><<<grid, 256, 0, st>>>((const bf16_t*)k_lr, (bf16_t*)k_lr_cache, d->Hkv,
                                                           d->Lk, d->r, d->Lmax);
    rc = check_launch();
  } else {
    rc = fill_rows(k_lr, k_lr_cache, d->r);
  }
  if (rc) return rc;
  rc = fill_rows(v, v_cache, d->d_k);
  if (rc == LISA_OK) g_path = "cache_fill";
  return rc;
}

int lisa_project_qkv(const lisa_proj_desc* d, const void* x, const void* w, void* q_lr, void* k_lr, void* v,
                     void* hip_stream) {
  if (!d || !x || !w || !q_lr || !k_lr || !v) return LISA_ERR_NULL;
  if (d->dtype != LISA_F32 && d->dtype != LISA_BF16) return LISA_ERR_UNSUPPORTED;
  if (d->B < 1 || d->L < 1 || d->d_model < 1 || d->H < 1 || d->Hkv < 1 || d->r < 1 || d->d_k < 1 ||
      d->pos0 < 0)
    return LISA_ERR_SHAPE;
  if (d->H % d->Hkv != 0) return LISA_ERR_SHAPE;
  if (d->kcache_dim_major != 0 && d->kcache_dim_major != 1) return LISA_ERR_SHAPE;
  if (!(d->rope_theta >= 0.f) || !std::isfinite(d->rope_theta)) return LISA_ERR_SHAPE;
  if (d->rope_theta > 0.f && d->r % 2 != 0) return LISA_ERR_SHAPE;
  if ((long long)d->pos0 + d->L > 0x7fffffffLL) return LISA_ERR_SHAPE;
  const int Lmax = d->Lmax > 0 ? d->Lmax : d->pos0 + d->L;
  if (Lmax < d->pos0 + d->L) return LISA_ERR_SHAPE;
  if ((long long)d->B * d->L > 0x7fffffffLL) return LISA_ERR_UNSUPPORTED;
  if (!aligned16(x) || !aligned16(w) || !aligned16(q_lr) || !aligned16(k_lr) || !aligned16(v))
    return LISA_ERR_ALIGN;
  hipStream_t st = (hipStream_t)hip_stream;
  ProjectArgs a{};
  a.x = x; a.w = w; a.q_lr = q_lr; a.k_lr = k_lr; a.v = v;
  a.B = d->B; a.L = d->L; a.D = d->d_model; a.H = d->H; a.Hkv = d->Hkv; a.r = d->r; a.dk = d->d_k;
  a.Lmax = Lmax; a.pos0 = d->pos0; a.k_dim_major = d->kcache_dim_major;
  a.rope = d->rope_theta > 0.f;
  a.freq_log2 = a.rope ? -2.0 * std::log2((double)d->rope_theta) / d->r : 0.0;
  const long long M = (long long)d->B * d->L;
  const long long n_real = (long long)(d->H + d->Hkv) * d->r + (long long)d->Hkv * d->d_k;
  const bool fast = d->dtype == LISA_BF16 && d->d_model % PJ_TK == 0 && d->r <= PJ_HEADW &&
                    d->d_k % 32 == 0;
  const char* path;
  if (fast && M <= 128) {
    // a decode step: few rows, bound by one pass over the weights
    const long long n_virtual = (long long)PJ_HEADW * (d->H + d->Hkv) + (long long)d->Hkv * d->d_k;
    const int mb = (int)((M + 31) / 32);
    // both operands through the LDS (whole-line loads) where the reduction axis splits into whole
    // chunks per wave and the staging regions fit
    const bool staged = d->d_model % 512 == 0 && mb <= 2;
    const int lds = std::max(8 * mb * 16 * 64 * (int)sizeof(float), staged ? 8 * (1 + mb) * 32 * PJS_ROW : 0);
    StageScope scope("k_project_skinny", st);
    auto launch = [&](auto kern) -> int {
      hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
      if (e != hipSuccess) return hip_fail(e);
      kern<<<dim3((unsigned)((n_virtual + 31) / 32)), 512, lds, st>>>(a);
      return LISA_OK;
    };
    int lrc = staged ? (mb == 1 ? launch(k_project_skinny_lds<1>) : launch(k_project_skinny_lds<2>))
            : mb == 1 ? launch(k_project_skinny<1>) : mb == 2 ? launch(k_project_skinny<2>)
            : mb == 3 ? launch(k_project_skinny<3>) : launch(k_project_skinny<4>);
    if (lrc) return lrc;
    path = "project_skinny";
  } else if (fast) {
    const long long n_virtual = (long long)PJ_HEADW * (d->H + d->Hkv) + (long long)d->Hkv * d->d_k;
    // tile width: the one whose workgroups fill the 256 CUs in fewer, fuller rounds (a round costs
    // in proportion to the tile width); the wider tile on a tie
    auto rounds_cost = [&](int tn) {
      const long long wgs = ((M + 255) / 256) * ((n_virtual + tn - 1) / tn);
      return ((wgs + kComputeUnits - 1) / kComputeUnits) * tn;
    };
    // (the narrower tile does less MFMA work per fetched byte: it must win by a margin)
    int tn = rounds_cost(192) * 8 < rounds_cost(256) * 7 ? 192 : 256;
    {                                                       // tests force either geometry
      const int v = g_tune[LISA_TUNE_PROJECT_TN];
      if (v == 192 || v == 256) tn = v;
    }
    a.n_m = (int)((M + 255) / 256);
    a.n_n = (int)((n_virtual + tn - 1) / tn);
    // which axis of the tile grid an XCD keeps to: the one that is balanced over 8 XCDs and
    // re-reads fewer operand bytes
    const bool n_ok = a.n_n % 8 == 0 || a.n_n >= 40, m_ok = a.n_m % 8 == 0 || a.n_m >= 40;
    const double xb = (double)M * d->d_model, wb = (double)n_real * d->d_model;
    a.own_n = n_ok && (!m_ok || wb / 8 + xb <= xb / 8 + wb);
    const int per_xcd = a.own_n ? (a.n_n + 7) / 8 * a.n_m : (a.n_m + 7) / 8 * a.n_n;
    StageScope scope("k_project_mfma", st);
    if (tn == 256) {
      auto kern = k_project_mfma<2, 4, 4, 2>;
      constexpr int lds = ProjTile<2, 4, 4, 2>::LDS;
      hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
      if (e != hipSuccess) return hip_fail(e);
      kern<<<dim3(8 * per_xcd), 512, lds, st>>>(a);
    } else {
      auto kern = k_project_mfma<4, 2, 2, 3>;
      constexpr int lds = ProjTile<4, 2, 2, 3>::LDS;
      hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
      if (e != hipSuccess) return hip_fail(e);
      kern<<<dim3(8 * per_xcd), 512, lds, st>>>(a);
    }
    path = "project_mfma";
  } else {
    const long long total = M * n_real;
    if ((total + 255) / 256 > 0x7fffffffLL) return LISA_ERR_UNSUPPORTED;
    StageScope scope("k_project_generic", st);
    dim3 grid((unsigned)((total + 255) / 256));
    if (d->dtype == LISA_F32)
      k_project_generic<float, double><<<grid, 256, 0, st>>>(a);
    else
      k_project_generic<bf16_t, float><<<grid, 256, 0, st>>>(a);
    path = "project_generic";
  }
  int rc = check_launch();
  if (rc == LISA_OK) g_path = path;
  return rc;
}

size_t lisa_score_elem_bytes(const lisa_desc* desc) {
  if (!desc || (desc->dtype != LISA_F32 && desc->dtype != LISA_BF16)) return 0;
  return score_elem(desc);
}

size_t lisa_scores_bytes(const lisa_desc* desc) {
  if (check_common(desc) != LISA_OK) return 0;
  return scores_bytes(desc);
}

size_t lisa_kcache_saved_bytes(const lisa_desc* desc, int n_lisa_layers) {
  if (check_common(desc) != LISA_OK || desc->r <= 0 || desc->r > desc->d_k || n_lisa_layers < 0)
    return 0;
  const size_t e = desc->dtype == LISA_F32 ? 4 : 2;
  return (size_t)n_lisa_layers * desc->B * desc->Hkv * desc->Lk * (size_t)(desc->d_k - desc->r) * e;
}

// The single-layer alignment FFN (y = W^T x), LiSA_plus (y = x) and direct sharing (y = x, no
// correction) are two-layer ReLU networks in disguise ([W,-W] then [I;-I]: relu(u) - relu(-u) = u),
// so they can run on the MFMA kernels, which implement ADD with ReLU: `eq` receives the
// equivalent descriptor (F = 2H).  The hidden units pass through half precision there, as for the
// two-layer form.  Direct sharing gets all-zero low-rank operands of width kShareRank, built in
// the workspace, so that its correction is exactly zero.
constexpr int kShareRank = 8;
bool relu_equivalent(const lisa_desc* d, lisa_desc* eq) {
  if (d->dtype != LISA_BF16) return false;
  const bool ffn = d->mix == LISA_MIX_ADD || d->mix == LISA_MIX_CONCAT;
  if (ffn && d->act != LISA_ACT_SINGLE) return false;      // two-layer forms run as they are
  if (2 * d->H > 128) return false;
  *eq = *d;
  eq->mix = d->mix == LISA_MIX_CONCAT ? LISA_MIX_CONCAT : LISA_MIX_ADD;
  eq->act = LISA_ACT_RELU;
  eq->F = 2 * d->H;
  if (d->mix == LISA_MIX_SHARE) eq->r = kShareRank;
  return true;
}
// Scratch behind the kernels' own workspace: the equivalent weights, then (direct sharing) the
// zero Q_LR [B,H,Lq,r0] and the zero K_LR (Lq > 1: [B,Hkv,Lk,r0]; decode: the cache shape).
struct SynthWs {
  size_t w, q0, k0, total;
};
SynthWs synth_ws(const lisa_desc* d) {
  SynthWs s;
  s.w = 0;
  const size_t Din = d->mix == LISA_MIX_CONCAT ? 2 * d->H : d->H;
  s.q0 = round_up((2 * Din * d->H + (size_t)2 * d->H * d->H) * 2, 256);
  s.k0 = s.q0;
  s.total = s.q0;
  if (d->mix == LISA_MIX_SHARE) {
    const size_t klen = d->Lq == 1 ? (size_t)d->Lmax : (size_t)d->Lk;
    s.k0 = s.q0 + round_up((size_t)d->B * d->H * d->Lq * kShareRank * 2, 256);
    s.total = s.k0 + round_up((size_t)d->B * d->Hkv * klen * kShareRank * 2, 256);
  }
  return s;
}
size_t synth_ffn_bytes(const lisa_desc* d) { return synth_ws(d).total; }

// Writes the equivalent operands behind `offset` bytes of the workspace; returns their addresses
// (q_lr / k_lr are replaced only for direct sharing).
int synth_relu_ffn(const lisa_desc* d, const void* w1_user, void* workspace, size_t offset, const void** w1o,
                   const void** w2o, const void** q_lr, const void** k_lr, hipStream_t st) {
  const SynthWs sw = synth_ws(d);
  char* base = (char*)workspace + offset;
  const int Din = d->mix == LISA_MIX_CONCAT ? 2 * d->H : d->H;
  const bool ffn = d->mix == LISA_MIX_ADD || d->mix == LISA_MIX_CONCAT;
  bf16_t* a = (bf16_t*)(base + sw.w);
  bf16_t* b = a + (size_t)2 * Din * d->H;
  StageScope prof("k_synth_relu_ffn", st);
  k_synth_relu_ffn<bf16_t><<<(2 * Din * d->H + 2 * d->H * d->H + 255) / 256, 256, 0, st>>>(
      ffn ? (const bf16_t*)w1_user : nullptr, a, b, Din, d->H);
  *w1o = a;
  *w2o = b;
  if (d->mix == LISA_MIX_SHARE) {
    const size_t n16 = (sw.total - sw.q0) / 16;
    k_zero16<<<(unsigned)((n16 + 255) / 256), 256, 0, st>>>((uint4*)(base + sw.q0), n16);
    *q_lr = base + sw.q0;
    *k_lr = base + sw.k0;
  }
  return check_launch();
}

// Workgroups of the loss kernel: four score rows each per pass, at most eight per compute unit.
int kd_blocks(const lisa_desc* d) {
  const long long rows = (long long)d->B * d->H * d->Lq;
  return (int)std::min<long long>((rows + 3) / 4, 2048);
}

int lisa_kd_huber(const lisa_desc* desc, const void* scores, const void* teacher, float delta,
                  float weight, int accumulate, double* out, void* workspace,
                  size_t workspace_bytes, void* hip_stream) {
  int rc = check_common(desc);
  if (rc) return rc;
  if (!scores || !teacher || !out) return LISA_ERR_NULL;
  if (!(delta > 0.f) || !std::isfinite(delta) || !std::isfinite(weight)) return LISA_ERR_SHAPE;
  if (accumulate != 0 && accumulate != 1) return LISA_ERR_SHAPE;
  if (desc->score_tiled && desc->dtype != LISA_BF16) return LISA_ERR_UNSUPPORTED;
  if (!aligned16(scores) || !aligned16(teacher) || !aligned16(out) || (workspace && !aligned16(workspace)))
    return LISA_ERR_ALIGN;
  const int n_blocks = kd_blocks(desc);
  if (!workspace || workspace_bytes < (size_t)n_blocks * sizeof(double)) return LISA_ERR_WORKSPACE;
  KdArgs g{};
  g.a = scores;
  g.t = teacher;
  g.part = (double*)workspace;
  g.out = out;
  g.B = desc->B;
  g.H = desc->H;
  g.Lq = desc->Lq;
  g.Lk = desc->Lk;
  g.causal = desc->causal;
  g.tiled = desc->score_tiled;
  g.delta = delta;
  g.weight = weight;
  g.accumulate = accumulate;
  g.n_blocks = n_blocks;
  g.n_rows = (long long)desc->B * desc->H * desc->Lq;
  // visible entries: row i sees min(Lk, i + 1 + Lk - Lq) keys (causal needs Lk >= Lq, checked above)
  double per_head = 0.0;
  if (desc->causal) {
    const double first = (double)desc->Lk - desc->Lq + 1, last = (double)desc->Lk;
    per_head = 0.5 * (first + last) * desc->Lq;
  } else {
    per_head = (double)desc->Lq * desc->Lk;
  }
  g.count = per_head * desc->B * desc->H;
  hipStream_t st = (hipStream_t)hip_stream;
  {
    StageScope prof("k_kd_huber_part", st);
    if (desc->dtype == LISA_F32)
      k_kd_huber_part<float><<<n_blocks, 256, 0, st>>>(g);
    else
      k_kd_huber_part<half_t><<<n_blocks, 256, 0, st>>>(g);
    rc = check_launch();
    if (rc) return rc;
  }
  StageScope prof("k_kd_huber_finish", st);
  k_kd_huber_finish<<<1, 256, 0, st>>>(g);
  rc = check_launch();
  if (rc == LISA_OK) g_path = "kd_huber";
  return rc;
}

size_t lisa_workspace_bytes(const lisa_desc* desc, int which) {
  switch (which) {
    case LISA_WS_PREFILL: {
      if (check_lisa(desc) != LISA_OK) return 0;
      lisa_desc eq;
      if (relu_equivalent(desc, &eq) && prefill_fused_ok(&eq))
        return round_up(prefill_fused_ws(&eq).total, 256) + synth_ffn_bytes(desc);
      if (prefill_fused_ok(desc)) return prefill_fused_ws(desc).total;
      if (scores_mfma_ok(desc)) return concat_ws(desc).total;
      if (relu_equivalent(desc, &eq) && scores_mfma_ok(&eq))
        return round_up(concat_ws(&eq).total, 256) + synth_ffn_bytes(desc);
      return exact_bytes(desc) + (std_prefill_fast_ok(desc) ? std_prefill_ws(desc) : 0);
    }
    case LISA_WS_DECODE: {
      if (check_decode(desc) != LISA_OK) return 0;
      lisa_desc eq;
      if (decode_fast_ok(desc, true)) return decode_fast_bytes(desc);
      if (relu_equivalent(desc, &eq) && decode_fast_ok(&eq, true))
        return round_up(decode_fast_bytes(&eq), 256) + synth_ffn_bytes(desc);
      return exact_bytes(desc);
    }
    case LISA_WS_STD:
      if (check_common(desc) != LISA_OK) return 0;
      // needed only when `out` is requested
      if (std_prefill_fast_ok(desc)) return std_prefill_ws(desc);
      return decode_fast_ok(desc, false) ? decode_fast_bytes(desc) : exact_bytes(desc);
    case LISA_WS_LAYER: {
      size_t q, k, v;
      if (lisa_layer_offsets(desc, &q, &k, &v) != LISA_OK) return 0;
      const size_t e = desc->dtype == LISA_F32 ? 4 : 2;
      return v + round_up((size_t)desc->B * desc->Hkv * desc->Lq * desc->d_k * e, 256);
    }
    case LISA_WS_LAYER_DECODE: {
      if (check_decode(desc) != LISA_OK || !has_delta(desc)) return 0;
      const size_t e = desc->dtype == LISA_F32 ? 4 : 2;
      return round_up(lisa_workspace_bytes(desc, LISA_WS_DECODE), 256) +
             round_up((size_t)desc->B * desc->H * desc->r * e, 256);
    }
    case LISA_WS_KD:
      if (check_common(desc) != LISA_OK) return 0;
      return (size_t)kd_blocks(desc) * sizeof(double);
    default:
      return 0;
  }
}

int lisa_layer_decode(const lisa_desc* desc, int32_t d_model, float rope_theta, const void* x,
                      const void* w_qkv, void* k_lr_cache, void* v_cache, const void* score_row_prev,
                      const void* w1, const void* w2, void* out, void* score_row_out, void* workspace,
                      size_t workspace_bytes, void* hip_stream) {
  int rc = check_decode(desc);
  if (rc) return rc;
  if (!has_delta(desc)) return LISA_ERR_UNSUPPORTED;       // nothing to project for: use lisa_attn_decode
  if (!x || !w_qkv || !k_lr_cache || !v_cache || !score_row_prev || !out) return LISA_ERR_NULL;
  if (!workspace) return LISA_ERR_WORKSPACE;
  if (!aligned16(workspace)) return LISA_ERR_ALIGN;
  if (workspace_bytes < lisa_workspace_bytes(desc, LISA_WS_LAYER_DECODE)) return LISA_ERR_WORKSPACE;
  const size_t qo = round_up(lisa_workspace_bytes(desc, LISA_WS_DECODE), 256);
  lisa_proj_desc pd{};
  pd.dtype = desc->dtype;
  pd.B = desc->B;
  pd.L = 1;
  pd.d_model = d_model;
  pd.H = desc->H;
  pd.Hkv = desc->Hkv;
  pd.r = desc->r;
  pd.d_k = desc->d_k;
  pd.Lmax = desc->Lmax;
  pd.pos0 = desc->Lk - 1;
  pd.kcache_dim_major = desc->kcache_dim_major;
  pd.rope_theta = rope_theta;
  char* ws = (char*)workspace;
  rc = lisa_project_qkv(&pd, x, w_qkv, ws + qo, k_lr_cache, v_cache, hip_stream);
  if (rc) return rc;
  return lisa_attn_decode(desc, ws + qo, nullptr, nullptr, k_lr_cache, v_cache, score_row_prev, w1, w2, out,
                          score_row_out, workspace, qo, hip_stream);
}

int lisa_layer_offsets(const lisa_desc* desc, size_t* q_lr_off, size_t* k_lr_off, size_t* v_off) {
  int rc = check_lisa(desc);
  if (rc) return rc;
  if (!q_lr_off || !k_lr_off || !v_off) return LISA_ERR_NULL;
  if (desc->Lq != desc->Lk) return LISA_ERR_SHAPE;
  const size_t e = desc->dtype == LISA_F32 ? 4 : 2;
  *q_lr_off = round_up(lisa_workspace_bytes(desc, LISA_WS_PREFILL), 256);
  *k_lr_off = *q_lr_off + round_up((size_t)desc->B * desc->H * desc->Lq * desc->r * e, 256);
  *v_off = *k_lr_off + round_up((size_t)desc->B * desc->Hkv * desc->Lq * desc->r * e, 256);
  return LISA_OK;
}

int lisa_layer_prefill(const lisa_desc* desc, int32_t d_model, float rope_theta, const void* x,
                       const void* w_qkv, const void* scores_prev, const void* w1, const void* w2,
                       void* out, void* scores_out, void* workspace, size_t workspace_bytes,
                       void* hip_stream) {
  size_t qo, ko, vo;
  int rc = lisa_layer_offsets(desc, &qo, &ko, &vo);
  if (rc) return rc;
  if (!x || !w_qkv || !scores_prev || !out) return LISA_ERR_NULL;
  if (!has_delta(desc)) return LISA_ERR_UNSUPPORTED;      // nothing to project for: use lisa_attn_prefill
  if (desc->write_scores && !scores_out) return LISA_ERR_NULL;
  if (!workspace || !aligned16(workspace)) return workspace ? LISA_ERR_ALIGN : LISA_ERR_WORKSPACE;
  if (workspace_bytes < lisa_workspace_bytes(desc, LISA_WS_LAYER)) return LISA_ERR_WORKSPACE;
  lisa_proj_desc pd{};
  pd.dtype = desc->dtype;
  pd.B = desc->B;
  pd.L = desc->Lq;
  pd.d_model = d_model;
  pd.H = desc->H;
  pd.Hkv = desc->Hkv;
  pd.r = desc->r;
  pd.d_k = desc->d_k;
  pd.Lmax = desc->Lq;
  pd.rope_theta = rope_theta;
  char* ws = (char*)workspace;
  rc = lisa_project_qkv(&pd, x, w_qkv, ws + qo, ws + ko, ws + vo, hip_stream);
  if (rc) return rc;
  return lisa_attn_prefill(desc, ws + qo, ws + ko, ws + vo, scores_prev, w1, w2, out, scores_out, workspace,
                           qo, hip_stream);
}

int lisa_supported(const lisa_desc* desc) { return check_lisa(desc); }

size_t lisa_scores_elems(const lisa_desc* desc) { return desc ? scores_elems(desc) : 0; }

const char* lisa_strerror(int status) {
  switch (status) {
    case LISA_OK: return "ok";
    case LISA_ERR_NULL: return "a required pointer is NULL";
    case LISA_ERR_SHAPE: return "a dimension or flag is invalid or inconsistent";
    case LISA_ERR_UNSUPPORTED: return "valid request outside the supported kernel range";
    case LISA_ERR_ALIGN: return "a base pointer is not 16-byte aligned";
    case LISA_ERR_WORKSPACE: return "workspace missing or too small";
    case LISA_ERR_HIP: return "a HIP call failed (see lisa_last_hip_error)";
    case LISA_ERR_SCRATCH:
      return "the problem needs more scratch than the static buffer of lisa_attn_decode_static holds";
    default: return "unknown status";
  }
}

int lisa_profile_enable(int on) {
  for (ProfRec& r : g_prof_recs) {
    g_prof_pool.push_back(r.beg);
    g_prof_pool.push_back(r.end);
  }
  g_prof_recs.clear();
  g_prof_on = on != 0;
  return LISA_OK;
}

int lisa_profile_collect(lisa_stage_time* out, int max_stages) {
  if (!out && max_stages > 0) return LISA_ERR_NULL;
  int n = 0;
  int rc = LISA_OK;
  for (ProfRec& r : g_prof_recs) {
    float ms = 0.f;
    hipError_t e = hipEventSynchronize(r.end);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.beg, r.end);
    if (e != hipSuccess) rc = hip_fail(e);
    g_prof_pool.push_back(r.beg);
    g_prof_pool.push_back(r.end);
    if (e != hipSuccess) continue;
    int s = 0;
    while (s < n && std::strcmp(out[s].name, r.name) != 0) ++s;
    if (s == n) {
      if (n >= max_stages) continue;
      out[n].name = r.name;
      out[n].launches = 0;
      out[n].total_ms = 0.f;
      ++n;
    }
    out[s].launches += 1;
    out[s].total_ms += ms;
  }
  g_prof_recs.clear();
  return rc == LISA_OK ? n : rc;
}

int lisa_tune_set(int knob, int value) {
  if (knob < 0 || knob >= LISA_TUNE_COUNT) return LISA_ERR_SHAPE;
  g_tune[knob] = value < 0 ? -1 : value;
  return LISA_OK;
}

int lisa_probe_hbm_read(const void* src, size_t bytes, void* sink, void* hip_stream) {
  if (!src || !sink) return LISA_ERR_NULL;
  if (!aligned16(src) || !aligned16(sink)) return LISA_ERR_ALIGN;
  if (bytes < 16) return LISA_ERR_SHAPE;
  k_probe_read<<<8 * kComputeUnits, 256, 0, (hipStream_t)hip_stream>>>((const probe_u32x4*)src, bytes / 16, (probe_u32x4*)sink);
  return check_launch();
}

int lisa_probe_hbm_write(void* dst, size_t bytes, unsigned seed, void* hip_stream) {
  if (!dst) return LISA_ERR_NULL;
  if (!aligned16(dst)) return LISA_ERR_ALIGN;
  if (bytes < 16) return LISA_ERR_SHAPE;
  k_probe_write<<<8 * kComputeUnits, 256, 0, (hipStream_t)hip_stream>>>((probe_u32x4*)dst, bytes / 16, seed);
  return check_launch();
}

int lisa_probe_mfma(int shape, int iters, int workgroups, void* sink, void* hip_stream) {
  if (!sink) return LISA_ERR_NULL;
  if ((shape != 0 && shape != 1) || iters < 1 || workgroups < 1 || workgroups > 65536) return LISA_ERR_SHAPE;
  hipStream_t st = (hipStream_t)hip_stream;
  if (shape == 0) k_probe_mfma<0><<<workgroups, 256, 0, st>>>(iters, 0.25f, (float*)sink);
  else k_probe_mfma<1><<<workgroups, 256, 0, st>>>(iters, 0.25f, (float*)sink);
  return check_launch();
}

const char* lisa_last_hip_error(void) { return g_hip_err; }
const char* lisa_last_path(void) { return g_path; }

int lisa_attn_prefill(const lisa_desc* desc, const void* q_lr, const void* k_lr, const void* v,
                      const void* scores_prev, const void* w1, const void* w2, void* out,
                      void* scores_out, void* workspace, size_t workspace_bytes,
                      void* hip_stream) {
  int rc = check_lisa(desc);
  if (rc) return rc;
  if (!v || !scores_prev || !out) return LISA_ERR_NULL;
  if (has_delta(desc) && (!q_lr || !k_lr)) return LISA_ERR_NULL;
  if ((has_ffn(desc) && !w1) || (has_w2(desc) && !w2)) return LISA_ERR_NULL;
  if (desc->write_scores && !scores_out) return LISA_ERR_NULL;
  if (desc->write_scores && scores_out == scores_prev) return LISA_ERR_SHAPE;
  const void* ptrs[] = {q_lr, k_lr, v, scores_prev, w1, w2, out, scores_out, workspace};
  for (const void* p : ptrs)
    if (p && !aligned16(p)) return LISA_ERR_ALIGN;
  if (!workspace || workspace_bytes < lisa_workspace_bytes(desc, LISA_WS_PREFILL))
    return LISA_ERR_WORKSPACE;
  void* scores = desc->write_scores ? scores_out : nullptr;
  float* exact = (float*)workspace;
  hipStream_t st = (hipStream_t)hip_stream;
  const KeyStrides ks = dense_keys(desc, desc->Lk, desc->r);
  const KeyStrides vs = dense_keys(desc, desc->Lk, desc->d_k);
  if (prefill_fused_ok(desc))
    return run_prefill_fused(desc, q_lr, k_lr, v, scores_prev, w1, w2, out, scores, workspace, st);
  lisa_desc eq;
  if (relu_equivalent(desc, &eq) && prefill_fused_ok(&eq)) {
    const void *w1e, *w2e;
    rc = synth_relu_ffn(desc, w1, workspace, round_up(prefill_fused_ws(&eq).total, 256), &w1e, &w2e, &q_lr, &k_lr,
                        st);
    if (rc) return rc;
    return run_prefill_fused(&eq, q_lr, k_lr, v, scores_prev, w1e, w2e, out, scores, workspace, st);
  }
  // tiles are read and written by the fused kernels and by the matrix-core CONCAT pipeline alone
  if (desc->score_tiled && !concat_tiled_ok(desc) && !(relu_equivalent(desc, &eq) && concat_tiled_ok(&eq)))
    return LISA_ERR_UNSUPPORTED;
  if (relu_equivalent(desc, &eq) && scores_mfma_ok(&eq)) {   // the single layer over the concatenation
    const void *w1e, *w2e;
    rc = synth_relu_ffn(desc, w1, workspace, round_up(concat_ws(&eq).total, 256), &w1e, &w2e, &q_lr, &k_lr, st);
    if (rc) return rc;
    return run_lisa<bf16_t, half_t>(&eq, q_lr, k_lr, ks, v, vs, scores_prev, w1e, w2e, out, scores, exact, st);
  }
  if (desc->dtype == LISA_F32)
    return run_lisa<float, float>(desc, q_lr, k_lr, ks, v, vs, scores_prev, w1, w2, out, scores,
                                  exact, st);
  return run_lisa<bf16_t, half_t>(desc, q_lr, k_lr, ks, v, vs, scores_prev, w1, w2, out, scores,
                                  exact, st);
}

// Argument checks of the decode step that need no workspace (host only).
static int check_decode_args(const lisa_desc* desc, const void* q_lr, const void* k_lr_new, const void* v_new,
                             void* k_lr_cache, void* v_cache, const void* score_row_prev, const void* w1,
                             const void* w2, void* out, void* score_row_out) {
  int rc = check_decode(desc);
  if (rc) return rc;
  if (!v_cache || !score_row_prev || !out) return LISA_ERR_NULL;
  if (has_delta(desc) && (!q_lr || !k_lr_cache)) return LISA_ERR_NULL;
  if ((has_ffn(desc) && !w1) || (has_w2(desc) && !w2)) return LISA_ERR_NULL;
  if ((k_lr_new == nullptr) != (v_new == nullptr)) return LISA_ERR_NULL;
  if (k_lr_new && !k_lr_cache) return LISA_ERR_NULL;
  if (desc->write_scores && !score_row_out) return LISA_ERR_NULL;
  if (desc->write_scores && score_row_out == score_row_prev) return LISA_ERR_SHAPE;
  const void* ptrs[] = {q_lr, k_lr_new, v_new, k_lr_cache, v_cache, score_row_prev, w1, w2, out, score_row_out};
  for (const void* p : ptrs)
    if (p && !aligned16(p)) return LISA_ERR_ALIGN;
  return LISA_OK;
}

// The decode step itself: arguments already checked, `workspace` holds at least
// lisa_workspace_bytes(desc, LISA_WS_DECODE) bytes.
static int run_attn_decode(const lisa_desc* desc, const void* q_lr, const void* k_lr_new, const void* v_new,
                           void* k_lr_cache, void* v_cache, const void* score_row_prev, const void* w1,
                           const void* w2, void* out, void* score_row_out, void* workspace, hipStream_t st) {
  int rc;
  void* scores = desc->write_scores ? score_row_out : nullptr;
  float* exact = (float*)workspace;
  KeyStrides ks = desc->kcache_dim_major ? dim_major_keys(desc, desc->Lmax, desc->r)
                                               : dense_keys(desc, desc->Lmax, desc->r);
  const KeyStrides vs = dense_keys(desc, desc->Lmax, desc->d_k);
  if (k_lr_new) {
    dim3 grid(desc->Hkv, desc->B);
    if (desc->dtype == LISA_F32)
      k_append<float><<<grid, 128, 0, st>>>((const float*)k_lr_new, (const float*)v_new,
                                            (float*)k_lr_cache, ks, (float*)v_cache, vs, desc->Hkv,
                                            desc->r, desc->d_k, desc->Lk - 1);
    else
      k_append<bf16_t><<<grid, 128, 0, st>>>((const bf16_t*)k_lr_new, (const bf16_t*)v_new,
                                             (bf16_t*)k_lr_cache, ks, (bf16_t*)v_cache, vs,
                                             desc->Hkv, desc->r, desc->d_k, desc->Lk - 1);
    rc = check_launch();
    if (rc) return rc;
  }
  lisa_desc eq;
  const lisa_desc* eff = desc;                             // the descriptor the fast kernels see
  if (!decode_fast_ok(desc, true) && relu_equivalent(desc, &eq) && decode_fast_ok(&eq, true)) {
    const void* k0 = k_lr_cache;
    rc = synth_relu_ffn(desc, w1, workspace, round_up(decode_fast_bytes(&eq), 256), &w1, &w2, &q_lr, &k0, st);
    if (rc) return rc;
    eff = &eq;
    if (desc->mix == LISA_MIX_SHARE) {                     // the all-zero K_LR cache of the equivalent layer
      k_lr_cache = const_cast<void*>(k0);
      ks = desc->kcache_dim_major ? dim_major_keys(eff, eff->Lmax, eff->r) : dense_keys(eff, eff->Lmax, eff->r);
    }
  }
  if (decode_fast_ok(eff, true)) {
    DecodeArgs a{};
    a.q = (const bf16_t*)q_lr;
    a.kc = (const bf16_t*)k_lr_cache;
    a.ks = ks;
    a.vc = (const bf16_t*)v_cache;
    a.vs = vs;
    a.prev = (const half_t*)score_row_prev;
    a.w1 = (const bf16_t*)w1;
    a.w2 = (const bf16_t*)w2;
    a.row_out = (half_t*)scores;
    return run_decode_fast(eff, true, a, out, workspace, st);
  }
  if (desc->dtype == LISA_F32)
    return run_lisa<float, float>(desc, q_lr, k_lr_cache, ks, v_cache, vs, score_row_prev, w1, w2,
                                  out, scores, exact, st);
  return run_lisa<bf16_t, half_t>(desc, q_lr, k_lr_cache, ks, v_cache, vs, score_row_prev, w1, w2,
                                  out, scores, exact, st);
}

int lisa_attn_decode(const lisa_desc* desc, const void* q_lr, const void* k_lr_new,
                     const void* v_new, void* k_lr_cache, void* v_cache,
                     const void* score_row_prev, const void* w1, const void* w2, void* out,
                     void* score_row_out, void* workspace, size_t workspace_bytes,
                     void* hip_stream) {
  int rc = check_decode_args(desc, q_lr, k_lr_new, v_new, k_lr_cache, v_cache, score_row_prev, w1, w2, out,
                             score_row_out);
  if (rc) return rc;
  if (workspace && !aligned16(workspace)) return LISA_ERR_ALIGN;
  if (!workspace || workspace_bytes < lisa_workspace_bytes(desc, LISA_WS_DECODE))
    return LISA_ERR_WORKSPACE;
  return run_attn_decode(desc, q_lr, k_lr_new, v_new, k_lr_cache, v_cache, score_row_prev, w1, w2, out,
                         score_row_out, workspace, (hipStream_t)hip_stream);
}

int lisa_attn_decode_static(const lisa_desc* desc, const void* q_lr, const void* k_lr_new,
                            const void* v_new, void* k_lr_cache, void* v_cache,
                            const void* score_row_prev, const void* w1, const void* w2, void* out,
                            void* score_row_out, void* hip_stream) {
  int rc = check_decode_args(desc, q_lr, k_lr_new, v_new, k_lr_cache, v_cache, score_row_prev, w1, w2, out,
                             score_row_out);
  if (rc) return rc;
  if (lisa_workspace_bytes(desc, LISA_WS_DECODE) > (size_t)LISA_STATIC_SCRATCH_BYTES) return LISA_ERR_SCRATCH;
  void* ws = nullptr;
  rc = static_scratch(&ws);
  if (rc) return rc;
  // stage timing creates HIP events: not in a call that promises to allocate nothing
  const bool prof = g_prof_on;
  g_prof_on = false;
  rc = run_attn_decode(desc, q_lr, k_lr_new, v_new, k_lr_cache, v_cache, score_row_prev, w1, w2, out,
                       score_row_out, ws, (hipStream_t)hip_stream);
  g_prof_on = prof;
  return rc;
}

// ---- a decode step through a stack of layers (Sec. 5.1: which layers share attention) -------------
namespace {
struct StackWs {
  size_t rows, layer, half, total;   // byte offsets: two score rows, then two per-layer workspaces of `half` bytes
};
// Descriptors of the three kinds of layer, derived from the LiSA layer's.
void stack_descs(const lisa_desc* d, lisa_desc* std_d, lisa_desc* share_d) {
  *std_d = *d;
  std_d->mix = LISA_MIX_ADD;
  std_d->act = LISA_ACT_RELU;
  std_d->r = 0;
  std_d->F = 0;
  std_d->write_scores = 0;
  std_d->kcache_dim_major = 0;
  *share_d = *d;
  share_d->mix = LISA_MIX_SHARE;
}
StackWs stack_ws(const lisa_desc* d) {
  lisa_desc sd, hd;
  stack_descs(d, &sd, &hd);
  StackWs w;
  w.rows = 0;
  w.layer = round_up(2 * scores_bytes(d), 256);
  const size_t a = lisa_workspace_bytes(d, LISA_WS_DECODE), b = lisa_workspace_bytes(&hd, LISA_WS_DECODE),
               c = lisa_workspace_bytes(&sd, LISA_WS_STD);
  // (two of them, used in turn: the partial results of a layer wait there for the launch of the
  // next layer, which combines them)
  w.half = round_up(std::max(a, std::max(b, c)), 256);
  w.total = w.layer + 2 * w.half;
  return w;
}
}  // namespace

size_t lisa_stack_workspace_bytes(const lisa_desc* desc) {
  if (check_decode(desc) != LISA_OK) return 0;
  return stack_ws(desc).total;
}

int lisa_decode_stack(const lisa_desc* desc, const lisa_stack_layer* layers, int32_t n_layers, void* workspace,
                      size_t workspace_bytes, void* hip_stream) {
  int rc = check_decode(desc);
  if (rc) return rc;
  if (!layers) return LISA_ERR_NULL;
  if (n_layers < 1) return LISA_ERR_SHAPE;
  if (desc->mix == LISA_MIX_SHARE) return LISA_ERR_SHAPE;   // (direct sharing is a kind of layer, not of stack)
  // the whole stack is checked on the host before the first launch
  for (int n = 0; n < n_layers; ++n) {
    const lisa_stack_layer& ly = layers[n];
    if (ly.kind < LISA_LAYER_STD || ly.kind > LISA_LAYER_SHARE) return LISA_ERR_SHAPE;
    if (n == 0 && ly.kind != LISA_LAYER_STD) return LISA_ERR_SHAPE;   // a sharing layer needs a front layer
    if (!ly.v_cache || !ly.out) return LISA_ERR_NULL;
    if (ly.kind != LISA_LAYER_SHARE && (!ly.q || !ly.k_cache)) return LISA_ERR_NULL;
    if (ly.kind == LISA_LAYER_LISA && ((has_ffn(desc) && !ly.w1) || (has_w2(desc) && !ly.w2))) return LISA_ERR_NULL;
    const void* ptrs[] = {ly.q, ly.k_cache, ly.v_cache, ly.w1, ly.w2, ly.out, ly.score_row};
    for (const void* p : ptrs)
      if (p && !aligned16(p)) return LISA_ERR_ALIGN;
  }
  if (!workspace) return LISA_ERR_WORKSPACE;
  if (!aligned16(workspace)) return LISA_ERR_ALIGN;
  const StackWs w = stack_ws(desc);
  if (workspace_bytes < w.total) return LISA_ERR_WORKSPACE;
  lisa_desc std_d, share_d;
  stack_descs(desc, &std_d, &share_d);
  char* ws = (char*)workspace;
  void* own[2] = {ws + w.rows, ws + w.rows + scores_bytes(desc)};
  const size_t lws_bytes = w.half;
  const void* cur = nullptr;                                 // the row A_{n-1} that the next layer may share
  hipStream_t st = (hipStream_t)hip_stream;
  g_dc = DeferredCombine{};
  g_dc.on = true;
  for (int n = 0; n < n_layers && rc == LISA_OK; ++n) {
    const lisa_stack_layer& ly = layers[n];
    void* lws = ws + w.layer + (n & 1) * w.half;
    const long calls_before = g_dc.fast_calls;
    const bool next_shares = n + 1 < n_layers && layers[n + 1].kind != LISA_LAYER_STD;
    void* dst = ly.score_row ? ly.score_row : (cur == own[0] ? own[1] : own[0]);
    if (ly.kind == LISA_LAYER_STD) {
      // its row is emitted only if somebody reads it
      const bool emit = next_shares || ly.score_row;
      rc = std_attn_scores(&std_d, ly.q, ly.k_cache, ly.v_cache, emit ? dst : nullptr, ly.out, lws, lws_bytes,
                           hip_stream);
      cur = emit ? dst : nullptr;
    } else if (ly.kind == LISA_LAYER_LISA) {
      lisa_desc d = *desc;
      d.write_scores = next_shares || ly.score_row;
      rc = lisa_attn_decode(&d, ly.q, nullptr, nullptr, ly.k_cache, ly.v_cache, cur, ly.w1, ly.w2, ly.out,
                            d.write_scores ? dst : nullptr, lws, lws_bytes, hip_stream);
      cur = d.write_scores ? dst : nullptr;
    } else {
      // direct sharing: A_n = A_{n-1}; the row passes through untouched unless the caller wants a copy
      share_d.write_scores = ly.score_row != nullptr;
      rc = lisa_attn_decode(&share_d, nullptr, nullptr, nullptr, nullptr, ly.v_cache, cur, nullptr, nullptr, ly.out,
                            share_d.write_scores ? dst : nullptr, lws, lws_bytes, hip_stream);
      if (share_d.write_scores) cur = dst;
    }
    // a layer that ran on other kernels took no combine with it: the one owed goes out now, before
    // its half of the workspace comes round again
    if (rc == LISA_OK && g_dc.fast_calls == calls_before) rc = flush_deferred_combine(st);
  }
  if (rc == LISA_OK) rc = flush_deferred_combine(st);
  g_dc = DeferredCombine{};
  return rc;
}

int std_attn_scores(const lisa_desc* desc, const void* q, const void* k, const void* v,
                    void* scores_out, void* out, void* workspace, size_t workspace_bytes,
                    void* hip_stream) {
  int rc = check_common(desc);
  if (rc) return rc;
  if (!q || !k) return LISA_ERR_NULL;
  if (!scores_out && !out) return LISA_ERR_NULL;
  if ((v == nullptr) != (out == nullptr)) return LISA_ERR_NULL;
  // Lmax is the capacity of K / V along the keys in the decode form (0: dense); a capacity below
  // the attended length, or one given for a prefill call, is a mistake of the caller
  if (desc->Lmax < 0 || (desc->Lmax > 0 && (desc->Lq != 1 || desc->Lmax < desc->Lk))) return LISA_ERR_SHAPE;
  const void* ptrs[] = {q, k, v, scores_out, out, workspace};
  for (const void* p : ptrs)
    if (p && !aligned16(p)) return LISA_ERR_ALIGN;
  float* exact = nullptr;
  if (out) {
    if (!workspace || workspace_bytes < lisa_workspace_bytes(desc, LISA_WS_STD))
      return LISA_ERR_WORKSPACE;
    exact = (float*)workspace;
  }
  hipStream_t st = (hipStream_t)hip_stream;
  // With Lq = 1 and Lmax set, K and V are caches of capacity Lmax along the key axis.
  const int cap = (desc->Lq == 1 && desc->Lmax >= desc->Lk) ? desc->Lmax : desc->Lk;
  const KeyStrides ks = dense_keys(desc, cap, desc->d_k);
  if (std_prefill_fast_ok(desc)) return run_std_prefill_fast(desc, q, k, v, scores_out, out, workspace, st);
  if (desc->score_tiled) return LISA_ERR_UNSUPPORTED;       // the matrix-core prefill kernel alone writes tiles
  if (out && decode_fast_ok(desc, false)) {
    DecodeArgs a{};
    a.q = (const bf16_t*)q;
    a.kc = (const bf16_t*)k;
    a.ks = ks;
    a.vc = (const bf16_t*)v;
    a.vs = ks;
    a.row_out = (half_t*)scores_out;
    return run_decode_fast(desc, false, a, out, workspace, st);
  }
  if (desc->dtype == LISA_F32) {
    rc = launch_std_scores<float, float>(desc, q, k, ks, scores_out, exact, st);
    if (rc == LISA_OK && out) rc = launch_softmax_v<float>(desc, exact, v, ks, out, st);
  } else {
    rc = launch_std_scores<bf16_t, half_t>(desc, q, k, ks, scores_out, exact, st);
    if (rc == LISA_OK && out) rc = launch_softmax_v<bf16_t>(desc, exact, v, ks, out, st);
  }
  if (rc == LISA_OK) g_path = "generic";
  return rc;
}

}  // extern "C"
