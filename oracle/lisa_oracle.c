/*
 * LiSA attention-layer oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, float64 CPU statement of what the LiSA attention path computes,
 * written from the paper's definitions (Sec. 2.1 Eq. 1-2: standard attention and
 * the pre-softmax score tensor A; Sec. 5.1: attention-heads alignment FFN over the
 * head axis, Eq. 3: low-rank difference A_delta, Eq. 4: Integrate).  It shares no
 * code with the HIP library and is only to be used by tests/, the smoke check and
 * the cpu_baseline leg of the benchmark.
 *
 * Conventions (one sequence per call; the caller loops over the batch):
 *   q_lr  [H  ][Lq][r ]     low-rank queries           (Eq. 3, H W^Q_LR split in heads)
 *   k_lr  [Hkv][Lk][r ]     low-rank keys              (Eq. 3, H W^K_LR split in heads)
 *   v     [Hkv][Lk][dk]     values                     (Eq. 1, H W^V_i)
 *   w1    [Din][F ]         first FFN weight, Din = H (ADD) or 2H (CONCAT)
 *   w2    [F  ][H ]         second FFN weight
 *   rows  [n_rows]          query-row indices i in [0,Lq) to evaluate
 *   prev_rows [n_rows][H][Lk]  A_{n-1}[:, i, :] for exactly those rows
 * Query row i sees keys j < n_vis(i) = i + 1 + (Lk - Lq)  (causal; decode is Lq = 1).
 * Query head h reads KV head h / (H / Hkv).
 * Outputs for invisible keys are written as 0.
 *
 * Everything is double; loops are written in the order of the definitions, with
 * no blocking, fusion or reordering.  Rows are independent, so the optional
 * OpenMP pragma over rows changes nothing in the arithmetic of any row.
 *
 * Pins (tests/test_oracle_pins.py): softmax rows sum to one and vanish above the
 * diagonal; identity FFN + zero correction equals textbook attention from a
 * library softmax/matmul; A_delta equals a brute-force triple loop; r = d_k reduces
 * Eq. 3 to Eq. 2; the h = 3 head permutation of Sec. 5.1; uniform and one-hot score
 * closed forms; GQA equals MHA with repeated K/V; prefill row L-1 equals decode; a
 * hand-evaluated 2-head example.  Variants: SiLU against a library sigmoid, the single-layer
 * FFN against a library matmul, LiSA_plus = A_{n-1} + brute-force A_delta, direct sharing =
 * textbook attention on A_{n-1}.  Projection front end: without rotation it equals a library
 * matrix product; unit-vector inputs give (cos, sin) closed forms that fix the pairing, the
 * sign and the frequency exponent; rotated dot products depend on the position difference only.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

#define LISA_ORACLE_MIX_ADD 0
#define LISA_ORACLE_MIX_CONCAT 1
#define LISA_ORACLE_MIX_PLUS 2  /* Sec. 5.5, LiSA_plus: A_n = A_{n-1} + A_delta, no FFN          */
#define LISA_ORACLE_MIX_SHARE 3 /* Sec. 4, directly sharing (DS): A_n = A_{n-1}                   */
#define LISA_ORACLE_ACT_RELU 0
#define LISA_ORACLE_ACT_SILU 1   /* Sec. 5.7, "DL + SiLU": x * sigmoid(x)                          */
#define LISA_ORACLE_ACT_SINGLE 2 /* Sec. 5.7, "SL": one layer, A_align = W1^T x with W1 [Din][H]  */

static int n_visible(int i, int Lq, int Lk) {
  int n = i + 1 + (Lk - Lq);
  if (n < 0) n = 0;
  if (n > Lk) n = Lk;
  return n;
}

/* Sec. 2.1 Eq. 2, the bracketed term A:  A[h,i,j] = scale * <Q[h,i,:], K[kv(h),j,:]>. */
int lisa_oracle_std_scores_rows(int H, int Hkv, int Lq, int Lk, int dk, double scale,
                                const double* q, const double* k, int n_rows,
                                const int* rows, double* scores_rows) {
  if (H <= 0 || Hkv <= 0 || H % Hkv != 0 || Lq <= 0 || Lk < Lq || dk <= 0) return -1;
  const int group = H / Hkv;
#pragma omp parallel for schedule(dynamic, 1)
  for (int n = 0; n < n_rows; ++n) {
    const int i = rows[n];
    const int nv = n_visible(i, Lq, Lk);
    for (int h = 0; h < H; ++h) {
      const int kv = h / group;
      double* dst = scores_rows + ((size_t)n * H + h) * Lk;
      for (int j = 0; j < Lk; ++j) {
        if (j >= nv) { dst[j] = 0.0; continue; }
        double acc = 0.0;
        for (int t = 0; t < dk; ++t)
          acc += q[((size_t)h * Lq + i) * dk + t] * k[((size_t)kv * Lk + j) * dk + t];
        dst[j] = scale * acc;
      }
    }
  }
  return 0;
}

/* Sec. 2.1 Eq. 1-2:  P = Softmax(A) over the visible keys of each row, O_h = P_h V_kv(h).
 * probs_rows may be NULL.  out_rows is [n_rows][H][dk]. */
int lisa_oracle_softmax_v_rows(int H, int Hkv, int Lq, int Lk, int dk, const double* v,
                               int n_rows, const int* rows, const double* scores_rows,
                               double* probs_rows, double* out_rows) {
  if (H <= 0 || Hkv <= 0 || H % Hkv != 0 || Lq <= 0 || Lk < Lq || dk <= 0) return -1;
  const int group = H / Hkv;
#pragma omp parallel for schedule(dynamic, 1)
  for (int n = 0; n < n_rows; ++n) {
    const int i = rows[n];
    const int nv = n_visible(i, Lq, Lk);
    double* p = (double*)malloc(sizeof(double) * (size_t)(Lk > 0 ? Lk : 1));
    for (int h = 0; h < H; ++h) {
      const int kv = h / group;
      const double* a = scores_rows + ((size_t)n * H + h) * Lk;
      double m = -INFINITY;
      for (int j = 0; j < nv; ++j)
        if (a[j] > m) m = a[j];
      double z = 0.0;
      for (int j = 0; j < nv; ++j) {
        p[j] = exp(a[j] - m);
        z += p[j];
      }
      for (int j = 0; j < Lk; ++j) p[j] = (j < nv) ? p[j] / z : 0.0;
      if (probs_rows) memcpy(probs_rows + ((size_t)n * H + h) * Lk, p, sizeof(double) * Lk);
      double* o = out_rows + ((size_t)n * H + h) * dk;
      for (int c = 0; c < dk; ++c) {
        double acc = 0.0;
        for (int j = 0; j < nv; ++j) acc += p[j] * v[((size_t)kv * Lk + j) * dk + c];
        o[c] = acc;
      }
    }
    free(p);
  }
  return 0;
}

/* Sec. 5.1: for every visible position (i,j)
 *   a_delta[h] = delta_scale * <Q_LR[h,i,:], K_LR[kv(h),j,:]>                    (Eq. 3)
 *   x = A_{n-1}[:,i,j]                      (ADD)    or [A_{n-1}[:,i,j] ; a_delta] (CONCAT)
 *   hid = act(W1^T x),  y = W2^T hid        (two-layer FFN over the head axis; act = ReLU or
 *                                            SiLU)   or   y = W1^T x  (SINGLE, W1 [Din][H])
 *   A_n[:,i,j] = y + a_delta                (ADD, Eq. 4 by addition)  or  y     (CONCAT)
 * and the two variants without an FFN: A_n = A_{n-1} + a_delta (PLUS), A_n = A_{n-1} (SHARE).
 * scores_rows receives A_n for the requested rows ([n_rows][H][Lk]).  */
int lisa_oracle_lisa_scores_rows(int H, int Hkv, int Lq, int Lk, int r, int F, int mix, int act,
                                 double delta_scale, const double* q_lr, const double* k_lr,
                                 const double* w1, const double* w2, int n_rows,
                                 const int* rows, const double* prev_rows,
                                 double* scores_rows) {
  if (H <= 0 || Hkv <= 0 || H % Hkv != 0 || Lq <= 0 || Lk < Lq) return -1;
  if (mix < LISA_ORACLE_MIX_ADD || mix > LISA_ORACLE_MIX_SHARE) return -1;
  if (act < LISA_ORACLE_ACT_RELU || act > LISA_ORACLE_ACT_SINGLE) return -1;
  const int has_ffn = mix == LISA_ORACLE_MIX_ADD || mix == LISA_ORACLE_MIX_CONCAT;
  const int has_delta = mix != LISA_ORACLE_MIX_SHARE;
  const int single = act == LISA_ORACLE_ACT_SINGLE;
  if (has_delta && r <= 0) return -1;
  if (has_ffn && (single ? F != H : F <= 0)) return -1;
  const int group = H / Hkv;
  const int Din = (mix == LISA_ORACLE_MIX_CONCAT) ? 2 * H : H;
#pragma omp parallel for schedule(dynamic, 1)
  for (int n = 0; n < n_rows; ++n) {
    const int i = rows[n];
    const int nv = n_visible(i, Lq, Lk);
    double* ad = (double*)malloc(sizeof(double) * (size_t)H);
    double* x = (double*)malloc(sizeof(double) * (size_t)Din);
    double* hid = (double*)malloc(sizeof(double) * (size_t)(F > 0 ? F : 1));
    for (int j = 0; j < Lk; ++j) {
      if (j >= nv) {
        for (int h = 0; h < H; ++h) scores_rows[((size_t)n * H + h) * Lk + j] = 0.0;
        continue;
      }
      for (int h = 0; h < H; ++h) {
        const int kv = h / group;
        double acc = 0.0;
        if (has_delta)
          for (int t = 0; t < r; ++t)
            acc += q_lr[((size_t)h * Lq + i) * r + t] * k_lr[((size_t)kv * Lk + j) * r + t];
        ad[h] = delta_scale * acc;
      }
      for (int h = 0; h < H; ++h) x[h] = prev_rows[((size_t)n * H + h) * Lk + j];
      if (!has_ffn) {
        for (int h = 0; h < H; ++h) scores_rows[((size_t)n * H + h) * Lk + j] = x[h] + ad[h];
        continue;
      }
      if (mix == LISA_ORACLE_MIX_CONCAT)
        for (int h = 0; h < H; ++h) x[H + h] = ad[h];
      for (int f = 0; f < F; ++f) {
        double acc = 0.0;
        for (int c = 0; c < Din; ++c) acc += x[c] * w1[(size_t)c * F + f];
        if (act == LISA_ORACLE_ACT_RELU)
          hid[f] = acc > 0.0 ? acc : 0.0;
        else if (act == LISA_ORACLE_ACT_SILU)
          hid[f] = acc / (1.0 + exp(-acc));
        else
          hid[f] = acc;
      }
      for (int h = 0; h < H; ++h) {
        double acc = 0.0;
        if (single)
          acc = hid[h];
        else
          for (int f = 0; f < F; ++f) acc += hid[f] * w2[(size_t)f * H + h];
        scores_rows[((size_t)n * H + h) * Lk + j] =
            (mix == LISA_ORACLE_MIX_ADD) ? acc + ad[h] : acc;
      }
    }
    free(ad);
    free(x);
    free(hid);
  }
  return 0;
}

/* The whole LiSA layer for the requested rows: scores (above), then Eq. 1-2. */
int lisa_oracle_lisa_rows(int H, int Hkv, int Lq, int Lk, int dk, int r, int F, int mix, int act,
                          double delta_scale, const double* q_lr, const double* k_lr,
                          const double* v, const double* w1, const double* w2, int n_rows,
                          const int* rows, const double* prev_rows, double* scores_rows,
                          double* probs_rows, double* out_rows) {
  int rc = lisa_oracle_lisa_scores_rows(H, Hkv, Lq, Lk, r, F, mix, act, delta_scale, q_lr, k_lr,
                                        w1, w2, n_rows, rows, prev_rows, scores_rows);
  if (rc) return rc;
  return lisa_oracle_softmax_v_rows(H, Hkv, Lq, Lk, dk, v, n_rows, rows, scores_rows,
                                    probs_rows, out_rows);
}

/* Front end of a LiSA layer for the requested token rows of one sequence:
 *   Q_LR = X W^Q_LR,  K_LR = X W^K_LR   (the two factors of Eq. 3),   V = X W^V   (Eq. 1),
 * each split in heads, followed, when theta > 0, by the rotary position embedding of the
 * LLaMA models of Sec. 5.3 on every Q_LR / K_LR head (r even): with half = r/2 and
 * angle(pos, t) = pos * theta^(-2t/r), the pair (y[t], y[t+half]) becomes
 *   (y[t] cos - y[t+half] sin,  y[t] sin + y[t+half] cos),      pos = pos0 + row index.
 *   x [L][D] hidden states;  w [H*r + Hkv*r + Hkv*dk][D]: one row per output feature, the
 *   rows of W^Q_LR^T first, then W^K_LR^T, then W^V^T.
 *   q_rows [n_rows][H][r],  k_rows [n_rows][Hkv][r],  v_rows [n_rows][Hkv][dk].  */
int lisa_oracle_project_rows(int L, int D, int H, int Hkv, int r, int dk, double theta,
                             int pos0, const double* x, const double* w, int n_rows,
                             const int* rows, double* q_rows, double* k_rows,
                             double* v_rows) {
  if (L <= 0 || D <= 0 || H <= 0 || Hkv <= 0 || r <= 0 || dk <= 0) return -1;
  if (theta > 0.0 && r % 2 != 0) return -1;
  const int nq = H * r, nk = Hkv * r, nv = Hkv * dk;
#pragma omp parallel for schedule(dynamic, 1)
  for (int n = 0; n < n_rows; ++n) {
    const int i = rows[n];
    const double* xi = x + (size_t)i * D;
    double* y = (double*)malloc(sizeof(double) * (size_t)(nq + nk + nv));
    for (int f = 0; f < nq + nk + nv; ++f) {
      double acc = 0.0;
      for (int c = 0; c < D; ++c) acc += xi[c] * w[(size_t)f * D + c];
      y[f] = acc;
    }
    if (theta > 0.0) {
      const int half = r / 2;
      const double pos = (double)(pos0 + i);
      for (int head = 0; head < H + Hkv; ++head) {
        double* yh = y + (size_t)head * r;
        for (int t = 0; t < half; ++t) {
          const double ang = pos * pow(theta, -2.0 * t / r);
          const double c = cos(ang), s = sin(ang);
          const double a = yh[t], b = yh[t + half];
          yh[t] = a * c - b * s;
          yh[t + half] = a * s + b * c;
        }
      }
    }
    memcpy(q_rows + (size_t)n * nq, y, sizeof(double) * (size_t)nq);
    memcpy(k_rows + (size_t)n * nk, y + nq, sizeof(double) * (size_t)nk);
    memcpy(v_rows + (size_t)n * nv, y + nq + nk, sizeof(double) * (size_t)nv);
    free(y);
  }
  return 0;
}

int lisa_oracle_num_threads(void) {
#ifdef _OPENMP
  extern int omp_get_max_threads(void);
  return omp_get_max_threads();
#else
  return 1;
#endif
}
