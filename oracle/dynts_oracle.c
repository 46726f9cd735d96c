/*
 * DynTS decode hot path -- float64 CPU oracle.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, deliberately unblocked C written from the paper's definitions.
 * It shares no code, header, table or helper with the HIP library; only the
 * tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * One call works on ONE layer.  State of a layer (row-major, C order):
 *   K, V     double [Nb][Hkv][cap][d]   (bf16 inputs are held exactly)
 *   S        double [Nb][Hkv][cap]      importance score per cached slot
 *   pos      int32  [Nb][Hkv][cap]      original token position of the slot
 *   seq_len  int32  [Nb]                slots in use (same for all KV heads)
 *   n_prompt int32  [Nb]                question-window length M of sequence b
 *   next_pos int32  [Nb]                position the next appended token gets
 * Slots [0, M) are the question window, the last `window` slots the local
 * window, the slots between them the selection window (Sec. 4.2).
 *
 * Every function returns 0, or a negative code: -1 bad argument, -2 the cache
 * is full, -3 a NaN score reached the selection.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int dynts_oracle_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void dynts_oracle_set_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

/*
 * Append the current token's key/value to every KV head's cache (Sec. 4.2,
 * second paragraph: new KV entries and their scores are appended in order).
 * The score starts at 0 when scores are accumulated from attention, or at the
 * supplied s_new [Nb][Hkv] when the score comes from outside (the predictor's
 * output in the paper's own inference mode).
 */
int dynts_oracle_append(int Nb, int Hkv, int d, int cap, const double *k_new,
                        const double *v_new, const double *s_new,
                        const uint8_t *active, double *K, double *V, double *S,
                        int32_t *pos, int32_t *seq_len, int32_t *next_pos) {
  if (Nb <= 0 || Hkv <= 0 || d <= 0 || cap <= 0) return -1;
  for (int b = 0; b < Nb; ++b) {
    if (active && !active[b]) continue;
    int n = seq_len[b];
    if (n >= cap) return -2;
    for (int h = 0; h < Hkv; ++h) {
      size_t unit = (size_t)b * Hkv + h;
      double *Krow = K + (unit * cap + n) * d;
      double *Vrow = V + (unit * cap + n) * d;
      for (int c = 0; c < d; ++c) {
        Krow[c] = k_new[unit * d + c];
        Vrow[c] = v_new[unit * d + c];
      }
      S[unit * cap + n] = s_new ? s_new[unit] : 0.0;
      pos[unit * cap + n] = next_pos[b];
    }
    seq_len[b] = n + 1;
    next_pos[b] += 1;
  }
  return 0;
}

/*
 * Single-query grouped-query attention over the retained slots (Eq. attn-score
 * and Eq. attn-o): e_j = q.k_j * scale, alpha = softmax_j(e), o = sum_j alpha_j v_j,
 * j over all seq_len[b] slots including the token just appended.  Query head
 * hq reads KV head hq / (Hq/Hkv).
 *   q     [Nb][Hq][d]      out  [Nb][Hq][d]
 *   alpha [Nb][Hq][cap]    (nullable) attention weights, slots >= n set to 0
 *   lse   [Nb][Hq]         (nullable) log sum_j exp(e_j)
 * Rows of inactive sequences are left untouched.
 */
int dynts_oracle_attend(int Nb, int Hq, int Hkv, int d, int cap, const double *q,
                        const double *K, const double *V, const int32_t *seq_len,
                        const uint8_t *active, double scale, double *out,
                        double *alpha, double *lse) {
  if (Nb <= 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || cap <= 0 || Hq % Hkv) return -1;
  const int G = Hq / Hkv;
  int bad = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int bh = 0; bh < Nb * Hq; ++bh) {
    int b = bh / Hq, hq = bh % Hq, h = hq / G;
    if (active && !active[b]) continue;
    int n = seq_len[b];
    if (n <= 0 || n > cap) { bad = 1; continue; }
    const double *qv = q + ((size_t)b * Hq + hq) * d;
    const double *Ku = K + ((size_t)b * Hkv + h) * (size_t)cap * d;
    const double *Vu = V + ((size_t)b * Hkv + h) * (size_t)cap * d;
    double *e = (double *)malloc(sizeof(double) * (size_t)n);
    double m = -INFINITY;
    for (int j = 0; j < n; ++j) {
      double acc = 0.0;
      for (int c = 0; c < d; ++c) acc += qv[c] * Ku[(size_t)j * d + c];
      e[j] = acc * scale;
      if (e[j] > m) m = e[j];
    }
    double l = 0.0;
    for (int j = 0; j < n; ++j) {
      e[j] = exp(e[j] - m);
      l += e[j];
    }
    double *o = out + ((size_t)b * Hq + hq) * d;
    for (int c = 0; c < d; ++c) o[c] = 0.0;
    for (int j = 0; j < n; ++j) {
      double a = e[j] / l;
      e[j] = a;
      for (int c = 0; c < d; ++c) o[c] += a * Vu[(size_t)j * d + c];
    }
    if (alpha) {
      double *arow = alpha + ((size_t)b * Hq + hq) * cap;
      for (int j = 0; j < n; ++j) arow[j] = e[j];
      for (int j = n; j < cap; ++j) arow[j] = 0.0;
    }
    if (lse) lse[(size_t)b * Hq + hq] = m + log(l);
    free(e);
  }
  return bad ? -1 : 0;
}

/*
 * Importance score as accumulated attention received (Eq. importance-score;
 * App. B.1: weights are summed over heads and over the query dimension).  In
 * the running form each decode query contributes one row: every thinking slot
 * j >= M of KV head h gains the sum over the head group of alpha[g][j].
 * Question slots keep their +inf score (Sec. 4.2, first paragraph).
 */
int dynts_oracle_update_scores(int Nb, int Hq, int Hkv, int cap, const double *alpha,
                               const int32_t *seq_len, const int32_t *n_prompt,
                               const uint8_t *active, double *S) {
  if (Nb <= 0 || Hq <= 0 || Hkv <= 0 || cap <= 0 || Hq % Hkv) return -1;
  const int G = Hq / Hkv;
  for (int b = 0; b < Nb; ++b) {
    if (active && !active[b]) continue;
    int n = seq_len[b], M = n_prompt[b];
    for (int h = 0; h < Hkv; ++h) {
      double *Su = S + ((size_t)b * Hkv + h) * cap;
      for (int j = M; j < n; ++j) {
        double add = 0.0;
        for (int g = 0; g < G; ++g)
          add += alpha[((size_t)b * Hq + (size_t)h * G + g) * cap + j];
        Su[j] += add;
      }
    }
  }
  return 0;
}

/*
 * Importance score from a block of queries at once (Eq. importance-score with
 * its sum over the K answer tokens written out; App. B.1 extracts the
 * answer-by-thinking sub-matrix of the attention weights of one forward pass
 * and sums it over heads and over the answer dimension).
 *   q_blk [Nb][T][Hq][d]   the T block queries a_1..a_T of every query head
 *   k_blk [Nb][T][Hkv][d]  their own keys, or NULL
 * Query i attends to the seq_len[b] cached slots and, when k_blk is given, to
 * block keys 0..i (causal, as in the forward pass the paper describes); the
 * softmax of Eq. attn-score runs over exactly those.  For every cached slot j
 *   I[b][h][j] += sum_{i<T} sum_{g in group of h} alpha_{(i,g), j}
 * (I [Nb][Hkv][cap], question and thinking slots alike; block tokens themselves
 * receive no score).
 */
int dynts_oracle_score_block(int Nb, int T, int Hq, int Hkv, int d, int cap,
                             const double *q_blk, const double *k_blk, const double *K,
                             const int32_t *seq_len, const uint8_t *active, double scale,
                             double *I) {
  if (Nb <= 0 || T <= 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || cap <= 0 || Hq % Hkv) return -1;
  const int G = Hq / Hkv;
  int bad = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int u = 0; u < Nb * Hkv; ++u) {
    int b = u / Hkv, h = u % Hkv;
    if (active && !active[b]) continue;
    int n = seq_len[b];
    if (n < 0 || n > cap) { bad = 1; continue; }
    const double *Ku = K + (size_t)u * cap * d;
    double *Iu = I + (size_t)u * cap;
    double *e = (double *)malloc(sizeof(double) * (size_t)(n + T));
    for (int i = 0; i < T; ++i) {
      int vis = k_blk ? i + 1 : 0; /* block keys this query sees */
      for (int g = 0; g < G; ++g) {
        const double *qv = q_blk + (((size_t)b * T + i) * Hq + (size_t)h * G + g) * d;
        double m = -INFINITY;
        for (int j = 0; j < n + vis; ++j) {
          const double *kv = j < n ? Ku + (size_t)j * d
                                   : k_blk + (((size_t)b * T + (j - n)) * Hkv + h) * d;
          double acc = 0.0;
          for (int c = 0; c < d; ++c) acc += qv[c] * kv[c];
          e[j] = acc * scale;
          if (e[j] > m) m = e[j];
        }
        double l = 0.0;
        for (int j = 0; j < n + vis; ++j) {
          e[j] = exp(e[j] - m);
          l += e[j];
        }
        for (int j = 0; j < n; ++j) Iu[j] += e[j] / l;
      }
    }
    free(e);
  }
  return bad ? -1 : 0;
}

/*
 * Importance Predictor (Sec. 4.1; App. A "Predictor Overhead"; App. C gives the sizes
 * 3584->7168->1792->1 and 4096->8192->2048->1): a three-layer MLP d -> m1 -> m2 -> 1 on the final
 * hidden state of the current token, one score per token.
 *   h  [Nb][d]     W1 [m1][d], b1 [m1]     W2 [m2][m1], b2 [m2]     w3 [m2], b3 [1]   (biases nullable)
 *   y1 = act(W1 h + b1),  y2 = act(W2 y1 + b2),  s = w3 . y2 + b3
 * act: 0 none (the paper calls the MLP "linear" and names no activation), 1 ReLU, 2 SiLU.
 * Nothing is rounded between the layers.
 */
static double oracle_act(double x, int act) {
  if (act == 1) return x > 0.0 ? x : 0.0;
  if (act == 2) return x / (1.0 + exp(-x));
  return x;
}

int dynts_oracle_predictor(int Nb, int d, int m1, int m2, const double *h, const double *W1,
                           const double *b1, const double *W2, const double *b2, const double *w3,
                           const double *b3, int act, double *s) {
  if (Nb <= 0 || d <= 0 || m1 <= 0 || m2 <= 0 || act < 0 || act > 2) return -1;
#pragma omp parallel for schedule(static)
  for (int b = 0; b < Nb; ++b) {
    double *y1 = (double *)malloc(sizeof(double) * (size_t)m1);
    double *y2 = (double *)malloc(sizeof(double) * (size_t)m2);
    for (int o = 0; o < m1; ++o) {
      double acc = b1 ? b1[o] : 0.0;
      for (int k = 0; k < d; ++k) acc += W1[(size_t)o * d + k] * h[(size_t)b * d + k];
      y1[o] = oracle_act(acc, act);
    }
    for (int o = 0; o < m2; ++o) {
      double acc = b2 ? b2[o] : 0.0;
      for (int k = 0; k < m1; ++k) acc += W2[(size_t)o * m1 + k] * y1[k];
      y2[o] = oracle_act(acc, act);
    }
    double acc = b3 ? b3[0] : 0.0;
    for (int k = 0; k < m2; ++k) acc += w3[k] * y2[k];
    s[b] = acc;
    free(y1);
    free(y2);
  }
  return 0;
}

/* ---- selection ---------------------------------------------------------- */

typedef struct {
  double s;
  int32_t p;
  int32_t slot;
} cand_t;

/* higher score first; equal scores (IEEE ==, so -0 equals +0): lower position first */
static int cand_before(const void *a, const void *b) {
  const cand_t *x = (const cand_t *)a, *y = (const cand_t *)b;
  if (x->s > y->s) return -1;
  if (x->s < y->s) return 1;
  if (x->p < y->p) return -1;
  if (x->p > y->p) return 1;
  return 0;
}

static int int_ascending(const void *a, const void *b) {
  int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
  return (x > y) - (x < y);
}

/*
 * KV-cache selection (Sec. 4.2, third paragraph; Fig. overview, right): for
 * each triggered sequence and each KV head, keep every question slot [0, M),
 * every local-window slot [n-window, n), and of the selection window
 * [M, n-window) the k_keep slots that come first in a full sort by
 * (score descending, position ascending).  keep_idx[b][h][0..new_len) lists the
 * retained slots in ascending order.  When the selection window holds k_keep
 * slots or fewer nothing is evicted (new_len = n).  Rows of sequences that are
 * not triggered are not written; their new_len is set to seq_len.
 */
int dynts_oracle_select(int Nb, int Hkv, int cap, const double *S, const int32_t *pos,
                        const int32_t *seq_len, const int32_t *n_prompt,
                        const uint8_t *trigger, int window, int k_keep,
                        int keep_stride, int32_t *keep_idx, int32_t *new_len) {
  if (Nb <= 0 || Hkv <= 0 || cap <= 0 || window < 0 || k_keep < 0) return -1;
  for (int b = 0; b < Nb; ++b) {
    int n = seq_len[b], M = n_prompt[b];
    new_len[b] = n;
    if (trigger && !trigger[b]) continue;
    int lo = M, hi = n - window;
    if (hi < lo) hi = lo;
    int nc = hi - lo;
    int kk = nc <= k_keep ? nc : k_keep;
    int out_len = M + kk + (n - hi);
    if (out_len > keep_stride) return -1;
    new_len[b] = out_len;
    for (int h = 0; h < Hkv; ++h) {
      const double *Su = S + ((size_t)b * Hkv + h) * cap;
      const int32_t *pu = pos + ((size_t)b * Hkv + h) * cap;
      int32_t *ku = keep_idx + ((size_t)b * Hkv + h) * keep_stride;
      cand_t *cv = (cand_t *)malloc(sizeof(cand_t) * (size_t)(nc > 0 ? nc : 1));
      for (int j = 0; j < nc; ++j) {
        if (isnan(Su[lo + j])) { free(cv); return -3; }
        cv[j].s = Su[lo + j];
        cv[j].p = pu[lo + j];
        cv[j].slot = lo + j;
      }
      qsort(cv, (size_t)nc, sizeof(cand_t), cand_before);
      int w = 0;
      for (int j = 0; j < M; ++j) ku[w++] = j;
      for (int j = 0; j < kk; ++j) ku[w++] = cv[j].slot;
      qsort(ku + M, (size_t)kk, sizeof(int32_t), int_ascending);
      for (int j = hi; j < n; ++j) ku[w++] = j;
      free(cv);
    }
  }
  return 0;
}

/*
 * Eviction (Sec. 4.2: the remainder is evicted): gather rows keep_idx[0..new_len)
 * of K, V, S and pos to the front, in order, and shorten the sequence.
 */
int dynts_oracle_compact(int Nb, int Hkv, int d, int cap, const uint8_t *trigger,
                         const int32_t *keep_idx, int keep_stride,
                         const int32_t *new_len, double *K, double *V, double *S,
                         int32_t *pos, int32_t *seq_len) {
  if (Nb <= 0 || Hkv <= 0 || d <= 0 || cap <= 0) return -1;
  double *tK = (double *)malloc(sizeof(double) * (size_t)cap * d);
  double *tV = (double *)malloc(sizeof(double) * (size_t)cap * d);
  double *tS = (double *)malloc(sizeof(double) * (size_t)cap);
  int32_t *tp = (int32_t *)malloc(sizeof(int32_t) * (size_t)cap);
  int rc = 0;
  for (int b = 0; b < Nb && !rc; ++b) {
    if (trigger && !trigger[b]) continue;
    int n = seq_len[b], m = new_len[b];
    if (m < 0 || m > n || m > keep_stride) { rc = -1; break; }
    for (int h = 0; h < Hkv; ++h) {
      size_t unit = (size_t)b * Hkv + h;
      const int32_t *ku = keep_idx + unit * keep_stride;
      double *Ku = K + unit * cap * d, *Vu = V + unit * cap * d;
      double *Su = S + unit * cap;
      int32_t *pu = pos + unit * cap;
      for (int i = 0; i < m; ++i) {
        int src = ku[i];
        if (src < 0 || src >= n || (i > 0 && src <= ku[i - 1])) { rc = -1; break; }
        memcpy(tK + (size_t)i * d, Ku + (size_t)src * d, sizeof(double) * d);
        memcpy(tV + (size_t)i * d, Vu + (size_t)src * d, sizeof(double) * d);
        tS[i] = Su[src];
        tp[i] = pu[src];
      }
      if (rc) break;
      memcpy(Ku, tK, sizeof(double) * (size_t)m * d);
      memcpy(Vu, tV, sizeof(double) * (size_t)m * d);
      memcpy(Su, tS, sizeof(double) * (size_t)m);
      memcpy(pu, tp, sizeof(int32_t) * (size_t)m);
    }
    if (!rc) seq_len[b] = m;
  }
  free(tK); free(tV); free(tS); free(tp);
  return rc;
}

/*
 * Effective cache length after decode step i (Sec. 5 "Notions" / App. A,
 * Definition "Effective KV Cache Length"): S_i = M + i - n_i*K with
 * n_i = max(0, floor(((M+i) - B)/K) + 1) eviction events, for total budget B
 * and eviction volume K.
 */
int dynts_oracle_eviction_events(int M, int i, int B, int K) {
  int num = (M + i) - B;
  int fl = num >= 0 ? num / K : -((-num + K - 1) / K);
  int n = fl + 1;
  return n > 0 ? n : 0;
}

int dynts_oracle_effective_length(int M, int i, int B, int K) {
  return M + i - dynts_oracle_eviction_events(M, i, B, K) * K;
}

/*
 * Cost model of Sec. 5 / App. A: predictor MLP d -> m1 -> m2 -> m3 costs
 * 2(d*m1 + m1*m2 + m2*m3) FLOPs per step; attention costs 4*L*d*S per step;
 * the break-even eviction volume is (6d^2+d)/(n*4*L*d).
 */
double dynts_oracle_mlp_flops(double d, double m1, double m2, double m3) {
  return 2.0 * (d * m1 + m1 * m2 + m2 * m3);
}

double dynts_oracle_attn_flops(double L, double d, double S) { return 4.0 * L * d * S; }

double dynts_oracle_break_even_volume(double d, double L, double n_events) {
  return dynts_oracle_mlp_flops(d, 2.0 * d, d / 2.0, 1.0) / (n_events * 4.0 * L * d);
}
