/*
 * AdaSD reference oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 * See adasd_oracle.h for scope, units and the rule that nothing here is ever
 * shared with, or called from, the GPU library.
 *
 * Style: float64 everywhere, loops in index order, no blocking, no fusion, no
 * SIMD.  Each step follows the paper's definition so it can be checked by eye.
 */
#include "adasd_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define LN2 0.693147180559945309417232121458176568
#define TWO_PI 6.283185307179586476925286766559005768

/* ------------------------------------------------------------------------- */
/* Philox4x32-10 (Salmon et al., SC'11): ten rounds of two 32x32->64 multiplies
 * with a Weyl-sequence key schedule.                                          */
/* ------------------------------------------------------------------------- */
void adasd_oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2],
                                uint32_t out[4]) {
  const uint64_t mul_a = 0xD2511F53u, mul_b = 0xCD9E8D57u;
  const uint32_t weyl_a = 0x9E3779B9u, weyl_b = 0xBB67AE85u;
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int r = 0; r < 10; ++r) {
    if (r > 0) { k0 += weyl_a; k1 += weyl_b; }
    uint64_t pa = mul_a * (uint64_t)c0;
    uint64_t pb = mul_b * (uint64_t)c2;
    uint32_t n0 = (uint32_t)(pb >> 32) ^ c1 ^ k0;
    uint32_t n1 = (uint32_t)pb;
    uint32_t n2 = (uint32_t)(pa >> 32) ^ c3 ^ k1;
    uint32_t n3 = (uint32_t)pa;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

double adasd_oracle_uniform24(uint32_t x) {
  return ((double)(x >> 8) + 0.5) / 16777216.0;
}
double adasd_oracle_uniform32(uint32_t x) {
  return ((double)x + 0.5) / 4294967296.0;
}

void adasd_oracle_accept_words(uint64_t seed, uint32_t seq, uint32_t round,
                               uint32_t pos, uint32_t *w_base, uint32_t *w_relaxed) {
  uint32_t ctr[4] = {0u, pos, round, seq};
  uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  uint32_t out[4];
  adasd_oracle_philox4x32_10(ctr, key, out);
  *w_base = out[0];
  *w_relaxed = out[1];
}

uint32_t adasd_oracle_gumbel_word(uint64_t seed, uint32_t seq, uint32_t round,
                                  uint32_t pos, uint32_t v) {
  uint32_t ctr[4] = {v >> 2, pos | (1u << 16), round, seq};
  uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  uint32_t out[4];
  adasd_oracle_philox4x32_10(ctr, key, out);
  return out[v & 3u];
}

/* ------------------------------------------------------------------------- */
/* logits: exact conversion to double                                          */
/* ------------------------------------------------------------------------- */
static double logit_at(const void *base, int dtype, int64_t i) {
  if (dtype == ADASD_ORACLE_F32) return (double)((const float *)base)[i];
  uint32_t w = (uint32_t)((const uint16_t *)base)[i] << 16; /* bf16 = top half of an f32 */
  float f;
  memcpy(&f, &w, sizeof f);
  return (double)f;
}
static const void *row_ptr(const void *base, int dtype, int64_t elem_offset) {
  size_t es = dtype == ADASD_ORACLE_F32 ? 4u : 2u;
  return (const char *)base + (size_t)elem_offset * es;
}

/* log-softmax of a row into lp[0..V): lp_v = z_v - lse.  Returns 1 if the row is
 * non-finite (a NaN or +inf logit, or no finite logit at all).                  */
static int row_log_softmax(const void *row, int dtype, int V, double *lp, double *lse_out) {
  double M = -INFINITY;
  int bad = 0;
  for (int v = 0; v < V; ++v) {
    double z = logit_at(row, dtype, v);
    if (isnan(z) || z == INFINITY) bad = 1;
    if (z > M) M = z;
  }
  if (bad || M == -INFINITY) {
    if (lse_out) *lse_out = NAN;
    return 1;
  }
  double S = 0.0;
  for (int v = 0; v < V; ++v) S += exp(logit_at(row, dtype, v) - M);
  double lse = M + log(S);
  for (int v = 0; v < V; ++v) lp[v] = logit_at(row, dtype, v) - lse;
  if (lse_out) *lse_out = lse;
  return 0;
}

/* H = -sum p ln p, with 0 ln 0 := 0 (Appendix A). */
static double entropy_from_logp(const double *lp, int V) {
  double H = 0.0;
  for (int v = 0; v < V; ++v) {
    double p = exp(lp[v]);
    if (p > 0.0) H -= p * lp[v];
  }
  return H;
}

int adasd_oracle_row_stats(const void *row, int dtype, int V, double *lse, double *H) {
  double *lp = (double *)malloc(sizeof(double) * (size_t)V);
  int bad = row_log_softmax(row, dtype, V, lp, lse);
  *H = bad ? NAN : entropy_from_logp(lp, V);
  free(lp);
  return bad;
}

/* D_JS = 1/2 KL(p||m) + 1/2 KL(q||m), m = (p+q)/2  (Section 2.2, first line). */
static double jsd_from_logp(const double *lp, const double *lq, int V) {
  double D = 0.0;
  for (int v = 0; v < V; ++v) {
    double p = exp(lp[v]), q = exp(lq[v]);
    double m = 0.5 * (p + q);
    if (p > 0.0) D += 0.5 * p * (lp[v] - log(m));
    if (q > 0.0) D += 0.5 * q * (lq[v] - log(m));
  }
  if (D < 0.0) D = 0.0;
  if (D > LN2) D = LN2;
  return D;
}

int adasd_oracle_jsd(const void *prow, const void *qrow, int dtype, int V, double *D) {
  double *lp = (double *)malloc(sizeof(double) * (size_t)V);
  double *lq = (double *)malloc(sizeof(double) * (size_t)V);
  int bad = row_log_softmax(prow, dtype, V, lp, NULL) | row_log_softmax(qrow, dtype, V, lq, NULL);
  *D = bad ? NAN : jsd_from_logp(lp, lq, V);
  free(lp);
  free(lq);
  return bad;
}

/* D_JS = H(m) - (H(p)+H(q))/2  (Section 2.2, second line); not clamped. */
int adasd_oracle_jsd_entropy_form(const void *prow, const void *qrow, int dtype, int V,
                                  double *D) {
  double *lp = (double *)malloc(sizeof(double) * (size_t)V);
  double *lq = (double *)malloc(sizeof(double) * (size_t)V);
  int bad = row_log_softmax(prow, dtype, V, lp, NULL) | row_log_softmax(qrow, dtype, V, lq, NULL);
  if (bad) {
    *D = NAN;
  } else {
    double Hm = 0.0;
    for (int v = 0; v < V; ++v) {
      double m = 0.5 * (exp(lp[v]) + exp(lq[v]));
      if (m > 0.0) Hm -= m * log(m);
    }
    *D = Hm - 0.5 * (entropy_from_logp(lp, V) + entropy_from_logp(lq, V));
  }
  free(lp);
  free(lq);
  return bad;
}

/* ------------------------------------------------------------------------- */
/* KDE and the Bayesian acceptance posterior (Section 4.4)                     */
/* ------------------------------------------------------------------------- */
static double sample_variance(const float *s, int n) {
  double mean = 0.0;
  for (int j = 0; j < n; ++j) mean += (double)s[j];
  mean /= (double)n;
  double ss = 0.0;
  for (int j = 0; j < n; ++j) {
    double e = (double)s[j] - mean;
    ss += e * e;
  }
  return ss / (double)(n - 1);
}

static double bandwidth_factor(int n, int bw_rule) {
  if (bw_rule == 1) return pow((double)n, -0.2);       /* Scott            */
  return pow(4.0 / (3.0 * (double)n), 0.2);            /* Silverman's reference rule */
}

/* ln of  (1/(n h sqrt(2 pi))) * sum_j exp(-(d - s_j)^2 / (2 h^2)) */
double adasd_oracle_kde_logpdf(double d, const float *s, int n, int bw_rule) {
  if (n < 2) return NAN;
  double var = sample_variance(s, n);
  if (!(var > 0.0)) return NAN;
  double h = bandwidth_factor(n, bw_rule) * sqrt(var);
  double tmax = -INFINITY;
  for (int j = 0; j < n; ++j) {
    double e = d - (double)s[j];
    double t = -(e * e) / (2.0 * h * h);
    if (t > tmax) tmax = t;
  }
  double acc = 0.0;
  for (int j = 0; j < n; ++j) {
    double e = d - (double)s[j];
    acc += exp(-(e * e) / (2.0 * h * h) - tmax);
  }
  return tmax + log(acc) - log((double)n * h * sqrt(TWO_PI));
}

/* P(A|d) = p(d|A)P(A) / (p(d|A)P(A) + p(d|R)P(R)),  P(A) = |L_A| / (|L_A|+|L_R|). */
double adasd_oracle_posterior(double d, const float *LA, int nA, const float *LR, int nR,
                              int min_n, int bw_rule) {
  if (min_n < 2) min_n = 2;
  if (nA < min_n || nR < min_n) return 0.0;
  double la = adasd_oracle_kde_logpdf(d, LA, nA, bw_rule);
  double lr = adasd_oracle_kde_logpdf(d, LR, nR, bw_rule);
  if (isnan(la) || isnan(lr)) return 0.0;
  double joint_a = la + log((double)nA / (double)(nA + nR));
  double joint_r = lr + log((double)nR / (double)(nA + nR));
  /* joint_a, joint_r are finite, so this is the Bayes ratio evaluated without 0/0 */
  return 1.0 / (1.0 + exp(joint_r - joint_a));
}

/* ------------------------------------------------------------------------- */
/* Draft side: entropy stop rule (Section 4.3; generation loop of Algorithm 1) */
/* ------------------------------------------------------------------------- */
void adasd_oracle_draft_entropy(const void *logits, int dtype, int B, int V,
                                int64_t row_stride, const float *T_G,
                                const uint8_t *active, int step, int k_max,
                                double *H_out, uint8_t *stop_out) {
  for (int b = 0; b < B; ++b) {
    if (active && !active[b]) {
      H_out[b] = 0.0;
      if (stop_out) stop_out[b] = 0;
      continue;
    }
    double lse, H;
    adasd_oracle_row_stats(row_ptr(logits, dtype, (int64_t)b * row_stride), dtype, V, &lse, &H);
    H_out[b] = H;
    if (stop_out) {
      int over = T_G ? (H > (double)T_G[b]) : 0;   /* strict: break when H(q_i) > T_G */
      stop_out[b] = (uint8_t)(over || (step + 1 >= k_max));
    }
  }
}

/* ------------------------------------------------------------------------- */
/* Verification of one sequence (verification loop of Algorithm 1)             */
/* ------------------------------------------------------------------------- */
static void verify_one(const adasd_oracle_verify_args *a, int b, double *lp, double *lq) {
  const int V = a->V, K = a->k_max;
  const int k = a->draft_len ? a->draft_len[b] : K;
  const uint32_t seq = a->seq_id ? a->seq_id[b] : (uint32_t)b;
  const uint32_t rnd = a->round ? a->round[b] : a->round0;
  const float *LA = a->LA ? a->LA + (size_t)b * (size_t)a->cap : NULL;
  const float *LR = a->LR ? a->LR + (size_t)b * (size_t)a->cap : NULL;
  int nA = a->nA ? a->nA[b] : 0;
  const int nR = a->nR ? a->nR[b] : 0;
  uint32_t st = 0;
  /* Algorithm 1 appends to L_D^A inside the verification loop: work on a copy of the list that grows
     as the loop goes (the state itself is still only changed by the update step, which repeats the
     same appends).  A position is only reached in the paper's loop if every earlier one was accepted,
     so "the distances of all earlier positions" is what it sees; positions after the first
     rejection are reported under the same rule. */
  float *work = NULL;
  if (a->list_update == 1 && LA) {
    work = (float *)malloc(sizeof(float) * (size_t)a->cap);
    memcpy(work, LA, sizeof(float) * (size_t)a->cap);
    LA = work;
  }

  for (int i = 0; i < K; ++i) {
    size_t o = (size_t)b * (size_t)K + (size_t)i;
    a->H_p[o] = a->H_q[o] = a->d_js[o] = a->p_accept[o] = 0.0;
    a->accept_mask[o] = 0;
    if (a->base_margin) a->base_margin[o] = 0.0;
    if (a->relaxed_margin) a->relaxed_margin[o] = 0.0;
  }

  int first_reject = k;
  for (int i = 0; i < k; ++i) {
    size_t o = (size_t)b * (size_t)K + (size_t)i;
    const void *prow = row_ptr(a->target_logits, a->dtype,
                               (int64_t)b * a->t_seq_stride + (int64_t)i * a->t_pos_stride);
    const void *qrow = row_ptr(a->draft_logits, a->dtype,
                               (int64_t)b * a->d_seq_stride + (int64_t)i * a->d_pos_stride);
    int bad = row_log_softmax(prow, a->dtype, V, lp, NULL) |
              row_log_softmax(qrow, a->dtype, V, lq, NULL);
    int accept = 0;
    if (bad) {
      st |= ADASD_ORACLE_ST_NONFINITE;
      a->H_p[o] = a->H_q[o] = a->d_js[o] = a->p_accept[o] = NAN;
    } else {
      a->H_p[o] = entropy_from_logp(lp, V);
      a->H_q[o] = entropy_from_logp(lq, V);
      double dhat = sqrt(jsd_from_logp(lp, lq, V) / LN2);
      a->d_js[o] = dhat;

      uint32_t w1, w2;
      adasd_oracle_accept_words(a->seed, seq, rnd, (uint32_t)i, &w1, &w2);
      double u1 = adasd_oracle_uniform24(w1), u2 = adasd_oracle_uniform24(w2);

      int base = 0;
      int32_t x = a->draft_tokens[o];
      if (x < 0 || x >= V) {
        st |= ADASD_ORACLE_ST_BAD_TOKEN;
        if (a->base_margin) a->base_margin[o] = INFINITY;
      } else if (a->base_test == 1) {
        /* Algorithm 1: y_i ~ p_i, accepted iff x_i = y_i, an event of probability p_i(x_i) */
        base = log(u1) < lp[x];
        if (a->base_margin) a->base_margin[o] = log(u1) - lp[x];
      } else {
        /* speculative-sampling test: accept with probability min(1, p(x)/q(x)) */
        double log_ratio = lp[x] - lq[x];
        if (log_ratio > 0.0) log_ratio = 0.0;
        base = log(u1) < log_ratio; /* false when log_ratio is NaN (both probabilities zero) */
        if (a->base_margin) a->base_margin[o] = log(u1) - log_ratio;
      }

      /* Bayesian test on the JS distance */
      double PA = a->relaxed_off ? 0.0
                                 : adasd_oracle_posterior(dhat, LA, nA, LR, nR, a->kde_min_n,
                                                          a->bw_rule);
      a->p_accept[o] = PA;
      int relaxed;
      if (a->reject_rule == 1) {
        relaxed = PA >= 0.5;
        if (a->relaxed_margin) a->relaxed_margin[o] = 0.5 - PA;
      } else {
        relaxed = u2 < PA;
        if (a->relaxed_margin) a->relaxed_margin[o] = u2 - PA;
      }
      /* a candidate is rejected only if BOTH tests reject it */
      accept = base || relaxed;
      a->accept_mask[o] = (uint8_t)(base | (relaxed << 1));
      /* in-loop append of the accepted distance (open-interval filter, capacity as in the update step) */
      if (work && dhat > a->d_eps && dhat < 1.0 - a->d_eps && nA < a->cap) work[nA++] = (float)dhat;
    }
    if (!accept && first_reject == k) first_reject = i;
  }
  a->n_accept[b] = first_reject;
  free(work);

  /* token appended after the accepted prefix */
  const int r = first_reject;
  const void *prow = row_ptr(a->target_logits, a->dtype,
                             (int64_t)b * a->t_seq_stride + (int64_t)r * a->t_pos_stride);
  int token = -1;
  double best = -INFINITY, second = -INFINITY;
  if (row_log_softmax(prow, a->dtype, V, lp, NULL)) {
    st |= ADASD_ORACLE_ST_NONFINITE;
  } else {
    int residual = 0;
    int excluded = -1;
    if (r < k && a->base_test == 1) {
      /* y_r given y_r != x_r: the target distribution with the drafted token excluded */
      int32_t x = a->draft_tokens[(size_t)b * (size_t)K + (size_t)r];
      if (x >= 0 && x < V) {
        double mass = 0.0;
        for (int v = 0; v < V; ++v)
          if (v != x) mass += exp(lp[v]);
        if (mass > 0.0) excluded = x;
        else st |= ADASD_ORACLE_ST_ZERO_MASS; /* all mass on x_r: fall back to the target distribution */
      }
    } else if (r < k) {
      const void *qrow = row_ptr(a->draft_logits, a->dtype,
                                 (int64_t)b * a->d_seq_stride + (int64_t)r * a->d_pos_stride);
      if (row_log_softmax(qrow, a->dtype, V, lq, NULL)) {
        st |= ADASD_ORACLE_ST_NONFINITE;
        goto done;
      }
      /* adjusted distribution: proportional to max(0, p - q) */
      double mass = 0.0;
      for (int v = 0; v < V; ++v) {
        double w = exp(lp[v]) - exp(lq[v]);
        if (w > 0.0) mass += w;
      }
      if (mass > 0.0) residual = 1;
      else st |= ADASD_ORACLE_ST_ZERO_MASS; /* fall back to the target distribution */
    }
    /* Gumbel-max: argmax_v ln w_v - ln(-ln u_v); first index wins ties */
    for (int v = 0; v < V; ++v) {
      double w = residual ? exp(lp[v]) - exp(lq[v]) : exp(lp[v]);
      if (v == excluded || !(w > 0.0)) continue;
      double u = adasd_oracle_uniform32(
          adasd_oracle_gumbel_word(a->seed, seq, rnd, (uint32_t)r, (uint32_t)v));
      double key = log(w) - log(-log(u));
      if (key > best) {
        second = best;
        best = key;
        token = v;
      } else if (key > second) {
        second = key;
      }
    }
  }
done:
  a->next_token[b] = token;
  if (a->top2_gap) a->top2_gap[b] = best - second;
  a->status[b] = st;
}

int adasd_oracle_verify(const adasd_oracle_verify_args *a) {
  if (!a || a->B < 0 || a->k_max < 0 || a->V < 1) return -1;
  if (a->draft_len)
    for (int b = 0; b < a->B; ++b)
      if (a->draft_len[b] < 0 || a->draft_len[b] > a->k_max) return -1;
#pragma omp parallel
  {
    double *lp = (double *)malloc(sizeof(double) * (size_t)a->V);
    double *lq = (double *)malloc(sizeof(double) * (size_t)a->V);
#pragma omp for schedule(dynamic, 1)
    for (int b = 0; b < a->B; ++b) verify_one(a, b, lp, lq);
    free(lp);
    free(lq);
  }
  return 0;
}

/* ------------------------------------------------------------------------- */
/* Drafting loop of Algorithm 1: x_i ~ q_i                                     */
/* ------------------------------------------------------------------------- */
void adasd_oracle_draft_sample(const void *logits, int dtype, int B, int V, int64_t row_stride,
                               const uint8_t *active, int step, uint64_t seed,
                               const uint32_t *seq_id, const uint32_t *round, uint32_t round0,
                               int32_t *token_out, double *top2_gap) {
#pragma omp parallel
  {
    double *lq = (double *)malloc(sizeof(double) * (size_t)V);
#pragma omp for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
      token_out[b] = -1;
      if (top2_gap) top2_gap[b] = 0.0;
      if (active && !active[b]) continue;
      if (row_log_softmax(row_ptr(logits, dtype, (int64_t)b * row_stride), dtype, V, lq, NULL)) continue;
      const uint32_t seq = seq_id ? seq_id[b] : (uint32_t)b;
      const uint32_t rnd = round ? round[b] : round0;
      const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
      double best = -INFINITY, second = -INFINITY;
      int token = -1;
      for (int v = 0; v < V; ++v) {
        if (!(exp(lq[v]) > 0.0)) continue;          /* no mass: never drawn */
        const uint32_t ctr[4] = {(uint32_t)v >> 2, (uint32_t)step | (2u << 16), rnd, seq};
        uint32_t out[4];
        adasd_oracle_philox4x32_10(ctr, key, out);
        const double u = adasd_oracle_uniform32(out[v & 3]);
        const double k = lq[v] - log(-log(u));
        if (k > best) {
          second = best;
          best = k;
          token = v;
        } else if (k > second) {
          second = k;
        }
      }
      token_out[b] = token;
      if (top2_gap) top2_gap[b] = best - second;
    }
    free(lq);
  }
}

/* ------------------------------------------------------------------------- */
/* Update step of Algorithm 1                                                  */
/* ------------------------------------------------------------------------- */
static void list_append(float *L, int32_t *n, int cap, double d, uint32_t *st) {
  if (*n >= cap) {
    if (st) *st |= ADASD_ORACLE_ST_OVERFLOW;
    return;
  }
  L[*n] = (float)d;
  *n += 1;
}

void adasd_oracle_update(int B, int k_max, int cap, const int32_t *n_accept,
                         const int32_t *draft_len, const double *H_q, const double *d_js,
                         double d_eps, float *LA, float *LR, int32_t *nA, int32_t *nR,
                         double *ent_sum, int32_t *ent_cnt, float *T_G, uint32_t *status) {
  for (int b = 0; b < B; ++b) {
    const int k = draft_len ? draft_len[b] : k_max;
    const int r = n_accept[b];
    uint32_t *st = status ? status + b : NULL;
    float *la = LA + (size_t)b * (size_t)cap, *lr = LR + (size_t)b * (size_t)cap;
    /* accepted positions: record the JS distance unless it sits on the boundary */
    for (int i = 0; i < r && i < k; ++i) {
      double d = d_js[(size_t)b * (size_t)k_max + (size_t)i];
      if (d > d_eps && d < 1.0 - d_eps) list_append(la, &nA[b], cap, d, st);
    }
    /* the rejected position: record its draft entropy and its JS distance */
    if (r < k) {
      double H = H_q[(size_t)b * (size_t)k_max + (size_t)r];
      if (isfinite(H)) { /* a row with broken logits has no entropy to record */
        ent_sum[b] += H;
        ent_cnt[b] += 1;
      }
      double d = d_js[(size_t)b * (size_t)k_max + (size_t)r];
      if (d > d_eps && d < 1.0 - d_eps) list_append(lr, &nR[b], cap, d, st);
    }
    /* generation threshold = mean rejected entropy (stays at its initial 0 while empty) */
    T_G[b] = ent_cnt[b] > 0 ? (float)(ent_sum[b] / (double)ent_cnt[b]) : 0.0f;
  }
}

int adasd_oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
