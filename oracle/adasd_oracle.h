/*
 * AdaSD reference oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, float64, index-order CPU implementation of the per-round
 * statistics + verification + update step of Adaptive Speculative Decoding
 * (Algorithm 1; Sections 2.1.3, 2.2, 4.3, 4.4; Appendix A of the paper).
 * It exists only so that tests, the smoke check and the benchmark's
 * cpu_baseline leg have something independent to compare the GPU library
 * against.  It shares no code, header, table or constant with the HIP path
 * and must never be linked into or called from it.
 *
 * Every function below is pinned by tests that do not call the oracle to
 * produce their expected values (closed forms, brute force on tiny
 * vocabularies, scipy/numpy library routines, the published Philox
 * known-answer vectors, invariants stated in the paper).
 *
 * Units: entropies in nats; JS divergence D in nats, JS distance reported as
 * dhat = sqrt(D / ln 2) in [0,1] (the base-2 normalisation under which the
 * paper states the [0,1] bound and the "exactly 0 or 1" exclusion).
 */
#ifndef ADASD_ORACLE_H
#define ADASD_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { ADASD_ORACLE_F32 = 0, ADASD_ORACLE_BF16 = 1 };

/* status bits, per sequence */
enum {
  ADASD_ORACLE_ST_BAD_TOKEN = 1u,  /* draft token id outside [0,V)            */
  ADASD_ORACLE_ST_NONFINITE = 2u,  /* NaN/+inf logit or an all -inf row       */
  ADASD_ORACLE_ST_ZERO_MASS = 4u,  /* residual max(0,p-q) had no mass         */
  ADASD_ORACLE_ST_OVERFLOW  = 8u   /* a history list was full; append dropped */
};

/* Philox4x32-10 block function (Salmon, Moraes, Dror, Shaw; SC'11). */
void adasd_oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2],
                                uint32_t out[4]);

/* Uniforms in the open interval (0,1). */
double adasd_oracle_uniform24(uint32_t x); /* ((x>>8)+0.5) / 2^24 */
double adasd_oracle_uniform32(uint32_t x); /* ( x    +0.5) / 2^32 */

/* The words this build draws for sequence `seq`, decode round `round`:
 *   acceptance uniforms of position i : block (0, i, round, seq), word 0 -> u1 (base test),
 *                                                                 word 1 -> u2 (relaxed test)
 *   Gumbel noise of vocabulary element v at sampled position r :
 *                                       block (v>>2, r | 1<<16, round, seq), word v&3
 * key = (seed low 32 bits, seed high 32 bits).                                  */
void adasd_oracle_accept_words(uint64_t seed, uint32_t seq, uint32_t round,
                               uint32_t pos, uint32_t *w_base, uint32_t *w_relaxed);
uint32_t adasd_oracle_gumbel_word(uint64_t seed, uint32_t seq, uint32_t round,
                                  uint32_t pos, uint32_t v);

/* Softmax normaliser and Shannon entropy of one row of logits (Appendix A).
 * Returns 0, or 1 if the row is non-finite (then *lse = *H = NaN).            */
int adasd_oracle_row_stats(const void *row, int dtype, int V, double *lse, double *H);

/* Jensen-Shannon divergence in nats between softmax(prow) and softmax(qrow)
 * (Section 2.2, first form), clamped to [0, ln 2].  Returns 0, or 1 if either
 * row is non-finite (then *D = NaN).                                           */
int adasd_oracle_jsd(const void *prow, const void *qrow, int dtype, int V, double *D);

/* Second form of Section 2.2: H(m) - (H(p)+H(q))/2, unclamped (used by tests). */
int adasd_oracle_jsd_entropy_form(const void *prow, const void *qrow, int dtype, int V,
                                  double *D);

/* Gaussian kernel density estimate at d from samples s[0..n) with bandwidth
 * h = factor(n) * sample-std(n-1): bw_rule 0 = Silverman's reference rule
 * (4/(3n))^(1/5), 1 = Scott's n^(-1/5).  Returns ln density (-inf never:
 * evaluated with a max-shifted log-sum-exp).  NaN if n<2 or zero variance.      */
double adasd_oracle_kde_logpdf(double d, const float *s, int n, int bw_rule);

/* Bayesian acceptance posterior P(A|d) of Section 4.4 with list-size priors
 * (Algorithm 1).  0 when either list has fewer than min_n samples or zero
 * variance.                                                                    */
double adasd_oracle_posterior(double d, const float *LA, int nA, const float *LR, int nR,
                              int min_n, int bw_rule);

/* Draft-side rule: H(q) for each row and stop = (H > T_G) or (step+1 == k_max). */
void adasd_oracle_draft_entropy(const void *logits, int dtype, int B, int V,
                                int64_t row_stride, const float *T_G,
                                const uint8_t *active, int step, int k_max,
                                double *H_out, uint8_t *stop_out);

/* Generation loop of Algorithm 1, "x_i ~ q_i": one token per active row from softmax(row), by
 * Gumbel-max, argmax_v ln q_v - ln(-ln u_v) with u_v the Philox word of counter
 * (v>>2, step | 2<<16, round, sequence), word v&3 (a stream of its own: stream 1 belongs to the
 * verification step's replacement draws); lowest index on ties.  token_out[b] = -1 for inactive rows
 * and rows with NaN/+inf or without a finite logit.  top2_gap (may be NULL): best minus second key. */
void adasd_oracle_draft_sample(const void *logits, int dtype, int B, int V, int64_t row_stride,
                               const uint8_t *active, int step, uint64_t seed,
                               const uint32_t *seq_id, const uint32_t *round, uint32_t round0,
                               int32_t *token_out, double *top2_gap);

typedef struct {
  /* inputs */
  const void *target_logits;  /* [B, k_max+1, V] */
  const void *draft_logits;   /* [B, k_max,   V] */
  int32_t dtype, B, k_max, V;
  int64_t t_seq_stride, t_pos_stride, d_seq_stride, d_pos_stride; /* elements */
  const int32_t *draft_tokens; /* [B,k_max] */
  const int32_t *draft_len;    /* [B] or NULL */
  /* state (read-only) */
  int32_t cap;
  const float *LA, *LR;        /* [B,cap] */
  const int32_t *nA, *nR;      /* [B] */
  /* randomness */
  uint64_t seed;
  const uint32_t *seq_id;      /* [B] or NULL -> b */
  const uint32_t *round;       /* [B] or NULL -> round0 */
  uint32_t round0;
  /* options */
  int32_t reject_rule;         /* 0 Bernoulli(P_A), 1 MAP (reject iff P_A < 1/2) */
  int32_t kde_min_n;           /* >= 2 */
  int32_t bw_rule;             /* 0 Silverman, 1 Scott */
  int32_t relaxed_off;         /* 1: posterior test disabled */
  int32_t base_test;           /* 0: speculative-sampling ratio test + residual resampling (Section 2.1.3);
                                  1: the test of Algorithm 1's verification loop, x_i != y_i with
                                     y_i ~ p_i, in its distribution-identical form: accept with
                                     probability p_i(x_i); on rejection the appended token is y_r
                                     given y_r != x_r, i.e. drawn from p_r with x_r excluded */
  int32_t list_update;         /* 0: every position of the round sees the lists as of the round's start;
                                  1: as in Algorithm 1's loop, position i sees the distances of
                                     positions 1..i-1 of this round already appended to L_D^A */
  double d_eps;                /* boundary band of the "0 < d < 1" filter used by list_update = 1 */
  /* outputs */
  int32_t *n_accept;           /* [B] */
  int32_t *next_token;         /* [B] */
  double *H_p, *H_q;           /* [B,k_max] nats */
  double *d_js;                /* [B,k_max] dhat */
  double *p_accept;            /* [B,k_max] */
  uint8_t *accept_mask;        /* [B,k_max] bit0 base, bit1 relaxed */
  uint32_t *status;            /* [B] */
  /* diagnostics for the tests' flip accounting */
  double *base_margin;         /* [B,k_max] ln u1 - min(0, ln p(x) - ln q(x)) */
  double *relaxed_margin;      /* [B,k_max] u2 - P_A */
  double *top2_gap;            /* [B] best key minus runner-up key at the sampled row */
} adasd_oracle_verify_args;

/* Returns 0, or -1 on invalid arguments. Threads over sequences when built with OpenMP. */
int adasd_oracle_verify(const adasd_oracle_verify_args *a);

/* Update step of Algorithm 1 (list appends with the open-interval filter,
 * running mean of rejected entropies).                                         */
void adasd_oracle_update(int B, int k_max, int cap, const int32_t *n_accept,
                         const int32_t *draft_len, const double *H_q, const double *d_js,
                         double d_eps, float *LA, float *LR, int32_t *nA, int32_t *nR,
                         double *ent_sum, int32_t *ent_cnt, float *T_G, uint32_t *status);

int adasd_oracle_num_threads(void);

#ifdef __cplusplus
}
#endif
#endif
