/*
 * adasd.h -- C ABI of the MI355X (gfx950) library for the per-round statistics,
 * verification and threshold update of Adaptive Speculative Decoding (AdaSD).
 *
 * One decode round of Algorithm 1 of the paper, seen from this library:
 *   generation  : for every drafting step call adasd_draft_step on the draft logits; it
 *                 draws the token x_i ~ q_i and returns H(q_i) and the stop flag
 *                 H(q_i) > T_G (Section 4.3; generation loop of Algorithm 1).  A
 *                 caller with a sampler of its own calls adasd_draft_entropy instead,
 *                 which leaves out the draw;
 *   verification: once the window is drafted call adasd_verify with the target and
 *                 draft logits of the k candidates (Sections 2.1.3, 2.2, 4.4;
 *                 verification loop of Algorithm 1);
 *   update      : then adasd_update_thresholds folds the round's outcome into the
 *                 history lists and the generation threshold (Section 4.3; update
 *                 lines of Algorithm 1).
 * The draft and target transformers are outside this library: it only sees logits.
 *
 * Conventions for every entry point
 *   - returns 0 (ADASD_OK) or a negative ADASD_ERR_* code; never throws;
 *   - every pointer is DEVICE memory owned by the caller unless the comment says
 *     "host"; struct arguments themselves (adasd_state, adasd_verify_args,
 *     adasd_options) are host structs holding device pointers;
 *   - work is enqueued on the HIP stream passed as `stream` (a hipStream_t cast to
 *     void*, NULL = the default stream); no entry point synchronises, allocates or
 *     frees device memory;
 *   - argument errors are detected on the host before anything is enqueued; problems
 *     that depend on device data (token id outside the vocabulary, NaN/+inf logits,
 *     full history list, ...) are reported per sequence in a `status` bit mask;
 *   - logits are row-major with the vocabulary contiguous; strides are in ELEMENTS;
 *     rows whose byte address is 16-byte aligned take the 128-bit load path, other
 *     rows are still handled correctly by an element-wise path;
 *   - units: entropies in nats; the Jensen-Shannon distance is reported as
 *     d = sqrt(D_JS / ln 2), i.e. the base-2 normalisation under which the paper
 *     states the [0,1] bound and the "exactly 0 or 1" exclusion (Sections 2.2, 4.4);
 *   - accuracy: every entropy and every distance within 1e-5 |x| + 1e-6 of its exact value x (float
 *     arithmetic on probabilities of total mass 1; sums in a fixed order, so results are reproducible bit
 *     for bit).  That holds down to distances of 1e-3 and below, where it is a relative bound (each term
 *     of the distance is formed from the exact difference of the two logits, and small differences go
 *     through a series instead of through logarithms that cancel), and whatever offsets the two rows of a
 *     position carry (softmax does not see them): rows whose log-normalisers lie far apart take a
 *     compensated form of the same term.
 */
#ifndef ADASD_H
#define ADASD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { ADASD_F32 = 0, ADASD_BF16 = 1 } adasd_dtype;

enum {
  ADASD_OK = 0,
  ADASD_ERR_INVALID_ARG = -1, /* NULL pointer, negative size, bad enum, bad stride */
  ADASD_ERR_MISALIGNED = -2,  /* pointer below the natural alignment of its element type */
  ADASD_ERR_UNSUPPORTED = -3, /* option value that is declared but not built */
  ADASD_ERR_WORKSPACE = -4,   /* workspace NULL or smaller than adasd_workspace_bytes */
  ADASD_ERR_CAPACITY = -5,    /* size beyond a compiled limit (k_max, V, B) */
  ADASD_ERR_HIP = -6          /* a HIP runtime call failed (launch error) */
};

/* Per-sequence status bits written by adasd_verify / adasd_update_thresholds. */
enum {
  ADASD_ST_BAD_TOKEN = 1u,   /* a draft token id was outside [0,V): that position fails the base test */
  ADASD_ST_NONFINITE = 2u,   /* a needed row held NaN/+inf or no finite logit: its statistics are NaN,
                                the position is rejected, a token drawn from such a row is -1 */
  ADASD_ST_ZERO_MASS = 4u,   /* max(0, p - q) had no mass at the rejected position: token drawn from p */
  ADASD_ST_OVERFLOW = 8u,    /* a history list was full: the append was dropped */
  ADASD_ST_EXACT_PATH = 16u, /* informational: the float64 tie-resolution path chose the token */
  ADASD_ST_BAD_LENGTH = 32u, /* draft_len[b] outside [0,k_max]: clamped */
  ADASD_ST_UNSETTLED = 64u   /* column-sharded sampling only: the draw could not be settled from the exchanged
                                records (no element with certain mass, too many close candidates, or error
                                bounds that overlap); next_token is the provisional winner or -1 */
};

/* Compiled limits. */
#define ADASD_MAX_K 64            /* k_max <= 64 (the paper caps the window at W = 20) */
#define ADASD_MAX_V (1 << 24)     /* vocabulary size */

/*
 * Per-sequence adaptive state of Algorithm 1 (initialisation block), structure of
 * arrays.  L_E^R is only ever used through its mean, so it is kept as (sum, count).
 */
typedef struct {
  int32_t B;        /* sequences */
  int32_t cap;      /* capacity of each history list, per sequence */
  float *T_G;       /* [B]      generation threshold, nats; initial value 0 */
  double *ent_sum;  /* [B]      sum of H(q) over rejected candidates (L_E^R summed) */
  int32_t *ent_cnt; /* [B]      |L_E^R| */
  float *LA;        /* [B,cap]  JS distances of accepted candidates, values in (0,1) (L_D^A) */
  float *LR;        /* [B,cap]  JS distances of rejected candidates, values in (0,1) (L_D^R) */
  int32_t *nA;      /* [B]      |L_D^A| */
  int32_t *nR;      /* [B]      |L_D^R| */
  double *mom;      /* [B,4] or NULL.  Running sums of long lists for the bandwidth of the Bayesian test
                       (Section 4.4): sum and sum of squares of (x - LA[b,0]) over L_D^A, then of
                       (x - LR[b,0]) over L_D^R.  A pair is valid, kept by the update step and used by the
                       decision stage once its list holds 4096 samples (shorter lists are added up in
                       every call: they fit the registers of one workgroup); after writing the lists by
                       other means call adasd_state_refresh.  NULL: lists of any length are added up in
                       every call (one more pass over them). */
} adasd_state;

/*
 * Readings of the points the paper leaves open; zero-initialised = the defaults.
 */
typedef struct {
  int32_t base_test;   /* 0: speculative-sampling ratio test min(1,p/q) with re-sampling from
                          max(0,p-q) (Section 2.1.3).
                          1: the test written in Algorithm 1's verification loop, "x_i != y_i" with
                          y_i drawn from p_i, in its distribution-identical form: the candidate
                          passes with probability p_i(x_i) (u1 < p_i(x_i)); after a rejection the
                          appended token is y_r given y_r != x_r, i.e. drawn from p_r with the drafted
                          token excluded.  The draft logits then only enter H(q) and the JS distance.
                          Other values: ADASD_ERR_INVALID_ARG. */
  int32_t reject_rule; /* the undefined Reject(P(A|d)) of Algorithm 1:
                          0: Bernoulli, candidate kept if u < P(A|d);  1: MAP, kept if P(A|d) >= 1/2 */
  int32_t kde_min_n;   /* the Bayesian test is off until both lists hold this many samples
                          (values < 2 mean 2) and have non-zero variance */
  int32_t bw_rule;     /* KDE bandwidth: 0 Silverman's reference rule (4/(3n))^(1/5) sigma,
                          1 Scott's n^(-1/5) sigma; Gaussian kernel either way */
  int32_t relaxed_off; /* 1: Bayesian test disabled (the "Gen-Only" ablation of Section 5.3) */
  float d_eps;         /* distances <= d_eps or >= 1-d_eps count as "exactly 0 or 1" and are not
                          recorded (Section 4.4); 0 selects the default 1e-6 */
  int32_t stats_path;  /* kernels of the statistics stage: 0 the library's choice; 1 the two-kernel path
                          (normalisers, then JS distance: the logits are read twice); 2 the single-read
                          kernel when every row is 16-byte aligned and V is a whole number of 16-byte
                          vectors of at most 2^18, else the two-kernel path.  Same results to the
                          documented tolerance either way. */
  int32_t apply_update; /* 1: adasd_verify also applies the round to args->state, exactly as
                          adasd_update_thresholds would with the same d_eps (the decision kernel
                          does it after the sequence's decisions, which saves a launch);
                          ADASD_ST_OVERFLOW is then OR-ed into the verify status.  Needs a state. */
  int32_t list_update; /* when the accepted-distance list grows:
                          0: after the round (every position of a round sees the lists as they were
                          when the round started);
                          1: inside the verification loop, as Algorithm 1 writes it: position i's
                          posterior uses L_D^A extended by the distances of positions 1..i-1 of this
                          round that pass the d_eps filter and fit the capacity (a position is only
                          reached if all earlier ones were accepted; positions after the first
                          rejection are reported under the same rule), with the list-size prior
                          counted on the extended list.  The state itself is still only written by
                          the update step, which leaves the same lists either way. */
  int32_t wait_polls;  /* single-read statistics kernel: how often a workgroup polls for the results of the
                          other workgroups of its position before it stops waiting and recomputes them
                          itself (bit-identical results either way).  0: the default (16384, about 25 ms);
                          negative: do not wait at all, which tests use to exercise the recomputation
                          without any wave ever spinning. */
} adasd_options;

/*
 * Scratch memory.  adasd_workspace_bytes writes to *bytes (host) the size needed by
 * adasd_verify / adasd_draft_entropy for the given shape; the caller allocates it on
 * the device (256-byte aligned), calls adasd_workspace_init once (it zeroes the
 * arrival counters the kernels use; they clean up after themselves), and may reuse it
 * for any smaller shape.  Calls that share a workspace must be ordered on one stream.
 */
int adasd_workspace_bytes(int B, int k_max, int V, adasd_dtype dt, size_t *bytes /* host */);
int adasd_workspace_init(void *workspace, size_t ws_bytes, void *stream);

/* Algorithm 1, initialisation: empty lists, T_G = 0.  `st` is a host struct of device pointers. */
int adasd_state_init(const adasd_state *st, void *stream);
/* Recomputes st->mom from the lists as they are (no-op when st->mom is NULL). */
int adasd_state_refresh(const adasd_state *st, void *stream);

/*
 * Draft side (Section 4.3; generation loop of Algorithm 1).  For every active row b:
 *   H_out[b]    = Shannon entropy of softmax(draft_logits[b, :]) in nats (Appendix A);
 *   stop_out[b] = 1 if H_out[b] > T_G[b] (strict) or step + 1 >= k_max (window cap), else 0.
 * draft_logits: [B, V] with `row_stride` elements between rows.  T_G, active, stop_out may be
 * NULL (no threshold test / all rows active / no flag wanted).  Inactive rows are not read and
 * get H_out = 0, stop_out = 0.  A non-finite row gives H_out = NaN and stop_out = 1.
 */
int adasd_draft_entropy(const void *draft_logits, adasd_dtype dt, int B, int V,
                        int64_t row_stride, const float *T_G, const uint8_t *active, int step,
                        int k_max, float *H_out, uint8_t *stop_out, void *workspace,
                        size_t ws_bytes, void *stream);

/*
 * Draft side with the token draw (generation loop of Algorithm 1: "x_i ~ q_i", then the test
 * H(q_i) > T_G; Section 4.3): everything adasd_draft_entropy returns, plus
 *   token_out[b] = a token drawn from softmax(draft_logits[b, :]) by Gumbel-max,
 *                  argmax_v z_v - ln(-ln u_v), lowest index on ties, in the same single pass over
 *                  the logits (the normaliser does not move the argmax).  u_v is word v&3 of
 *                  Philox4x32-10 with key `seed` and counter (v>>2, step | 2<<16, round, sequence),
 *                  u = (w + 0.5) / 2^32: a stream of its own, disjoint from those of adasd_verify.
 *                  sequence = seq_id[b] (b if NULL), round = round[b] (round0 if NULL).
 *   status_out[b] (may be NULL) = ADASD_ST_NONFINITE for a row with NaN/+inf or no finite logit
 *                  (token -1, H NaN, stop 1), ADASD_ST_EXACT_PATH if the draw was settled in
 *                  float64, else 0.
 * Inactive rows are not read and get H 0, stop 0, token -1.  Pointers are device memory owned by the
 * caller; T_G, active, stop_out, seq_id, round, status_out may be NULL.  step must be below 65536.
 * Errors as for adasd_draft_entropy; nothing is launched when one is returned.
 */
int adasd_draft_step(const void *draft_logits, adasd_dtype dt, int B, int V, int64_t row_stride,
                     const float *T_G, const uint8_t *active, int step, int k_max, uint64_t seed,
                     const uint32_t *seq_id, const uint32_t *round, uint32_t round0, float *H_out,
                     uint8_t *stop_out, int32_t *token_out, uint32_t *status_out, void *workspace,
                     size_t ws_bytes, void *stream);

/*
 * Verification of one round (Sections 2.1.3, 2.2, 4.4; verification loop of Algorithm 1).
 * For sequence b with k_b = draft_len[b] candidates x_1..x_k (0-based position i below):
 *   p_i = softmax(target_logits[b,i,:]),  q_i = softmax(draft_logits[b,i,:]);
 *   H_p, H_q   : entropies (nats);   d_js : sqrt(D_JS(p_i||q_i) / ln 2);
 *   p_accept   : P(A|d) from Gaussian KDEs of the two history lists with list-size priors;
 *   base test  : u1 < min(1, p_i(x_i)/q_i(x_i));  Bayesian test per options.reject_rule on u2;
 *   a candidate is rejected only if BOTH tests reject it; n_accept = index of the first
 *   rejected candidate (k_b if none);
 *   next_token : drawn from max(0, p_r - q_r) normalised at the first rejected position r
 *                (from p_r if that has no mass), or from p_{k_b} (row k_b of the target, the
 *                "bonus" row) when everything was accepted, by Gumbel-max over the vocabulary:
 *                argmax_v ln w_v - ln(-ln u_v), lowest index on ties.
 * Random numbers: Philox4x32-10 keyed by `seed`; counter = (block, position | stream<<16, round,
 * sequence) where sequence = seq_id[b] (b if NULL) and round = round[b] (round0 if NULL).
 *   acceptance uniforms of position i: block 0, stream 0, word 0 -> u1, word 1 -> u2,
 *                                      u = ((word>>8) + 0.5) / 2^24;
 *   Gumbel noise of element v        : block v>>2, stream 1, word v&3, u = (word + 0.5) / 2^32.
 * Statistics are produced for every i < k_b (also after the first rejection); entries with
 * i >= k_b are set to 0.  The state is only read unless options.apply_update is set; otherwise apply
 * the round with adasd_update_thresholds.
 */
typedef struct {
  /* inputs */
  const void *target_logits;   /* [B, k_max+1, V] */
  const void *draft_logits;    /* [B, k_max,   V] */
  adasd_dtype dt;
  int32_t B, k_max, V;
  int64_t t_seq_stride, t_pos_stride; /* elements between sequences / positions of the target */
  int64_t d_seq_stride, d_pos_stride; /* same for the draft */
  const int32_t *draft_tokens; /* [B, k_max] */
  const int32_t *draft_len;    /* [B] or NULL (= k_max everywhere) */
  const adasd_state *state;    /* host struct; NULL = empty history (Bayesian test off) */
  uint64_t seed;
  const uint32_t *seq_id;      /* [B] or NULL */
  const uint32_t *round;       /* [B] or NULL */
  uint32_t round0;
  /* outputs */
  int32_t *n_accept;           /* [B]        0..k_b */
  int32_t *next_token;         /* [B] */
  float *H_p;                  /* [B, k_max] or NULL */
  float *H_q;                  /* [B, k_max] */
  float *d_js;                 /* [B, k_max] */
  float *p_accept;             /* [B, k_max] or NULL */
  uint8_t *accept_mask;        /* [B, k_max] or NULL; bit 0 base test, bit 1 Bayesian test */
  uint32_t *status;            /* [B] */
  void *workspace;
  size_t ws_bytes;
} adasd_verify_args;

int adasd_verify(const adasd_verify_args *args /* host */, const adasd_options *opt /* host, may be NULL */,
                 void *stream);

/*
 * adasd_verify for callers that cannot allocate device memory or pass a workspace: code that runs under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels
 * and bit-identical results; args->workspace and args->ws_bytes are ignored, the scratch memory is an
 * array of ADASD_NOALLOC_SCRATCH_BYTES inside the library's device image (every GPU the library runs on
 * holds its own copy until the process ends).  Calls no hipMalloc / hipFree or any allocating routine.
 * Limit: adasd_workspace_bytes(B, k_max, V, dt) must not exceed ADASD_NOALLOC_SCRATCH_BYTES (about 1200
 * candidate positions B * k_max), else ADASD_ERR_CAPACITY and nothing is launched.  All calls on one GPU
 * share that GPU's array: they must be ordered (one stream, or events between streams); calls that
 * overlap on one GPU race.  The first call on a GPU, and the first after a call that returned
 * ADASD_ERR_HIP, zeroes the array with a fill kernel on `stream`; after that every kernel leaves the
 * counters and hand-off words it used at zero, as with a caller's workspace.
 */
#define ADASD_NOALLOC_SCRATCH_BYTES ((size_t)8 << 20)
int adasd_verify_noalloc(const adasd_verify_args *args /* host */, const adasd_options *opt /* host, may be NULL */,
                         void *stream);

/*
 * Column-sharded verification.  With a tensor-parallel output layer every holder g of G has the columns
 * col_begin_g .. col_begin_g + V_g - 1 of every logit row.  The statistics of Appendix A and Section 2.2
 * are sums over the vocabulary, so each holder forms partial results over its own columns and only small
 * records travel (the caller moves them: on one device the G "holders" are G calls on column slices):
 *
 *   1. adasd_verify_shard_stats  (local)  -> triples_out  [rows][4]      rows = B*k_max*2, row 2*(b*k_max+i)
 *        is the target row and the next one the draft row of position (b,i): (reference m, sum of
 *        2^(z log2 e - m), sum of the same weighted by its exponent, 0) over the local columns;
 *   2. gather the triples of all holders into triples_all [G][rows][4];
 *      adasd_verify_shard_jsd    (local)  -> pos_out [B*k_max][4]: (partial Jensen-Shannon sum over the
 *        local columns under the global normalisers, z_p(x), z_q(x), 1 if the drafted token x of the
 *        position is a local column else 0);
 *   3. gather into pos_all [G][B*k_max][4];
 *      adasd_verify_shard_decide (replicated: every holder makes the same call and gets the same
 *        results)                 -> everything adasd_verify writes except next_token: n_accept, H_p,
 *        H_q, d_js, p_accept, accept_mask, status, and with options.apply_update the state.
 *
 * "local" calls take an adasd_verify_args whose V, logit pointers and strides describe the local column
 * slice (outputs and state are not touched); the "replicated" call takes the whole-vocabulary V =
 * shard->V_total, no logits, and the outputs.  All of a holder's calls of one round use the same
 * workspace, in this order, on one stream.  Results agree with adasd_verify to the documented tolerance
 * (the normalisers are folded from G partial sums instead of one launch's slices).  The holders' columns
 * must tile 0 .. V_total-1; col_begin must be a multiple of 8; G <= ADASD_MAX_SHARDS.
 */
#define ADASD_MAX_SHARDS 64
typedef struct {
  int32_t n_shards;  /* G */
  int32_t shard;     /* g: the holder whose columns a local call is given (ignored by replicated calls) */
  int32_t V_total;   /* vocabulary size over all holders */
  int32_t col_begin; /* first column of holder g (local calls) */
} adasd_shard;

int adasd_verify_shard_stats(const adasd_verify_args *local /* host */, const adasd_shard *shard /* host */,
                             float *triples_out, void *stream);
int adasd_verify_shard_jsd(const adasd_verify_args *local /* host */, const adasd_shard *shard /* host */,
                           const float *triples_all, float *pos_out, void *stream);
int adasd_verify_shard_decide(const adasd_verify_args *meta /* host */, const adasd_shard *shard /* host */,
                              const float *triples_all, const float *pos_all,
                              const adasd_options *opt /* host, may be NULL */, void *stream);

/*
 * Column-sharded sampling of the correction / bonus token (Section 2.1.3; last lines of the verification
 * step of Algorithm 1), after adasd_verify_shard_decide on the same workspace (it leaves the row, the
 * kind of draw and the normalisers of every sequence there).  The Gumbel noise of an element depends on
 * its vocabulary index only, so the holders' draws are those of adasd_verify.
 *
 *   4. adasd_verify_shard_sample (local)      -> top_out [B][4]: (best upper-bound key over the local
 *        columns, its vocabulary index as an int32 bit pattern (-1 none, -2 NaN/+inf in the row), the
 *        runner-up key, the margin by which the best's true key may lie below its bound);
 *   5. gather into top_all [G][B][4];
 *      adasd_verify_shard_pick   (replicated) -> next_token [B] where the winner is certain; tau_out [B]
 *        = +inf for those, else the key a candidate must reach (next_token then holds the provisional
 *        winner);
 *   6. adasd_verify_shard_refine (local)      -> cand_out [B] records of ADASD_SHARD_CAND_BYTES: for the
 *        open sequences the local elements that reach tau (vocabulary index and logits, at most 8) and
 *        the refined normaliser sums of the local columns;
 *   7. gather into cand_all [G][B];
 *      adasd_verify_shard_settle (replicated) -> next_token of the open sequences from float64 keys, with
 *        ADASD_ST_EXACT_PATH, and tau = +inf for them (candidates with identical logits and identical
 *        noise have identical keys whatever the normalisers are: an exact tie, won by the lower index);
 *        where the error bounds of the normalisers still overlap, ADASD_ST_UNSETTLED is set, the
 *        provisional token stays and tau stays finite;
 *   8. steps 6 and 7 once more with exact_sums = 1 (every term of the normaliser sums in float64, about
 *        a millisecond per open sequence and holder at V = 128256) close those: the settle call clears
 *        ADASD_ST_UNSETTLED when it succeeds.  What stays flagged has no sharded form: no element with
 *        certain mass (e.g. identical target and draft rows: adasd_verify then draws from the target row
 *        in float64 over the whole row) or more than 8 close candidates in one holder.
 * Steps 6 to 8 do nothing for sequences that are settled (about 1.7e-4 of the draws are open after step 5).
 * Local calls use args->seed, seq_id, round, round0; replicated calls write args->next_token and
 * args->status (bits are OR-ed into what adasd_verify_shard_decide wrote).
 */
#define ADASD_SHARD_CAND_BYTES 128
int adasd_verify_shard_sample(const adasd_verify_args *local /* host */, const adasd_shard *shard /* host */,
                              float *top_out, void *stream);
int adasd_verify_shard_pick(const adasd_verify_args *meta /* host */, const adasd_shard *shard /* host */,
                            const float *top_all, float *tau_out, void *stream);
int adasd_verify_shard_refine(const adasd_verify_args *local /* host */, const adasd_shard *shard /* host */,
                              const float *tau, int exact_sums, void *cand_out, void *stream);
int adasd_verify_shard_settle(const adasd_verify_args *meta /* host */, const adasd_shard *shard /* host */,
                              float *tau /* in, out */, const void *cand_all, void *stream);

/*
 * Update step (Section 4.3, Section 4.4 last paragraph; update lines of Algorithm 1).
 * For sequence b with r = n_accept[b]:
 *   every accepted position i < r : append d_js[b,i] to L_D^A unless it is "exactly 0 or 1";
 *   if r < k_b (a rejection)      : add H_q[b,r] to the rejected-entropy sum, append d_js[b,r] to
 *                                    L_D^R under the same filter;
 *   T_G[b] = mean rejected entropy (stays 0 while there is none).
 * A full list drops the append and sets ADASD_ST_OVERFLOW in status[b] (status may be NULL; bits are
 * OR-ed into it).  Non-finite H_q / d_js values are not recorded.
 */
int adasd_update_thresholds(const adasd_state *st /* host */, int k_max, const int32_t *n_accept,
                            const int32_t *draft_len /* or NULL */, const float *H_q,
                            const float *d_js, const adasd_options *opt /* host, may be NULL */,
                            uint32_t *status /* or NULL */, void *stream);

/*
 * Optional kernel timing for benchmarks (host side only; not for production loops).
 * adasd_profile_enable(n) creates n pairs of HIP events per kernel class and makes the entry points
 * hand one pair to each kernel launch (the dispatch stamps them at its start and end, so the
 * durations hold no launch or queueing time); adasd_profile_read waits for the recorded events and
 * returns the summed duration and the number of kernels of one class since the last enable;
 * adasd_profile_disable frees the events.  Kernel classes: 0 row statistics (normalisers + entropy; on
 * the single-read path the one kernel of the whole statistics stage, class 1 then stays empty),
 * 1 JS distance (two-kernel path), 2 decision, 3 token sampling, 4 state update, 5 drafting calls
 * (adasd_draft_entropy and adasd_draft_step: one kernel per call), 6 adasd_stream_read.
 * NOT thread-safe: there is one set of events per process, and while it is enabled every entry point
 * records into it.  Enable, the calls to be timed, read and disable must all come from one thread, with
 * no other thread inside the library meanwhile.  With timing disabled (the initial state) the entry
 * points share no mutable host state and may be called from several threads, each on its own stream
 * and workspace (adasd_verify_noalloc: see there).
 */
int adasd_profile_enable(int max_launches);
int adasd_profile_read(int kernel_class, double *total_ms /* host */, int *launches /* host */);
int adasd_profile_disable(void);

/*
 * Diagnostics for benchmarks: reads `bytes` bytes of device memory at `src` once, with 128-bit loads
 * in the launch shape of the statistics kernels (one workgroup per 32 KiB), and does nothing with them
 * beyond folding them into one word per workgroup, written to sink[0 .. ceil(bytes / 32768)).  Its
 * duration (kernel class 6) is the rate at which the chip streams that memory to a kernel without
 * arithmetic: the practical ceiling beside which the bandwidth of the statistics kernels is read.
 * src: device, 16-byte aligned, bytes a multiple of 16 (else ADASD_ERR_MISALIGNED); sink: device,
 * caller-owned, sink_words >= ceil(bytes / 32768) (else ADASD_ERR_WORKSPACE); bytes == 0
 * does nothing.  Enqueues one kernel on `stream`; allocates nothing and does not synchronise.
 */
int adasd_stream_read(const void *src, size_t bytes, uint32_t *sink, size_t sink_words, void *stream);

const char *adasd_strerror(int code);
int adasd_version(void);

#ifdef __cplusplus
}
#endif
#endif
