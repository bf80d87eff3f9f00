// Device code of the acceptance decisions of one sequence (Section 2.1.3, Section 4.4 and the
// verification loop of Algorithm 1 of the paper) and of the update step.
#pragma once
#include "internal.h"

namespace adasd {

// ---- reductions over half a wavefront (32 lanes) in double precision: rotations inside the rows of
// 16 lanes on the two 32-bit halves, then one exchange between the two rows.  All 32 lanes get the result.
template <int CTRL> __device__ __forceinline__ double dpp_rot_d(double v) {
  const int lo = __double2loint(v), hi = __double2hiint(v);
  return __hiloint2double(__builtin_amdgcn_update_dpp(0, hi, CTRL, 0xf, 0xf, false),
                          __builtin_amdgcn_update_dpp(0, lo, CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ double half_sum_d(double v) {
  v += dpp_rot_d<0x121>(v);
  v += dpp_rot_d<0x122>(v);
  v += dpp_rot_d<0x124>(v);
  v += dpp_rot_d<0x128>(v);
  return v + __shfl_xor(v, 16);
}
__device__ __forceinline__ double half_max_d(double v) {
  v = fmax(v, dpp_rot_d<0x121>(v));
  v = fmax(v, dpp_rot_d<0x122>(v));
  v = fmax(v, dpp_rot_d<0x124>(v));
  v = fmax(v, dpp_rot_d<0x128>(v));
  return fmax(v, __shfl_xor(v, 16));
}

// The lists hold distances strictly inside (d_eps, 1 - d_eps) (Section 4.4 leaves out the values "exactly 0
// or 1").  1 - d is exact in float from d = 1/2 on, so this is the comparison of the real numbers; 1 - d_eps
// rounded to float would shut out the float just below it.  NaN fails both.
__device__ __forceinline__ bool inside_open_interval(float d, float d_eps) { return d > d_eps && 1.0f - d > d_eps; }

struct Kde {
  double inv2h2;   // 1 / (2 h^2)
  double log_norm; // ln(n h sqrt(2 pi)) - ln prior  (subtracted from the log kernel sum)
};

// Gaussian-kernel constants of a history list from its shifted moments (sum and sum of squares of
// x - shift): sample variance with n-1, the bandwidth rule, the list-size prior.
__device__ inline bool kde_constants(double s1, double s2, int n, int n_other, int bw_rule, Kde* out) {
  const double var = (s2 - s1 * s1 / (double)n) / (double)(n - 1);
  if (!(var > 0.0)) return false;
  // x^(1/5) through the hardware exp2 / log2 (relative error about 1e-7: far inside what the
  // posterior's tolerance asks of the bandwidth)
  const float base = bw_rule == 1 ? 1.0f / (float)n : 4.0f / (3.0f * (float)n);
  const double factor = (double)ex2((float)(0.2 * log2_acc(base)));
  const double h = factor * sqrt(var);
  out->inv2h2 = 1.0 / (2.0 * h * h);
  const float prior = (float)n / (float)(n + n_other);
  out->log_norm = kLn2 * (log2_acc((float)((double)n * h * 2.50662827463100050242)) - log2_acc(prior));
  return true;
}

// ln [ p(d | list) P(list) ] evaluated by half a wavefront: max-shifted log-sum-exp of the kernels.
__device__ inline double half_log_joint(double d, const float* L, int n, const Kde& k) {
  const int l32 = threadIdx.x & 31;
  double tmax = -INFINITY;
  for (int j = l32; j < n; j += 32) {
    double e = d - (double)L[j];
    tmax = fmax(tmax, -(e * e) * k.inv2h2);
  }
  tmax = half_max_d(tmax);
  float acc = 0.f;
  for (int j = l32; j < n; j += 32) {
    double e = d - (double)L[j];
    double t = -(e * e) * k.inv2h2 - tmax;            // <= 0
    acc += ex2((float)(t * 1.44269504088896340736));  // e^t; terms below 2^-126 vanish
  }
  const double total = half_sum_d((double)acc);
  return tmax + kLn2 * log2_acc((float)total) - k.log_norm;
}

// The same over a list that continues in a second array: samples 0..n-1 from L, n..n+nx-1 from X.
__device__ inline double half_log_joint_ext(double d, const float* L, int n, const float* X, int nx, const Kde& k) {
  const int l32 = threadIdx.x & 31, nt = n + nx;
  double tmax = -INFINITY;
  for (int j = l32; j < nt; j += 32) {
    double e = d - (double)(j < n ? L[j] : X[j - n]);
    tmax = fmax(tmax, -(e * e) * k.inv2h2);
  }
  tmax = half_max_d(tmax);
  float acc = 0.f;
  for (int j = l32; j < nt; j += 32) {
    double e = d - (double)(j < n ? L[j] : X[j - n]);
    double t = -(e * e) * k.inv2h2 - tmax;
    acc += ex2((float)(t * 1.44269504088896340736));
  }
  const double total = half_sum_d((double)acc);
  return tmax + kLn2 * log2_acc((float)total) - k.log_norm;
}

struct DecideShared {
  int first_reject, k_b;            // of the sequence, for a fused update step
  float extra[ADASD_MAX_K];         // in-loop appends: this round's distances that pass the filter, in position order
  uint8_t n_before[ADASD_MAX_K];    // in-loop appends: how many of them come from earlier positions
  double mom[kWaves][4];            // per-wave shifted moments of the two lists
  double lse2[ADASD_MAX_K][2];      // normalisers of the candidate positions (for the sampling plan)
  uint8_t acc[ADASD_MAX_K];         // 1: position accepted
  uint8_t bad[ADASD_MAX_K];
  float dist[ADASD_MAX_K];          // the round's distances (in-loop appends; the fused update step)
  float hq[ADASD_MAX_K];            // the round's draft entropies (the fused update step)
  float la[kNarrowMax], lr[kNarrowMax];   // both lists, staged while their moments are formed
  uint32_t status;
};

// Everything a candidate position needs from memory, and its two uniforms.
struct PosLoad {
  int x;
  bool x_ok;
  float zp, zq, p0, p1;
  RowResult rp, rq;
  double log_u1, u2;
};

template <int DT>
__device__ __forceinline__ PosLoad load_position(const DecideArgs& a, const Workspace& ws, int b, int i, uint32_t rnd,
                                                 uint32_t seq) {
  const int l32 = threadIdx.x & 31, K = a.map.K;
  PosLoad L;
  const size_t o = (size_t)b * K + i;
  L.x = a.draft_tokens[o];
  L.x_ok = L.x >= 0 && L.x < a.map.V;
  const char* prow = a.map.base[0] +
      ((int64_t)b * a.map.seq_stride[0] + (int64_t)i * a.map.pos_stride[0]) * Elem<DT>::bytes;
  const char* qrow = a.map.base[1] +
      ((int64_t)b * a.map.seq_stride[1] + (int64_t)i * a.map.pos_stride[1]) * Elem<DT>::bytes;
  if (a.tok) {            // looked up already (by the JS kernel, or by the shard that owns the column)
    const float2 z = a.tok[o];
    L.zp = z.x;
    L.zq = z.y;
  } else {
    L.zp = load_elem<DT>(prow, L.x_ok ? L.x : 0);
    L.zq = load_elem<DT>(qrow, L.x_ok ? L.x : 0);
  }
  L.rp = ws.rows[2 * o];
  L.rq = ws.rows[2 * o + 1];
  L.p0 = L.p1 = 0.f;
  if (a.jsd_split > 0) {
    const float* part = reinterpret_cast<const float*>(ws.part2 + o * kMaxSplit);
    L.p0 = l32 < a.jsd_split ? part[2 * l32] : 0.f;
    L.p1 = l32 + 32 < a.jsd_split ? part[2 * (l32 + 32)] : 0.f;
  }
  const U4 r = philox4x32_10(0u, (uint32_t)i, rnd, seq, a.seed_lo, a.seed_hi);
  // u1 = (w + 0.5) / 2^24 rounded to float: 3e-8 relative, i.e. 3e-8 absolute on its logarithm
  L.log_u1 = kLn2 * log2_acc((float)(((double)(r.w[0] >> 8) + 0.5) * (1.0 / 16777216.0)));
  L.u2 = ((double)(r.w[1] >> 8) + 0.5) * (1.0 / 16777216.0);
  return L;
}

// Two-kernel path: the JS kernel left one partial sum per slice.  Half a wavefront adds them up in a
// fixed tree, corrects the common scale to first order (the weights were formed with the float
// roundings cp, cq of the normalisers, i.e. they are p(1+c), q(1+c') with c = ln2 (lse2_p - cp)) and
// takes the root.
__device__ __forceinline__ float fold_distance(const PosLoad& L) {
  const double A = half_sum_d((double)L.p0 + (double)L.p1);
  const double c0 = kLn2 * (L.rp.lse2 - (double)(float)L.rp.lse2), c1 = kLn2 * (L.rq.lse2 - (double)(float)L.rq.lse2);
  double D = 0.5 * A * (1.0 - 0.5 * (c0 + c1));   // bits
  D = fmin(fmax(D, 0.0), 1.0);
  return (L.rp.bad || L.rq.bad) ? NAN : (float)sqrt(D);
}

// The hand-off words that the single-read statistics kernel left for `count` positions from `first` on go
// back to zero (they are only read inside that kernel, which has finished; the next call finds them clear).
// The stores are dealt to the threads from the last one backwards: the first wavefront, which carries the
// latency chains of these kernels, gets none unless there are more than 192 words.
__device__ __forceinline__ void clear_exchange_words(const DecideArgs& a, const Workspace& ws, size_t first, int count) {
  if (a.xchg_split <= 0) return;
  const int per_pos = a.xchg_split * kXchgWords;
  for (int j = kBlock - 1 - (int)threadIdx.x; j < count * per_pos; j += kBlock) {
    const int i = j / per_pos, w = j - i * per_pos;
    __hip_atomic_store(ws.xchg + (first + i) * (size_t)(kMaxSplit * kXchgWords) + w, 0ull, __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
  }
}

// The decisions of one sequence by one workgroup of 256 threads.  INLOOP: the accepted list grows
// inside the verification loop (Algorithm 1): position i sees the list of the state followed by the
// distances of positions 0..i-1 of this round that pass the open-interval filter, up to the capacity.
template <int DT, bool INLOOP>
__device__ void decide_sequence(const DecideArgs& a, const Workspace& ws, int b, DecideShared& sh) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = tid & 31, grp = tid >> 5;
  constexpr int kGroups = kBlock / 32;
  const int K = a.map.K;
  if (tid == 0) sh.status = 0;

  int kb = K;
  uint32_t st = 0;
  if (a.map.draft_len) {
    int raw = a.map.draft_len[b];
    kb = min(max(raw, 0), K);
    if (raw != kb) st |= ADASD_ST_BAD_LENGTH;
  }

  const uint32_t seq = a.seq_id ? a.seq_id[b] : (uint32_t)b;
  const uint32_t rnd = a.round ? a.round[b] : a.round0;

  // Two chains of dependent loads run side by side: list lengths -> samples and, where the token's
  // logits were not looked up beforehand, token -> its logits.  The lengths are asked for first, then
  // the first position of each group, then the samples: a wavefront issues in order, so whatever
  // stands behind the wait for the token must not be the start of the other chain.
  const int min_n = a.kde_min_n < 2 ? 2 : a.kde_min_n;
  int nA = 0, nR = 0;
  const float* LA = nullptr;
  const float* LR = nullptr;
  if (a.LA && a.LR && a.nA && a.nR) {
    nA = min(max(a.nA[b], 0), a.cap);
    nR = min(max(a.nR[b], 0), a.cap);
    LA = a.LA + (size_t)b * a.cap;
    LR = a.LR + (size_t)b * a.cap;
  }
  auto load_pos = [&](int i) { return load_position<DT>(a, ws, b, i, rnd, seq); };
  PosLoad first;
  if (grp < kb) first = load_pos(grp);

  // ---- Bayesian test set-up: both lists need enough samples and spread (else P(A|d) = 0).
  // One pass over both lists (moments about the first element), one workgroup reduction; the samples
  // stay in shared memory for the kernel sums of the positions.
  int n_room = 0;        // in-loop appends the list can still take
  if (INLOOP) {
    // All distances of the round first: the groups fold them, one wavefront ranks those that pass.
    for (int i = grp; i < kb; i += kGroups) {
      const size_t o = (size_t)b * K + i;
      const PosLoad L = (i == grp) ? first : load_pos(i);
      float dv;
      if (a.jsd_split > 0) {
        dv = fold_distance(L);
        if (l32 == 0) a.d_js[o] = dv;
      } else {
        dv = (L.rp.bad || L.rq.bad) ? NAN : a.d_js[o];
      }
      if (l32 == 0) sh.dist[i] = dv;
    }
    __syncthreads();
    if (wave == 0) {
      const float dv = lane < kb ? sh.dist[lane] : NAN;
      const bool pass = inside_open_interval(dv, a.d_eps);
      const unsigned long long mask = __ballot(pass);
      const int rank = __popcll(mask & ((1ull << lane) - 1ull));
      if (lane < kb) sh.n_before[lane] = (uint8_t)rank;
      if (pass) sh.extra[rank] = dv;
    }
    __syncthreads();
    n_room = LA ? max(a.cap - nA, 0) : 0;
  }
  // (no positions, no test: the launch sends lists of kNarrowMax samples or more to the other form unless k_max is 0)
  bool kde_on = K > 0 && !a.relaxed_off && nR >= min_n && (INLOOP ? (LA != nullptr && nA + n_room >= min_n) : nA >= min_n);
  Kde kA, kR;
  double cA = 0.0, cR = 0.0;
  double m[4] = {0.0, 0.0, 0.0, 0.0};
  if (kde_on) {          // uniform over the workgroup
    cA = nA > 0 ? (double)LA[0] : (double)sh.extra[0];   // (with an empty list the shift is only used once an extra exists)
    cR = (double)LR[0];
    // (lists this short never have running sums in the state: they are added up here)
    for (int j = tid; j < nA; j += kBlock) {
      const float v = LA[j];
      if (j < kNarrowMax) sh.la[j] = v;
      const double e = (double)v - cA;
      m[0] += e;
      m[1] += e * e;
    }
    for (int j = tid; j < nR; j += kBlock) {
      const float v = LR[j];
      if (j < kNarrowMax) sh.lr[j] = v;
      const double e = (double)v - cR;
      m[2] += e;
      m[3] += e * e;
    }
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      m[x] = half_sum_d(m[x]);
      m[x] += __shfl_xor(m[x], 32);
    }
    if (lane == 0) {
#pragma unroll
      for (int x = 0; x < 4; ++x) sh.mom[wave][x] = m[x];
    }
    __syncthreads();     // (also: the staged samples are in place)
#pragma unroll
    for (int x = 0; x < 4; ++x) m[x] = (sh.mom[0][x] + sh.mom[1][x]) + (sh.mom[2][x] + sh.mom[3][x]);
    if (!INLOOP) {
      const bool okA = kde_constants(m[0], m[1], nA, nR, a.bw_rule, &kA);
      const bool okR = kde_constants(m[2], m[3], nR, nA, a.bw_rule, &kR);
      kde_on = okA && okR;
    }
  }

  // ---- half a wavefront per candidate position
  for (int i = grp; i < K; i += kGroups) {
    const size_t o = (size_t)b * K + i;
    if (i >= kb) {
      if (l32 == 0) {
        if (a.H_p) a.H_p[o] = 0.f;
        a.H_q[o] = 0.f;
        a.d_js[o] = 0.f;
        if (a.p_accept) a.p_accept[o] = 0.f;
        if (a.accept_mask) a.accept_mask[o] = 0;
        sh.acc[i] = 0;
        sh.bad[i] = 0;
      }
      continue;
    }
    const PosLoad L = (i == grp) ? first : load_pos(i);
    const RowResult& rp = L.rp;
    const RowResult& rq = L.rq;
    const bool bad = rp.bad || rq.bad;
    double d;
    if (INLOOP) {
      d = (double)sh.dist[i];
    } else if (a.jsd_split > 0) {
      const float d_out = fold_distance(L);
      if (l32 == 0) {
        a.d_js[o] = d_out;
        sh.dist[i] = d_out;
      }
      d = (double)d_out;
    } else {
      const float d_in = a.d_js[o];
      if (l32 == 0) sh.dist[i] = bad ? NAN : d_in;
      d = (double)d_in;
    }
    if (l32 == 0) sh.hq[i] = bad ? NAN : rq.H;
    double PA = 0.0;
    if (INLOOP) {
      if (!bad && kde_on) {
        // the list as position i sees it: its size, its moments, the prior on the sizes
        const int ne = min((int)sh.n_before[i], n_room), n_i = nA + ne;
        double s1 = m[0], s2 = m[1];
        for (int j = 0; j < ne; ++j) {
          const double e = (double)sh.extra[j] - cA;
          s1 += e;
          s2 += e * e;
        }
        if (n_i >= min_n && kde_constants(s1, s2, n_i, nR, a.bw_rule, &kA) &&
            kde_constants(m[2], m[3], nR, n_i, a.bw_rule, &kR)) {
          double ja = half_log_joint_ext(d, sh.la, nA, sh.extra, ne, kA);
          double jr = half_log_joint(d, sh.lr, nR, kR);
          PA = 1.0 / (1.0 + (double)ex2((float)((jr - ja) * 1.44269504088896340736)));
        }
      }
    } else if (!bad && kde_on) {
      double ja = half_log_joint(d, sh.la, nA, kA);
      double jr = half_log_joint(d, sh.lr, nR, kR);
      PA = 1.0 / (1.0 + (double)ex2((float)((jr - ja) * 1.44269504088896340736)));
    }
    if (l32 != 0) continue;
    sh.lse2[i][0] = rp.lse2;
    sh.lse2[i][1] = rq.lse2;
    sh.bad[i] = bad;
    if (bad) {
      if (a.H_p) a.H_p[o] = NAN;
      a.H_q[o] = NAN;
      a.d_js[o] = NAN;
      if (a.p_accept) a.p_accept[o] = NAN;
      if (a.accept_mask) a.accept_mask[o] = 0;
      sh.acc[i] = 0;
      atomicOr(&sh.status, (uint32_t)ADASD_ST_NONFINITE);
      continue;
    }
    // speculative-sampling test: accept with probability min(1, p(x)/q(x)), in the log domain; or the
    // loop's own match test: accept with probability p(x)
    int base = 0;
    if (!L.x_ok) {
      atomicOr(&sh.status, (uint32_t)ADASD_ST_BAD_TOKEN);
    } else if (a.base_test == 1) {
      base = L.log_u1 < (double)L.zp - rp.lse2 * kLn2;
    } else {
      double lp = (double)L.zp - rp.lse2 * kLn2;
      double lq = (double)L.zq - rq.lse2 * kLn2;
      double log_ratio = lp - lq;
      if (log_ratio > 0.0) log_ratio = 0.0;
      base = L.log_u1 < log_ratio;   // false for NaN (both probabilities zero)
    }
    const int relaxed = a.reject_rule == 1 ? (PA >= 0.5) : (L.u2 < PA);
    if (a.p_accept) a.p_accept[o] = (float)PA;
    if (a.accept_mask) a.accept_mask[o] = (uint8_t)(base | (relaxed << 1));
    sh.acc[i] = (uint8_t)(base || relaxed);   // rejected only if both tests reject
  }
  __syncthreads();
  if (tid == 0) {
    int r = kb;
    for (int i = 0; i < kb; ++i)
      if (!sh.acc[i]) {
        r = i;
        break;
      }
    a.n_accept[b] = r;
    st |= sh.status;
    SamplePlan plan;
    plan.row = r;
    plan.excluded = -1;
    if (r < kb) {
      plan.residual = 1;
      if (a.base_test == 1) {
        // replacement from the target row without the drafted token (a broken token excludes nothing)
        const int x = a.draft_tokens[(size_t)b * K + r];
        const bool x_ok = x >= 0 && x < a.map.V;
        plan.residual = x_ok ? 2 : 0;
        plan.excluded = x_ok ? x : -1;
      }
      plan.valid = !sh.bad[r];
      plan.lse2_p = sh.lse2[r][0];
      plan.lse2_q = sh.lse2[r][1];
    } else {
      plan.residual = 0;   // bonus row: Gumbel-max needs no normaliser
      plan.valid = 1;
      plan.lse2_p = 0.0;
      plan.lse2_q = 0.0;
    }
    ws.plan[b] = plan;
    a.status[b] = st;
    sh.first_reject = r;
    sh.k_b = kb;
  }
  clear_exchange_words(a, ws, (size_t)b * K, K);
  __syncthreads();
}

}  // namespace adasd

namespace adasd {

// Update step of one sequence (Section 4.3, last paragraph of Section 4.4; update lines of Algorithm 1)
// by one wavefront, one lane per candidate position (k_max <= 64).  Every lane reads its position's
// distance at once; accepted positions that pass the open-interval filter are appended in position
// order (rank = number of passing positions before it, from a ballot).
// d: the lane's distance (lanes <= r, below kb), H: the draft entropy of the rejected position (lane r).
// Returns the status bits of the step (complete in the lane that finishes the sequence: lane r, or 63);
// with or_status they are also OR-ed into status[b].
__device__ inline uint32_t update_sequence_core(const UpdateArgs& a, int b, int lane, int r, int kb, float d, float H,
                                                bool or_status = true) {
  const int nA = a.nA[b], nR = a.nR[b];
  double ent_sum = a.ent_sum[b];      // (asked for with the lengths: the last lane needs them at the very end)
  int ent_cnt = a.ent_cnt[b];
  if (!(lane <= r && lane < kb)) d = 0.f;
  const bool pass = inside_open_interval(d, a.d_eps);
  uint32_t st = 0;
  // accepted positions 0 .. r-1
  const unsigned long long acc = __ballot(pass && lane < r);
  if (pass && lane < r) {
    const int slot = nA + __popcll(acc & ((1ull << lane) - 1ull));
    if (slot < a.cap) a.LA[(size_t)b * a.cap + slot] = d;
  }
  const int nA_new = min(nA + __popcll(acc), a.cap);
  if (nA + __popcll(acc) > a.cap) st |= ADASD_ST_OVERFLOW;
  // the lane of the rejected position finishes the sequence (with all 64 positions accepted: the last lane)
  const int fin = r < 64 ? r : 63;
  // Running sums of the lists about their first elements: kept from the moment a list reaches kSumsMin
  // samples (added up from scratch in that call), so short lists cost nothing here.
  if (a.mom && (nA_new >= kSumsMin || nR + 1 >= kSumsMin)) {       // (uniform)
    const bool rej_appended = r < kb && __shfl((int)pass, fin) && nR < a.cap;
    const int nR_after = nR + (rej_appended ? 1 : 0);
    const float d_rej = __shfl(d, fin);
    if (nA_new >= kSumsMin && nA_new > nA) {
      const float* LAb = a.LA + (size_t)b * a.cap;
      const double c = (double)LAb[0];          // nA >= kSumsMin - 64 > 0: the first element is an old one
      double s1 = 0.0, s2 = 0.0;
      if (nA < kSumsMin) {                       // the list crosses the mark: everything it held before
        for (int j = lane; j < nA; j += 64) {
          const double e = (double)LAb[j] - c;
          s1 += e;
          s2 += e * e;
        }
      }
      if (pass && lane < r && nA + __popcll(acc & ((1ull << lane) - 1ull)) < a.cap) {
        const double e = (double)d - c;
        s1 += e;
        s2 += e * e;
      }
      s1 = half_sum_d(s1);
      s1 += __shfl_xor(s1, 32);
      s2 = half_sum_d(s2);
      s2 += __shfl_xor(s2, 32);
      if (lane == 0) {
        const bool fresh = nA < kSumsMin;
        a.mom[4 * b + 0] = (fresh ? 0.0 : a.mom[4 * b + 0]) + s1;
        a.mom[4 * b + 1] = (fresh ? 0.0 : a.mom[4 * b + 1]) + s2;
      }
    }
    if (nR_after >= kSumsMin && rej_appended) {
      const float* LRb = a.LR + (size_t)b * a.cap;
      const double c = (double)LRb[0];
      double s1 = 0.0, s2 = 0.0;
      if (nR < kSumsMin) {
        for (int j = lane; j < nR; j += 64) {
          const double e = (double)LRb[j] - c;
          s1 += e;
          s2 += e * e;
        }
      }
      if (lane == 0) {
        const double e = (double)d_rej - c;
        s1 += e;
        s2 += e * e;
      }
      s1 = half_sum_d(s1);
      s1 += __shfl_xor(s1, 32);
      s2 = half_sum_d(s2);
      s2 += __shfl_xor(s2, 32);
      if (lane == 0) {
        const bool fresh = nR < kSumsMin;
        a.mom[4 * b + 2] = (fresh ? 0.0 : a.mom[4 * b + 2]) + s1;
        a.mom[4 * b + 3] = (fresh ? 0.0 : a.mom[4 * b + 3]) + s2;
      }
    }
  }
  if (lane != fin) return st;
  int nR_new = nR;
  if (r < kb) {
    if (isfinite(H)) {
      ent_sum += (double)H;
      ent_cnt += 1;
      a.ent_sum[b] = ent_sum;
      a.ent_cnt[b] = ent_cnt;
    }
    if (pass) {
      if (nR < a.cap) a.LR[(size_t)b * a.cap + nR_new++] = d;
      else st |= ADASD_ST_OVERFLOW;
    }
  }
  a.nA[b] = nA_new;
  a.nR[b] = nR_new;
  a.T_G[b] = ent_cnt > 0 ? (float)(ent_sum / (double)ent_cnt) : 0.f;
  if (or_status && a.status && st) a.status[b] |= st;
  return st;
}

// The update step right after the decisions of the same workgroup: distances and entropies as that
// left them in shared memory (the values it wrote to d_js / H_q).
__device__ inline void update_sequence_shared(const UpdateArgs& a, int b, int lane, int r, int kb,
                                              const DecideShared& sh) {
  float d = 0.f, H = 0.f;
  if (lane <= r && lane < kb) d = sh.dist[lane];
  if (lane == r && r < kb) H = sh.hq[r];
  update_sequence_core(a, b, lane, r, kb, d, H);
}

__device__ inline void update_sequence(const UpdateArgs& a, int b, int lane, int r, int kb) {
  float d = 0.f, H = 0.f;
  if (lane <= r && lane < kb) d = a.d_js[(size_t)b * a.K + lane];
  if (lane == r && r < kb) H = a.H_q[(size_t)b * a.K + r];
  update_sequence_core(a, b, lane, r, kb, d, H);
}


// ---------------------------------------------------------------------------------------------
// Long histories.  The cost of the Bayesian test grows with the lists (Section 4.4 flags it): with
// thousands of samples per list one workgroup per sequence and half a wavefront per position is far
// too little.  Here one workgroup of 256 threads takes ONE position: every thread walks a stride of
// both lists once (running maximum and rescaled sum, so no separate pass for the maximum), the
// workgroups of a sequence leave one record per position, and the one that arrives last takes the
// sequence's decisions (first rejection, sampling plan, status, update step).
// ---------------------------------------------------------------------------------------------
struct WideShared {
  double m[2][kWaves], s[2][kWaves];
  int last;
  int n_pass;           // in-loop appends: earlier positions of this round that pass the filter
};

constexpr int kWideU = 16;   // samples per thread in flight: one workgroup walks a list alone, so the latency of
                             // a load is only hidden by the thread's own other loads

// One batch of kernel exponents joins a thread's running maximum m and rescaled sum s: the batch's
// largest exponent first, then ONE rescale of the old sum.  valid: how many of x[] hold samples.
__device__ __forceinline__ void joint_terms(double d, const float (&x)[kWideU], int first, int nt, double inv2h2,
                                            double& m, double& s) {
  double t[kWideU];
  double hi = m;
#pragma unroll
  for (int u = 0; u < kWideU; ++u) {
    const double e = d - (double)x[u];
    t[u] = first + u * kBlock < nt ? -(e * e) * inv2h2 : -INFINITY;
    hi = fmax(hi, t[u]);
  }
  if (hi > -INFINITY) {                  // (a thread past the end of the list has nothing to add)
    // all exponents are <= 0; with m = -inf the old sum is 0 and its factor 2^-inf = 0
    float add = 0.f;
#pragma unroll
    for (int u = 0; u < kWideU; ++u) add += ex2((float)((t[u] - hi) * 1.44269504088896340736));
    s = s * (double)ex2((float)((m - hi) * 1.44269504088896340736)) + (double)add;
    m = hi;
  }
}

// Workgroup-wide log-sum of N lists' per-thread (m, s) pairs at once: common maximum, rescaled sums (a
// thread without samples has s = 0).  out[q] = ln sum_j exp(t_j) of list q.
template <int N>
__device__ __forceinline__ void joint_reduce(const double (&m)[N], const double (&s)[N], WideShared& w, double (&out)[N]) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  double M[N], sc[N];
#pragma unroll
  for (int q = 0; q < N; ++q) {
    M[q] = half_max_d(m[q]);
    M[q] = fmax(M[q], __shfl_xor(M[q], 32));
    sc[q] = m[q] > -INFINITY ? s[q] * (double)ex2((float)((m[q] - M[q]) * 1.44269504088896340736)) : 0.0;
    sc[q] = half_sum_d(sc[q]);
    sc[q] += __shfl_xor(sc[q], 32);
  }
  __syncthreads();
  if (lane == 0) {
#pragma unroll
    for (int q = 0; q < N; ++q) {
      w.m[q][wave] = M[q];
      w.s[q][wave] = sc[q];
    }
  }
  __syncthreads();
#pragma unroll
  for (int q = 0; q < N; ++q) {
    double Mb = w.m[q][0];
#pragma unroll
    for (int v = 1; v < kWaves; ++v) Mb = fmax(Mb, w.m[q][v]);
    double total = 0.0;
#pragma unroll
    for (int v = 0; v < kWaves; ++v)
      total += w.m[q][v] > -INFINITY ? w.s[q][v] * (double)ex2((float)((w.m[q][v] - Mb) * 1.44269504088896340736)) : 0.0;
    out[q] = Mb + kLn2 * log2_acc((float)total);
  }
}

// ln [ p(d | list) P(list) ] by the whole workgroup, streaming a list of any length; the list continues
// in X (nx samples).
__device__ inline double block_log_joint(double d, const float* L, int n, const float* X, int nx, const Kde& k,
                                         WideShared& w) {
  const int tid = threadIdx.x, nt = n + nx;
  double m[1] = {-INFINITY}, s[1] = {0.0}, out[1];
  for (int base = 0; base < nt; base += kWideU * kBlock) {
    float x[kWideU];
#pragma unroll
    for (int u = 0; u < kWideU; ++u) {
      const int j = min(base + tid + u * kBlock, nt - 1);
      x[u] = j < n ? L[j] : X[j - n];
    }
    joint_terms(d, x, base + tid, nt, k.inv2h2, m[0], s[0]);
  }
  joint_reduce<1>(m, s, w, out);
  return out[0] - k.log_norm;
}

template <int DT, bool INLOOP>
__device__ void decide_position_wide(const DecideArgs& a, const UpdateArgs& upd, const Workspace& ws,
                                     PosRecord* records, int b, int i, DecideShared& sh, WideShared& wsh) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = tid & 31, grp = tid >> 5;
  constexpr int kGroups = kBlock / 32;
  const int K = a.map.K;
  int kb = K;
  uint32_t st_seq = 0;
  if (a.map.draft_len) {
    const int raw = a.map.draft_len[b];
    kb = min(max(raw, 0), K);
    if (raw != kb) st_seq |= ADASD_ST_BAD_LENGTH;
  }
  const uint32_t seq = a.seq_id ? a.seq_id[b] : (uint32_t)b;
  const uint32_t rnd = a.round ? a.round[b] : a.round0;
  const size_t o = (size_t)b * K + i;

  PosRecord rec{0, 0u, 0.f, 0.f};
  if (i >= kb) {
    if (tid == 0) {
      if (a.H_p) a.H_p[o] = 0.f;
      a.H_q[o] = 0.f;
      a.d_js[o] = 0.f;
      if (a.p_accept) a.p_accept[o] = 0.f;
      if (a.accept_mask) a.accept_mask[o] = 0;
    }
  } else {
    const PosLoad L = load_position<DT>(a, ws, b, i, rnd, seq);
    const bool bad = L.rp.bad || L.rq.bad;
    const int min_n = a.kde_min_n < 2 ? 2 : a.kde_min_n;
    int nA = 0, nR = 0;
    const float* LA = nullptr;
    const float* LR = nullptr;
    if (a.LA && a.LR && a.nA && a.nR) {
      nA = min(max(a.nA[b], 0), a.cap);
      nR = min(max(a.nR[b], 0), a.cap);
      LA = a.LA + (size_t)b * a.cap;
      LR = a.LR + (size_t)b * a.cap;
    }
    // the state's running sums of a list are valid once it holds kSumsMin samples; requested with the lengths
    const bool sums_A = a.mom && LA && nA >= kSumsMin, sums_R = a.mom && LA && nR >= kSumsMin;
    double mom_pre[4] = {0.0, 0.0, 0.0, 0.0};
    if (sums_A) { mom_pre[0] = a.mom[4 * b + 0]; mom_pre[1] = a.mom[4 * b + 1]; }
    if (sums_R) { mom_pre[2] = a.mom[4 * b + 2]; mom_pre[3] = a.mom[4 * b + 3]; }
    int ne = 0;                            // in-loop appends this position sees
    if (INLOOP) {
      // distances of the earlier positions (each workgroup of the sequence forms them for itself)
      for (int j = grp; j < i; j += kGroups) {
        const PosLoad Lj = load_position<DT>(a, ws, b, j, rnd, seq);
        float dv;
        if (a.jsd_split > 0) dv = fold_distance(Lj);
        else dv = (Lj.rp.bad || Lj.rq.bad) ? NAN : a.d_js[(size_t)b * K + j];
        if (l32 == 0) sh.dist[j] = dv;
      }
      __syncthreads();
      if (wave == 0) {
        const float dv = lane < i ? sh.dist[lane] : NAN;
        const bool pass = inside_open_interval(dv, a.d_eps);
        const unsigned long long mask = __ballot(pass);
        if (pass) sh.extra[__popcll(mask & ((1ull << lane) - 1ull))] = dv;
        if (lane == 0) wsh.n_pass = __popcll(mask);
      }
      __syncthreads();
      ne = LA ? min(wsh.n_pass, max(a.cap - nA, 0)) : 0;
    }
    float d_out;
    if (a.jsd_split > 0) {
      d_out = fold_distance(L);
      if (tid == 0) a.d_js[o] = d_out;
    } else {
      d_out = bad ? NAN : a.d_js[o];
    }
    const double d = (double)d_out;
    const int n_i = nA + ne;
    double PA = 0.0;
    if (!a.relaxed_off && !bad && LA && n_i >= min_n && nR >= min_n) {      // uniform over the workgroup
      const double cA = nA > 0 ? (double)LA[0] : (double)sh.extra[0], cR = (double)LR[0];
      double m[4] = {0.0, 0.0, 0.0, 0.0};
      constexpr int U = kWideU;
      // Lists of up to U samples per thread are read ONCE, both at the same time, and stay in registers for
      // the moments and for the kernel sums; longer ones are streamed twice.
      const bool resident = n_i <= U * kBlock && nR <= U * kBlock;
      float xa[U], xr[U];
      if (resident) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int ja = min(tid + u * kBlock, n_i - 1), jr = min(tid + u * kBlock, nR - 1);
          xa[u] = ja < nA ? LA[ja] : sh.extra[ja - nA];
          xr[u] = LR[jr];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const double ea = tid + u * kBlock < n_i ? (double)xa[u] - cA : 0.0;
          const double er = tid + u * kBlock < nR ? (double)xr[u] - cR : 0.0;
          m[0] += ea;
          m[1] += ea * ea;
          m[2] += er;
          m[3] += er * er;
        }
      } else {
        if (!sums_A)
          for (int base = 0; base < n_i; base += U * kBlock) {
            float x[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
              const int j = min(base + tid + u * kBlock, n_i - 1);
              x[u] = j < nA ? LA[j] : sh.extra[j - nA];
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
              const double e = base + tid + u * kBlock < n_i ? (double)x[u] - cA : 0.0;
              m[0] += e;
              m[1] += e * e;
            }
          }
        if (!sums_R)
          for (int base = 0; base < nR; base += U * kBlock) {
            float x[U];
#pragma unroll
            for (int u = 0; u < U; ++u) x[u] = LR[min(base + tid + u * kBlock, nR - 1)];
#pragma unroll
            for (int u = 0; u < U; ++u) {
              const double e = base + tid + u * kBlock < nR ? (double)x[u] - cR : 0.0;
              m[2] += e;
              m[3] += e * e;
            }
          }
      }
      const bool both_sums = !resident && sums_A && sums_R;
      if (!both_sums) {              // (uniform) something was added up by the threads
#pragma unroll
        for (int x = 0; x < 4; ++x) {
          m[x] = half_sum_d(m[x]);
          m[x] += __shfl_xor(m[x], 32);
        }
        if (lane == 0) {
#pragma unroll
          for (int x = 0; x < 4; ++x) sh.mom[wave][x] = m[x];
        }
        __syncthreads();
#pragma unroll
        for (int x = 0; x < 4; ++x) m[x] = (sh.mom[0][x] + sh.mom[1][x]) + (sh.mom[2][x] + sh.mom[3][x]);
      }
      if (!resident && sums_A) {     // the state's sums, and the in-loop appends on top (every thread the same)
        m[0] = mom_pre[0];
        m[1] = mom_pre[1];
        for (int j = 0; j < ne; ++j) {
          const double e = (double)sh.extra[j] - cA;
          m[0] += e;
          m[1] += e * e;
        }
      }
      if (!resident && sums_R) {
        m[2] = mom_pre[2];
        m[3] = mom_pre[3];
      }
      Kde kA, kR;
      if (kde_constants(m[0], m[1], n_i, nR, a.bw_rule, &kA) && kde_constants(m[2], m[3], nR, n_i, a.bw_rule, &kR)) {
        double ja, jr;
        if (resident) {
          double mm[2] = {-INFINITY, -INFINITY}, ss[2] = {0.0, 0.0}, out[2];
          joint_terms(d, xa, tid, n_i, kA.inv2h2, mm[0], ss[0]);
          joint_terms(d, xr, tid, nR, kR.inv2h2, mm[1], ss[1]);
          joint_reduce<2>(mm, ss, wsh, out);
          ja = out[0] - kA.log_norm;
          jr = out[1] - kR.log_norm;
        } else {
          ja = block_log_joint(d, LA, nA, sh.extra, ne, kA, wsh);
          jr = block_log_joint(d, LR, nR, nullptr, 0, kR, wsh);
        }
        PA = 1.0 / (1.0 + (double)ex2((float)((jr - ja) * 1.44269504088896340736)));
      }
    }
    if (tid == 0) {
      rec.d = d_out;
      if (bad) {
        if (a.H_p) a.H_p[o] = NAN;
        a.H_q[o] = NAN;
        a.d_js[o] = NAN;
        if (a.p_accept) a.p_accept[o] = NAN;
        if (a.accept_mask) a.accept_mask[o] = 0;
        rec.bits = 2;
        rec.status = ADASD_ST_NONFINITE;
        rec.d = NAN;
      } else {
        int base = 0;
        if (!L.x_ok) {
          rec.status |= ADASD_ST_BAD_TOKEN;
        } else if (a.base_test == 1) {
          base = L.log_u1 < (double)L.zp - L.rp.lse2 * kLn2;
        } else {
          double log_ratio = ((double)L.zp - L.rp.lse2 * kLn2) - ((double)L.zq - L.rq.lse2 * kLn2);
          if (log_ratio > 0.0) log_ratio = 0.0;
          base = L.log_u1 < log_ratio;
        }
        const int relaxed = a.reject_rule == 1 ? (PA >= 0.5) : (L.u2 < PA);
        if (a.p_accept) a.p_accept[o] = (float)PA;
        if (a.accept_mask) a.accept_mask[o] = (uint8_t)(base | (relaxed << 1));
        rec.bits = (base || relaxed) ? 1 : 0;
      }
    }
  }
  // ---- the position's record, then the arrival counter of the sequence
  if (tid == 0) {
    PosRecord* dst = records + o;
    st_agent(&dst->bits, rec.bits);
    st_agent(reinterpret_cast<int*>(&dst->status), (int)rec.status);
    st_agent(&dst->d, rec.d);
    publish_barrier();
    const int ticket = atomicAdd(&ws.ticket2[b * ticket_stride(a.map.B, kTicket2Len)], 1);
    wsh.last = ticket == K - 1;
  }
  __syncthreads();
  clear_exchange_words(a, ws, o, 1);
  if (!wsh.last || wave != 0) return;

  // ---- last workgroup of the sequence, one wavefront, one lane per position
  // Every lane also asks for what the sampling plan and the update step need of ITS position (the
  // normalisers, the drafted token, the draft entropy: all left by earlier kernels), so that nothing is
  // loaded once the rejected position is known; its lane hands them over.
  int bits = 0;
  uint32_t pst = 0;
  float dl = 0.f, Hl = 0.f;
  double lse_p = 0.0, lse_q = 0.0;
  int xl = -1;
  if (lane < K) {
    const size_t ol = (size_t)b * K + lane;
    const PosRecord* src = records + ol;
    bits = ld_agent(&src->bits);
    pst = (uint32_t)ld_agent(reinterpret_cast<const int*>(&src->status));
    dl = ld_agent(&src->d);
    if (lane < kb) {
      lse_p = ws.rows[2 * ol].lse2;
      lse_q = ws.rows[2 * ol + 1].lse2;
      if (a.base_test == 1) xl = a.draft_tokens[ol];
      if (upd.B > 0) Hl = upd.H_q[ol];
    }
  }
  const unsigned long long rejected = __ballot(lane < kb && !(bits & 1));
  const int r = rejected ? __ffsll((long long)rejected) - 1 : kb;
  uint32_t st_all = pst;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) st_all |= __shfl_xor(st_all, off);
  const int src_lane = r < 64 ? r : 63;
  const int bad_r = __shfl(bits, src_lane) & 2;
  const double lse_p_r = __shfl(lse_p, src_lane), lse_q_r = __shfl(lse_q, src_lane);
  const int x_r = __shfl(xl, src_lane);
  if (lane == 0) {
    a.n_accept[b] = r;
    SamplePlan plan;
    plan.row = r;
    plan.excluded = -1;
    if (r < kb) {
      plan.residual = 1;
      if (a.base_test == 1) {
        const bool x_ok = x_r >= 0 && x_r < a.map.V;
        plan.residual = x_ok ? 2 : 0;
        plan.excluded = x_ok ? x_r : -1;
      }
      plan.valid = !bad_r;
      plan.lse2_p = lse_p_r;
      plan.lse2_q = lse_q_r;
    } else {
      plan.residual = 0;
      plan.valid = 1;
      plan.lse2_p = 0.0;
      plan.lse2_q = 0.0;
    }
    ws.plan[b] = plan;
    __hip_atomic_store(&ws.ticket2[b * ticket_stride(a.map.B, kTicket2Len)], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  uint32_t st_upd = 0;
  if (upd.B > 0) {
    // (a position with non-finite rows records nothing, whatever its entropy word holds by now)
    const float H = (lane == r && r < kb && !(bits & 2)) ? Hl : NAN;
    st_upd = update_sequence_core(upd, b, lane, r, kb, dl, H, false);
  }
  // one store of the sequence's status word, the update step's bits included (they are complete in its last lane)
  st_upd = __shfl(st_upd, src_lane);
  if (lane == 0) a.status[b] = st_seq | st_all | st_upd;
}

}  // namespace adasd
