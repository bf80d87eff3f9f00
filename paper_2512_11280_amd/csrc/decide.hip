// Acceptance decisions of one round (Section 2.1.3, Section 4.4 and the verification loop of
// Algorithm 1 of the paper) and the update of the adaptive state (Section 4.3; update lines).
#include "internal.h"

namespace adasd {

namespace {

__device__ __forceinline__ double block_sum(double v, double* sh) {
  v = wave_sum(v);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) sh[wave] = v;
  __syncthreads();
  double t = 0.0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) t += sh[w];
  return t;
}

struct Kde {
  double inv2h2;   // 1 / (2 h^2)
  double log_norm; // ln(n h sqrt(2 pi)) - ln prior  (subtracted from the log kernel sum)
};

// Sample variance (n-1) of a history list and the resulting Gaussian-kernel constants.
__device__ bool kde_setup(const float* L, int n, int n_other, int bw_rule, double* sh, Kde* out) {
  double part = 0.0;
  for (int j = threadIdx.x; j < n; j += kBlock) part += (double)L[j];
  const double mean = block_sum(part, sh) / (double)n;
  part = 0.0;
  for (int j = threadIdx.x; j < n; j += kBlock) {
    double e = (double)L[j] - mean;
    part += e * e;
  }
  const double var = block_sum(part, sh) / (double)(n - 1);
  if (!(var > 0.0)) return false;
  const double factor = bw_rule == 1 ? pow((double)n, -0.2) : pow(4.0 / (3.0 * (double)n), 0.2);
  const double h = factor * sqrt(var);
  out->inv2h2 = 1.0 / (2.0 * h * h);
  const double prior = (double)n / (double)(n + n_other);
  out->log_norm = log((double)n * h * 2.50662827463100050242) - log(prior);
  return true;
}

// ln [ p(d | list) P(list) ] evaluated by one wavefront: max-shifted log-sum-exp of the kernels.
__device__ double wave_log_joint(double d, const float* L, int n, const Kde& k) {
  const int lane = threadIdx.x & 63;
  double tmax = -INFINITY;
  for (int j = lane; j < n; j += 64) {
    double e = d - (double)L[j];
    tmax = fmax(tmax, -(e * e) * k.inv2h2);
  }
  tmax = wave_max(tmax);
  float acc = 0.f;
  for (int j = lane; j < n; j += 64) {
    double e = d - (double)L[j];
    double t = -(e * e) * k.inv2h2 - tmax;            // <= 0
    acc += ex2((float)(t * 1.44269504088896340736));  // e^t; terms below 2^-126 vanish
  }
  double total = wave_sum((double)acc);
  return tmax + log(total) - k.log_norm;
}

template <int DT>
__global__ void __launch_bounds__(kBlock) k_decide(DecideArgs a, Workspace ws) {
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int K = a.map.K;
  __shared__ double sh_red[kWaves];
  __shared__ uint8_t sh_acc[ADASD_MAX_K];
  __shared__ uint32_t sh_status;
  if (tid == 0) sh_status = 0;

  int kb = K;
  uint32_t st = 0;
  if (a.map.draft_len) {
    int raw = a.map.draft_len[b];
    kb = min(max(raw, 0), K);
    if (raw != kb) st |= ADASD_ST_BAD_LENGTH;
  }

  // ---- Bayesian test set-up: both lists need enough samples and spread (else P(A|d) = 0)
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
  bool kde_on = !a.relaxed_off && nA >= min_n && nR >= min_n;
  Kde kA, kR;
  if (kde_on) {
    bool okA = kde_setup(LA, nA, nR, a.bw_rule, sh_red, &kA);
    bool okR = kde_setup(LR, nR, nA, a.bw_rule, sh_red, &kR);
    kde_on = okA && okR;
  }
  __syncthreads();

  const uint32_t seq = a.seq_id ? a.seq_id[b] : (uint32_t)b;
  const uint32_t rnd = a.round ? a.round[b] : a.round0;

  // ---- one wavefront per candidate position
  for (int i = wave; i < K; i += kWaves) {
    const size_t o = (size_t)b * K + i;
    if (i >= kb) {
      if (lane == 0) {
        if (a.H_p) a.H_p[o] = 0.f;
        a.H_q[o] = 0.f;
        a.d_js[o] = 0.f;
        if (a.p_accept) a.p_accept[o] = 0.f;
        if (a.accept_mask) a.accept_mask[o] = 0;
        sh_acc[i] = 0;
      }
      continue;
    }
    const RowResult rp = ws.rows[2 * o], rq = ws.rows[2 * o + 1];
    const bool bad = rp.bad || rq.bad;
    const double d = (double)a.d_js[o];
    double PA = 0.0;
    if (!bad && kde_on) {
      double ja = wave_log_joint(d, LA, nA, kA);
      double jr = wave_log_joint(d, LR, nR, kR);
      PA = 1.0 / (1.0 + exp(jr - ja));
    }
    if (lane != 0) continue;
    if (bad) {
      if (a.H_p) a.H_p[o] = NAN;
      a.H_q[o] = NAN;
      a.d_js[o] = NAN;
      if (a.p_accept) a.p_accept[o] = NAN;
      if (a.accept_mask) a.accept_mask[o] = 0;
      sh_acc[i] = 0;
      atomicOr(&sh_status, (uint32_t)ADASD_ST_NONFINITE);
      continue;
    }
    const U4 r = philox4x32_10(0u, (uint32_t)i, rnd, seq, a.seed_lo, a.seed_hi);
    const double u1 = ((double)(r.w[0] >> 8) + 0.5) * (1.0 / 16777216.0);
    const double u2 = ((double)(r.w[1] >> 8) + 0.5) * (1.0 / 16777216.0);
    // speculative-sampling test: accept with probability min(1, p(x)/q(x)), in the log domain
    int base = 0;
    const int x = a.draft_tokens[o];
    if (x < 0 || x >= a.map.V) {
      atomicOr(&sh_status, (uint32_t)ADASD_ST_BAD_TOKEN);
    } else {
      const char* prow = a.map.base[0] +
          ((int64_t)b * a.map.seq_stride[0] + (int64_t)i * a.map.pos_stride[0]) * Elem<DT>::bytes;
      const char* qrow = a.map.base[1] +
          ((int64_t)b * a.map.seq_stride[1] + (int64_t)i * a.map.pos_stride[1]) * Elem<DT>::bytes;
      double lp = (double)load_elem<DT>(prow, x) - rp.lse2 * kLn2;
      double lq = (double)load_elem<DT>(qrow, x) - rq.lse2 * kLn2;
      double log_ratio = lp - lq;
      if (log_ratio > 0.0) log_ratio = 0.0;
      base = log(u1) < log_ratio;   // false for NaN (both probabilities zero)
    }
    const int relaxed = a.reject_rule == 1 ? (PA >= 0.5) : (u2 < PA);
    if (a.p_accept) a.p_accept[o] = (float)PA;
    if (a.accept_mask) a.accept_mask[o] = (uint8_t)(base | (relaxed << 1));
    sh_acc[i] = (uint8_t)(base || relaxed);   // rejected only if both tests reject
  }
  __syncthreads();
  if (tid != 0) return;

  int r = kb;
  for (int i = 0; i < kb; ++i)
    if (!sh_acc[i]) {
      r = i;
      break;
    }
  a.n_accept[b] = r;
  st |= sh_status;
  SamplePlan plan;
  plan.row = r;
  plan.pad = 0;
  if (r < kb) {
    const size_t o = (size_t)b * K + r;
    const RowResult rp = ws.rows[2 * o], rq = ws.rows[2 * o + 1];
    plan.residual = 1;
    plan.valid = !(rp.bad || rq.bad);
    plan.lse2_p = rp.lse2;
    plan.lse2_q = rq.lse2;
  } else {
    plan.residual = 0;   // bonus row: Gumbel-max needs no normaliser
    plan.valid = 1;
    plan.lse2_p = 0.0;
    plan.lse2_q = 0.0;
  }
  ws.plan[b] = plan;
  a.status[b] = st;
}

// ---------------------------------------------------------------------------------------------
// Update step: one thread per sequence (at most k_max appends each).
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(64) k_update(UpdateArgs a) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= a.B) return;
  int kb = a.K;
  if (a.draft_len) kb = min(max(a.draft_len[b], 0), a.K);
  const int r = min(max(a.n_accept[b], 0), kb);
  uint32_t st = 0;
  float* LA = a.LA + (size_t)b * a.cap;
  float* LR = a.LR + (size_t)b * a.cap;
  int nA = a.nA[b], nR = a.nR[b];
  const float lo = a.d_eps, hi = 1.0f - a.d_eps;
  for (int i = 0; i < r; ++i) {
    float d = a.d_js[(size_t)b * a.K + i];
    if (d > lo && d < hi) {            // NaN fails both comparisons
      if (nA < a.cap) LA[nA++] = d;
      else st |= ADASD_ST_OVERFLOW;
    }
  }
  if (r < kb) {
    float H = a.H_q[(size_t)b * a.K + r];
    if (isfinite(H)) {
      a.ent_sum[b] += (double)H;
      a.ent_cnt[b] += 1;
    }
    float d = a.d_js[(size_t)b * a.K + r];
    if (d > lo && d < hi) {
      if (nR < a.cap) LR[nR++] = d;
      else st |= ADASD_ST_OVERFLOW;
    }
  }
  a.nA[b] = nA;
  a.nR[b] = nR;
  const int cnt = a.ent_cnt[b];
  a.T_G[b] = cnt > 0 ? (float)(a.ent_sum[b] / (double)cnt) : 0.f;
  if (a.status && st) a.status[b] |= st;
}

__global__ void __launch_bounds__(64) k_state_init(UpdateArgs a) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= a.B) return;
  a.T_G[b] = 0.f;
  a.ent_sum[b] = 0.0;
  a.ent_cnt[b] = 0;
  a.nA[b] = 0;
  a.nR[b] = 0;
}

__global__ void __launch_bounds__(256) k_zero(uint32_t* p, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = 0u;
}

}  // namespace

hipError_t launch_decide(const DecideArgs& a, const Workspace& ws, hipStream_t st) {
  if (a.map.B <= 0) return hipSuccess;
  if (a.dt == ADASD_BF16)
    hipLaunchKernelGGL(k_decide<ADASD_BF16>, dim3(a.map.B), dim3(kBlock), 0, st, a, ws);
  else
    hipLaunchKernelGGL(k_decide<ADASD_F32>, dim3(a.map.B), dim3(kBlock), 0, st, a, ws);
  return hipGetLastError();
}

hipError_t launch_update(const UpdateArgs& a, hipStream_t st) {
  if (a.B <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_update, dim3((a.B + 63) / 64), dim3(64), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_state_init(const UpdateArgs& a, hipStream_t st) {
  if (a.B <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_state_init, dim3((a.B + 63) / 64), dim3(64), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_zero(void* p, size_t bytes, hipStream_t st) {
  const size_t n = bytes / 4;
  if (n == 0) return hipSuccess;
  int blocks = (int)((n + 255) / 256);
  if (blocks > 1024) blocks = 1024;
  hipLaunchKernelGGL(k_zero, dim3(blocks), dim3(256), 0, st, (uint32_t*)p, n);
  return hipGetLastError();
}

}  // namespace adasd
