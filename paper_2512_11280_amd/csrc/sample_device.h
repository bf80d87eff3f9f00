// Device code of the Gumbel-max draws (Section 2.1.3: re-sampling from the adjusted distribution;
// generation loop of Algorithm 1: x_i ~ q_i), shared by the verification step's sampling kernel and
// by the drafting step: float keys that are upper bounds of the true keys, running winner and
// runner-up, and the float64 settlement of close calls.
#pragma once
#include "internal.h"

namespace adasd {
namespace sampling {


constexpr float kErrRel = 1.52587890625e-05f;   // 2^-16: bound on the relative error of a float p or q
constexpr float kGuard = 1.220703125e-04f;      // 2^-13: bound on the log2-domain rounding of two keys

// Word (i & 3) of a Philox block by selects: indexing the array with a run-time value would make the
// compiler move it to LDS, and that lowering reads the dispatch packet for the workgroup size.
__device__ __forceinline__ uint32_t pick_word(const U4& r, int i) {
  const uint32_t lo = (i & 1) ? r.w[1] : r.w[0], hi = (i & 1) ? r.w[3] : r.w[2];
  return (i & 2) ? hi : lo;
}

__device__ __forceinline__ bool better(float ka, int ia, float kb, int ib) {
  return ka > kb || (ka == kb && (unsigned)ia < (unsigned)ib);
}

// Running winner (key, index) and the runner-up's KEY (its index is never needed).  One lane sees its
// elements in increasing index order, so a strict comparison keeps the lowest index on equal keys;
// across lanes `better` decides.  No branches.
__device__ __forceinline__ void top2_push(Top2& t, float k, int i) {
  const bool gt = k > t.k1;
  t.k2 = fmaxf(t.k2, gt ? t.k1 : k);
  t.i1 = gt ? i : t.i1;
  t.k1 = gt ? k : t.k1;
}

__device__ __forceinline__ Top2 top2_merge(const Top2& a, const Top2& b) {
  const bool aw = better(a.k1, a.i1, b.k1, b.i1);
  Top2 r;
  r.k2 = fmaxf(fmaxf(a.k2, b.k2), aw ? b.k1 : a.k1);
  r.k1 = aw ? a.k1 : b.k1;
  r.i1 = aw ? a.i1 : b.i1;
  r.i2 = -1;
  return r;
}

template <int CTRL> __device__ __forceinline__ int dpp_rot_i(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, false);
}
template <int CTRL> __device__ __forceinline__ Top2 top2_rot(const Top2& v) {
  Top2 o;
  o.k1 = dpp_rot<CTRL>(v.k1);
  o.i1 = dpp_rot_i<CTRL>(v.i1);
  o.k2 = dpp_rot<CTRL>(v.k2);
  o.i2 = -1;
  return o;
}
__device__ __forceinline__ Top2 top2_lane(const Top2& v, int lane) {
  Top2 o;
  o.k1 = lane_value(v.k1, lane);
  o.i1 = __builtin_amdgcn_readlane(v.i1, lane);
  o.k2 = lane_value(v.k2, lane);
  o.i2 = -1;
  return o;
}
// Wave-uniform result: rotations inside the rows of 16 lanes, then the four rows through scalars.
__device__ __forceinline__ Top2 top2_wave_reduce(Top2 v) {
  v = top2_merge(v, top2_rot<0x121>(v));
  v = top2_merge(v, top2_rot<0x122>(v));
  v = top2_merge(v, top2_rot<0x124>(v));
  v = top2_merge(v, top2_rot<0x128>(v));
  return top2_merge(top2_merge(top2_lane(v, 0), top2_lane(v, 16)), top2_merge(top2_lane(v, 32), top2_lane(v, 48)));
}

// log2 of E = -ln(u), u = (word + 0.5) / 2^32, accurate to a few 1e-6 relative in E everywhere:
// near u = 1 the series of -ln(1 - t) in t = 1 - u is used (t is exact there).
__device__ __forceinline__ float log2_exponential(uint32_t word) {
  float u = fmaf((float)word, 0x1p-32f, 0x1p-33f);
  float e_direct = -0.69314718056f * lg2(u);
  float t = fmaf((float)(~word), 0x1p-32f, 0x1p-33f);
  float e_series = t * fmaf(t, fmaf(t, fmaf(t, fmaf(t, 0.2f, 0.25f), 0.33333333333f), 0.5f), 1.0f);
  float e = word >= 0xF0000000u ? e_series : e_direct;
  return lg2(e);
}

// Sampling modes of a sequence (SamplePlan::residual)
constexpr int kPlain = 0;      // the target row as it is (bonus row)
constexpr int kResidual = 1;   // max(0, p - q)
constexpr int kExclude = 2;    // the target row without one token (replacement after the loop's match test)

// Upper-bound key of one vocabulary element.
template <bool RESIDUAL>
__device__ __forceinline__ float key_ub(float zp, float zq, float cp, float cq, uint32_t word) {
  float lE = log2_exponential(word);
  if (!RESIDUAL) return fmaf(zp, kLog2e, -lE);         // log2 w = z log2 e + const
  float p = ex2(fmaf(zp, kLog2e, -cp)), q = ex2(fmaf(zq, kLog2e, -cq));
  float w = fmaxf(fmaf(kErrRel, p + q, p - q), 0.f);   // (p - q) + error bound; <= 0: certainly no mass
  return lg2(w) - lE;
}

// ---- float64 re-evaluation of one sequence by one workgroup ------------------------------------
__device__ inline double block_max_d(double v, double* sh) {
  v = wave_max(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  double t = sh[0];
#pragma unroll
  for (int w = 1; w < kWaves; ++w) t = fmax(t, sh[w]);
  return t;
}
__device__ inline double block_sum_d(double v, double* sh) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  double t = 0.0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) t += sh[w];
  return t;
}

template <int DT>
__device__ double row_lse_exact(const char* row, int V, double* sh) {
  double m = -INFINITY;
  for (int v = threadIdx.x; v < V; v += kBlock) m = fmax(m, (double)load_elem<DT>(row, v));
  m = block_max_d(m, sh);
  if (!(m > -INFINITY)) return NAN;
  double s = 0.0;
  for (int v = threadIdx.x; v < V; v += kBlock) s += exp((double)load_elem<DT>(row, v) - m);
  s = block_sum_d(s, sh);
  return m + log(s);
}

// Returns the token (all threads), -1 if the row has no finite logit.
template <int DT>
__device__ int sample_exact(const char* prow, const char* qrow, bool residual, int excluded, int V, uint32_t c1,
                            uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1, double* sh,
                            uint32_t* status_bits) {
  const double lse_p = row_lse_exact<DT>(prow, V, sh);
  if (isnan(lse_p)) {
    *status_bits |= ADASD_ST_NONFINITE;
    return -1;
  }
  double lse_q = 0.0;
  if (residual) {
    lse_q = row_lse_exact<DT>(qrow, V, sh);
    double mass = 0.0;
    for (int v = threadIdx.x; v < V; v += kBlock) {
      double w = exp((double)load_elem<DT>(prow, v) - lse_p) - exp((double)load_elem<DT>(qrow, v) - lse_q);
      if (w > 0.0) mass += w;
    }
    mass = block_sum_d(mass, sh);
    if (!(mass > 0.0)) {           // no residual mass: the token comes from the target distribution
      residual = false;
      *status_bits |= ADASD_ST_ZERO_MASS;
    }
  }
  if (excluded >= 0) {
    double mass = 0.0;
    for (int v = threadIdx.x; v < V; v += kBlock)
      if (v != excluded) mass += exp((double)load_elem<DT>(prow, v) - lse_p);
    mass = block_sum_d(mass, sh);
    if (!(mass > 0.0)) {           // everything sits on the excluded token: the target row as it is
      excluded = -1;
      *status_bits |= ADASD_ST_ZERO_MASS;
    }
  }
  double best = -INFINITY;
  int tok = 0x7fffffff;
  for (int v = threadIdx.x; v < V; v += kBlock) {
    double w = exp((double)load_elem<DT>(prow, v) - lse_p);
    if (residual) w -= exp((double)load_elem<DT>(qrow, v) - lse_q);
    if (v == excluded || !(w > 0.0)) continue;
    const U4 r = philox4x32_10((uint32_t)v >> 2, c1, c2, c3, k0, k1);
    const double u = ((double)pick_word(r, v) + 0.5) * (1.0 / 4294967296.0);
    const double key = log(w) - log(-log(u));
    if (key > best) {               // v increases per thread: the first index keeps a tie
      best = key;
      tok = v;
    }
  }
  // block argmax with lowest index on equal keys
  const double bmax = block_max_d(best, sh);
  int cand = (best == bmax && tok != 0x7fffffff) ? tok : 0x7fffffff;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) cand = min(cand, __shfl_xor(cand, off));
  __shared__ int sh_tok[kWaves];
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh_tok[threadIdx.x >> 6] = cand;
  __syncthreads();
  int t = sh_tok[0];
#pragma unroll
  for (int w = 1; w < kWaves; ++w) t = min(t, sh_tok[w]);
  return t == 0x7fffffff ? -1 : t;
}

// Element ranges of slice s as scan_slice covers them: [a0, a1) and the row's unaligned tail [b0, b1).
template <int DT>
__device__ __forceinline__ void slice_ranges(bool fast, int V, int s, int S, int& a0, int& a1, int& b0, int& b1) {
  constexpr int EPV = Elem<DT>::per_vec;
  if (fast) {
    const int nv = V / EPV, chunk = (nv + S - 1) / S, v0 = min(s * chunk, nv), v1 = min(v0 + chunk, nv);
    a0 = v0 * EPV;
    a1 = v1 * EPV;
    b0 = nv * EPV;
    b1 = (s == S - 1) ? V : b0;
  } else {
    a0 = (int)(((int64_t)s * V) / S);
    a1 = (int)(((int64_t)(s + 1) * V) / S);
    b0 = b1 = 0;
  }
}

constexpr int kMaxCand = 64;      // elements that may still win
constexpr int kMaxRescan = 8;     // slices that hold more than one of them

struct RefineShared {
  int n_cand, n_rescan;
  int cand[kMaxCand];
  int rescan[kMaxRescan];
  double key[kMaxCand], err[kMaxCand];
  int result;                     // token, or -1: too close, the whole row is needed
};

// Normaliser of a row to float64 accuracy in the arguments and one float ulp per term: sum of
// 2^(z log2 e - c) around a first value c of the normaliser, each term the hardware exponential of the
// float part of the argument times the first-order factor of the remainder.  Returns ln sum exp z.
// (the sum itself, all threads get it: column shards add theirs up before the logarithm)
template <int DT>
__device__ double row_pow2_sum_refined(const char* row, int V, double c_lse2, double* sh) {
  constexpr int EPV = Elem<DT>::per_vec;
  auto term = [&](float z) {
    const double x = (double)z * 1.44269504088896340736 - c_lse2;
    const float xf = (float)x;
    return xf > -140.f ? (double)ex2(xf) * (1.0 + (x - (double)xf) * 0.69314718055994530942) : 0.0;
  };
  const int tid = threadIdx.x;
  double acc = 0.0;
  // one workgroup walks the whole row: several vectors per thread in flight, or the latency of each
  // load is paid in full
  const int nv = (reinterpret_cast<uintptr_t>(row) & 15u) == 0 ? V / EPV : 0;
  const uint4* vp = reinterpret_cast<const uint4*>(row);
  constexpr int NB = 2;   // more would raise the register count of every kernel this is inlined into
  for (int base = 0; base < nv; base += NB * kBlock) {
    uint4 x[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) x[j] = vp[min(base + tid + j * kBlock, nv - 1)];
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      float z[EPV];
      unpack<DT>(x[j], z);
      double part = 0.0;
#pragma unroll
      for (int e = 0; e < EPV; ++e) part += term(z[e]);
      if (base + tid + j * kBlock < nv) acc += part;
    }
  }
  for (int v = nv * EPV + tid; v < V; v += kBlock) acc += term(load_elem<DT>(row, v));
  return block_sum_d(acc, sh);
}
template <int DT>
__device__ double row_lse_refined(const char* row, int V, double c_lse2, double* sh) {
  const double acc = row_pow2_sum_refined<DT>(row, V, c_lse2, sh);
  return (c_lse2 + log(acc) * 1.44269504088896340736) * 0.69314718055994530942;
}

// Collects into R.cand the elements (vocabulary indices) whose upper-bound key is at least tau, from the
// per-slice records of the scan (a slice whose runner-up also reaches tau is scanned again).  All threads
// of the workgroup call it; false: more candidates or slices than the lists hold.  col0: vocabulary index
// of the row's first element (the rows are column slices of V elements when it is not 0).
template <int DT>
__device__ bool refine_gather(const char* prow, const char* qrow, bool residual, int excluded, int V, int col0, int b,
                              int S, float tau, float cp, float cq, uint32_t c1, uint32_t c2, uint32_t c3,
                              uint32_t k0, uint32_t k1, const Workspace& ws, RefineShared& R) {
  const int tid = threadIdx.x;
  if (tid == 0) R.n_cand = R.n_rescan = 0;
  __syncthreads();
  // per-slice records: the slice's best element if it reaches tau; the slice itself if its runner-up does
  for (int j = tid; j < S; j += kBlock) {
    const Top2* src = &ws.part3[(size_t)b * kMaxSampleSplit + j];
    const float s_k1 = ld_agent(&src->k1), s_k2 = ld_agent(&src->k2);
    const int s_i1 = ld_agent(&src->i1);
    if (s_k2 >= tau) {
      const int at = atomicAdd(&R.n_rescan, 1);
      if (at < kMaxRescan) R.rescan[at] = j;
    } else if (s_k1 >= tau && s_i1 >= 0) {
      const int at = atomicAdd(&R.n_cand, 1);
      if (at < kMaxCand) R.cand[at] = s_i1;
    }
  }
  __syncthreads();
  const int n_rescan = R.n_rescan;
  if (n_rescan > kMaxRescan) return false;
  const bool fast = (reinterpret_cast<uintptr_t>(prow) & 15u) == 0 &&
                    (!residual || (reinterpret_cast<uintptr_t>(qrow) & 15u) == 0);
  for (int n = 0; n < n_rescan; ++n) {
    int lo[2], hi[2];
    slice_ranges<DT>(fast, V, R.rescan[n], S, lo[0], hi[0], lo[1], hi[1]);
    for (int part = 0; part < 2; ++part)
      for (int v = lo[part] + tid; v < hi[part]; v += kBlock) {
        const int gv = col0 + v;
        const U4 r = philox4x32_10((uint32_t)gv >> 2, c1, c2, c3, k0, k1);
        const float zp = load_elem<DT>(prow, v);
        const float k = residual ? key_ub<true>(zp, load_elem<DT>(qrow, v), cp, cq, pick_word(r, gv))
                                 : key_ub<false>(zp, 0.f, cp, cq, pick_word(r, gv));
        if (k >= tau && gv != excluded) {
          const int at = atomicAdd(&R.n_cand, 1);
          if (at < kMaxCand) R.cand[at] = gv;
        }
      }
  }
  __syncthreads();
  return R.n_cand <= kMaxCand;
}

// Settles a sequence among the elements whose upper-bound key is at least tau.  All threads of the
// workgroup call it; returns the token, or -1 if the decision needs the whole row in float64.
template <int DT>
__device__ int sample_refine(const char* prow, const char* qrow, int mode, int excluded, int V, int b, int S,
                             float tau, float cp, float cq, double lse2_p, double lse2_q, uint32_t c1,
                             uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1, const Workspace& ws,
                             double* sh_red, RefineShared& R) {
  const int tid = threadIdx.x;
  const bool residual = mode == kResidual;
  if (!refine_gather<DT>(prow, qrow, residual, excluded, V, 0, b, S, tau, cp, cq, c1, c2, c3, k0, k1, ws, R)) return -1;
  const int n_cand = R.n_cand;
  if (n_cand == 0) return -1;
  // float64 keys of the candidates.  Without a draft row the normaliser is a common shift and drops
  // out; with it both normalisers are refined first (workgroup-wide), and each key carries the bound
  // 2^-21 (p + q) / w of what their remaining error can do to ln w.
  double lse_p = 0.0, lse_q = 0.0;
  if (residual) {
    lse_p = row_lse_refined<DT>(prow, V, lse2_p, sh_red);
    lse_q = row_lse_refined<DT>(qrow, V, lse2_q, sh_red);
  }
  if (tid < n_cand) {
    const int v = R.cand[tid];
    const U4 r = philox4x32_10((uint32_t)v >> 2, c1, c2, c3, k0, k1);
    const double u = ((double)pick_word(r, v) + 0.5) * (1.0 / 4294967296.0);
    const double g = log(-log(u));
    double key, err = 0.0;
    if (residual) {
      const double p = exp((double)load_elem<DT>(prow, v) - lse_p), q = exp((double)load_elem<DT>(qrow, v) - lse_q);
      const double w = p - q;
      err = w > 0.0 ? 0x1p-21 * (p + q) / w : INFINITY;
      key = w > 0.0 ? log(w) - g : -INFINITY;
    } else {
      key = (double)load_elem<DT>(prow, v) - g;
    }
    R.key[tid] = key;
    R.err[tid] = err;
  }
  __syncthreads();
  if (tid == 0) {
    int best = 0;
    for (int c = 1; c < n_cand; ++c)
      if (R.key[c] > R.key[best] || (R.key[c] == R.key[best] && R.cand[c] < R.cand[best])) best = c;
    int result = R.cand[best];
    if (residual) {
      // final only if no other candidate can overtake within the error bounds; a candidate whose mass
      // is not certain at this accuracy sends the sequence to the whole-row path
      if (!(R.err[best] < 0.25)) result = -1;
      for (int c = 0; c < n_cand && result >= 0; ++c) {
        if (c == best) continue;
        if (!(R.err[c] < 0.25)) result = -1;
        else if (!(R.key[best] - R.err[best] > R.key[c] + R.err[c])) result = -1;
      }
    }
    R.result = result;
  }
  __syncthreads();
  return R.result;
}

}  // namespace sampling
}  // namespace adasd
