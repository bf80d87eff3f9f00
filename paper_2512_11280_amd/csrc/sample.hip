// Correction / bonus token (Section 2.1.3: re-sampling from the adjusted distribution; last lines of
// the verification step of Algorithm 1): Gumbel-max over the vocabulary with counter-based Philox
// noise, argmax_v ln w_v - ln(-ln u_v), lowest index on ties.
//
// Fast path: float keys in the log2 domain that are UPPER BOUNDS of the true keys, running top-2 per
// sequence.  The winner is final only if its lower bound beats the runner-up's upper bound;
// otherwise the workgroup that arrives last re-does the sequence in float64 (exact path).
#include "internal.h"

namespace adasd {

namespace {

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

template <int DT, int MODE>
__device__ __forceinline__ void scan_slice(const char* prow, const char* qrow, int V, int s, int S,
                                           float cp, float cq, int excluded, uint32_t c1, uint32_t c2, uint32_t c3,
                                           uint32_t k0, uint32_t k1, Top2& best, bool& poison) {
  constexpr bool RESIDUAL = MODE == kResidual;
  constexpr int EPV = Elem<DT>::per_vec;
  const int tid = threadIdx.x;
  const bool fast = (reinterpret_cast<uintptr_t>(prow) & 15u) == 0 &&
                    (!RESIDUAL || (reinterpret_cast<uintptr_t>(qrow) & 15u) == 0);
  const int nv = fast ? V / EPV : 0;
  if (fast) {
    const int chunk = (nv + S - 1) / S, v0 = min(s * chunk, nv), v1 = min(v0 + chunk, nv);
    const uint4* vp = reinterpret_cast<const uint4*>(prow);
    const uint4* vq = reinterpret_cast<const uint4*>(qrow);
    constexpr int NB = 2;                       // vectors per thread and batch, all loads in flight at once
    for (int base_v = v0; base_v < v1; base_v += NB * kBlock) {
      uint4 xp[NB], xq[NB];
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        const int idx = min(base_v + tid + j * kBlock, v1 - 1);
        xp[j] = vp[idx];
        if (RESIDUAL) xq[j] = vq[idx];
      }
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        const int idx = base_v + tid + j * kBlock;
        const bool in = idx < v1;
        float zp[EPV], zq[EPV];
        unpack<DT>(xp[j], zp);
        if (RESIDUAL) unpack<DT>(xq[j], zq);
        const int base = idx * EPV;
#pragma unroll
        for (int g = 0; g < EPV / 4; ++g) {
          const U4 r = philox4x32_10((uint32_t)(base >> 2) + g, c1, c2, c3, k0, k1);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float a = zp[4 * g + e];
            if (MODE == kPlain) poison |= in && !(a < INFINITY);   // NaN or +inf in the bonus row
            float k = key_ub<RESIDUAL>(a, RESIDUAL ? zq[4 * g + e] : 0.f, cp, cq, r.w[e]);
            const bool use = MODE == kExclude ? (in && base + 4 * g + e != excluded) : in;
            top2_push(best, use ? k : -INFINITY, base + 4 * g + e);
          }
        }
      }
    }
  }
  // elements not covered by whole aligned vectors: tail of the last slice, or the whole slice
  int e0, e1;
  if (fast) {
    e0 = nv * EPV;
    e1 = (s == S - 1) ? V : e0;
  } else {
    e0 = (int)(((int64_t)s * V) / S);
    e1 = (int)(((int64_t)(s + 1) * V) / S);
  }
  for (int v = e0 + tid; v < e1; v += kBlock) {
    const U4 r = philox4x32_10((uint32_t)v >> 2, c1, c2, c3, k0, k1);
    const float a = load_elem<DT>(prow, v);
    if (MODE == kPlain) poison |= !(a < INFINITY);
    float k = key_ub<RESIDUAL>(a, RESIDUAL ? load_elem<DT>(qrow, v) : 0.f, cp, cq, pick_word(r, v));
    top2_push(best, (MODE == kExclude && v == excluded) ? -INFINITY : k, v);
  }
}

// ---- float64 re-evaluation of one sequence by one workgroup ------------------------------------
__device__ double block_max_d(double v, double* sh) {
  v = wave_max(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  double t = sh[0];
#pragma unroll
  for (int w = 1; w < kWaves; ++w) t = fmax(t, sh[w]);
  return t;
}
__device__ double block_sum_d(double v, double* sh) {
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

template <int DT>
__global__ void __launch_bounds__(kBlock) k_sample(SampleArgs a, int S, Workspace ws) {
  warm_kernargs<sizeof(SampleArgs) + sizeof(int) + sizeof(Workspace)>();
  const int b = blockIdx.y, s = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const SamplePlan plan = ws.plan[b];
  if (!plan.valid) {
    if (s == 0 && tid == 0) a.next_token[b] = -1;   // status already carries NONFINITE
    return;
  }
  const int V = a.map.V;
  const char* prow = a.map.base[0] + ((int64_t)b * a.map.seq_stride[0] +
                                      (int64_t)plan.row * a.map.pos_stride[0]) * Elem<DT>::bytes;
  const char* qrow = a.map.base[1] + ((int64_t)b * a.map.seq_stride[1] +
                                      (int64_t)plan.row * a.map.pos_stride[1]) * Elem<DT>::bytes;
  const uint32_t c1 = (uint32_t)plan.row | (1u << 16);
  const uint32_t c2 = a.round ? a.round[b] : a.round0;
  const uint32_t c3 = a.seq_id ? a.seq_id[b] : (uint32_t)b;
  const float cp = (float)plan.lse2_p, cq = (float)plan.lse2_q;

  Top2 best{-INFINITY, -1, -INFINITY, -1};
  bool poison = false;
  if (plan.residual == kResidual)
    scan_slice<DT, kResidual>(prow, qrow, V, s, S, cp, cq, -1, c1, c2, c3, a.seed_lo, a.seed_hi, best, poison);
  else if (plan.residual == kExclude)
    scan_slice<DT, kExclude>(prow, qrow, V, s, S, cp, cq, plan.excluded, c1, c2, c3, a.seed_lo, a.seed_hi, best, poison);
  else
    scan_slice<DT, kPlain>(prow, qrow, V, s, S, cp, cq, -1, c1, c2, c3, a.seed_lo, a.seed_hi, best, poison);

  __shared__ Top2 sh_top[kWaves];
  __shared__ int sh_flag[kWaves];
  __shared__ int sh_mode;   // 0: not last, 1: last & certain, 2: last & needs the exact path
  __shared__ double sh_red[kWaves];
  best = top2_wave_reduce(best);
  const int any_poison = __any(poison);
  if (lane == 0) {
    sh_top[wave] = best;
    sh_flag[wave] = any_poison;
  }
  __syncthreads();
  if (tid == 0) {
    Top2 t = sh_top[0];
    int flag = sh_flag[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) {
      t = top2_merge(t, sh_top[w]);
      flag |= sh_flag[w];
    }
    t.i2 = flag ? -2 : -1;   // poison marker travels in the runner-up index
    Top2* dst = &ws.part3[(size_t)b * kMaxSampleSplit + s];
    st_agent(&dst->k1, t.k1); st_agent(&dst->i1, t.i1);
    st_agent(&dst->k2, t.k2); st_agent(&dst->i2, t.i2);
    publish_barrier();
    int ticket = atomicAdd(&ws.ticket3[b], 1);
    sh_mode = (ticket == S - 1) ? 1 : 0;
  }
  __syncthreads();
  if (!sh_mode) return;

  // ---- last workgroup of this sequence: fold the S partial top-2 sets
  if (wave == 0) {
    Top2 t{-INFINITY, -1, -INFINITY, -1};
    int flag = 0;
    for (int j = lane; j < S; j += 64) {
      const Top2* src = &ws.part3[(size_t)b * kMaxSampleSplit + j];
      Top2 o;
      o.k1 = ld_agent(&src->k1); o.i1 = ld_agent(&src->i1);
      o.k2 = ld_agent(&src->k2); o.i2 = ld_agent(&src->i2);
      if (o.i2 == -2) { flag = 1; o.i2 = -1; }
      t = top2_merge(t, o);
    }
    t = top2_wave_reduce(t);
    flag = __any(flag);
    if (lane == 0) {
      int mode = 1;
      if (flag) {
        mode = 3;   // NaN / +inf in the bonus row
      } else if (t.i1 < 0) {
        mode = 2;   // nothing had (certain) mass
      } else {
        float margin = kGuard;
        if (plan.residual == kResidual) {
          float p = ex2(fmaf(load_elem<DT>(prow, t.i1), kLog2e, -cp));
          float q = ex2(fmaf(load_elem<DT>(qrow, t.i1), kLog2e, -cq));
          float err = kErrRel * (p + q), w = p - q;
          // true key >= key_ub - log2((w+err)/(w-err)); for err/w < 1/2 that is < 3 log2(e) err/w
          if (!(w > 2.f * err)) mode = 2;
          else margin += 3.f * kLog2e * err / w;
        }
        if (!(t.k1 - t.k2 > margin)) mode = 2;
      }
      if (mode == 1) a.next_token[b] = t.i1;
      sh_mode = mode;
      __hip_atomic_store(&ws.ticket3[b], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  __syncthreads();
  const int mode = sh_mode;
  if (mode == 1) return;
  if (mode == 3) {
    if (tid == 0) {
      a.next_token[b] = -1;
      a.status[b] |= ADASD_ST_NONFINITE;
    }
    return;
  }
  uint32_t bits = ADASD_ST_EXACT_PATH;
  int tok = sample_exact<DT>(prow, qrow, plan.residual == kResidual,
                             plan.residual == kExclude ? plan.excluded : -1, V, c1, c2, c3, a.seed_lo,
                             a.seed_hi, sh_red, &bits);
  if (tid == 0) {
    a.next_token[b] = tok;
    a.status[b] |= bits;
  }
}

}  // namespace

hipError_t launch_sample(const SampleArgs& a, int S, const Workspace& ws, hipStream_t st) {
  if (a.map.B <= 0) return hipSuccess;
  dim3 grid(S, a.map.B), block(kBlock);
  if (a.dt == ADASD_BF16) launch_kernel(k_sample<ADASD_BF16>, grid, block, st, a, S, ws);
  else launch_kernel(k_sample<ADASD_F32>, grid, block, st, a, S, ws);
  return hipGetLastError();
}

}  // namespace adasd
