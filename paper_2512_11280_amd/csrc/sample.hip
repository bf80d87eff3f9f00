// Correction / bonus token (Section 2.1.3: re-sampling from the adjusted distribution; last lines of
// the verification step of Algorithm 1): Gumbel-max over the vocabulary with counter-based Philox
// noise, argmax_v ln w_v - ln(-ln u_v), lowest index on ties.
//
// Fast path: float keys in the log2 domain that are UPPER BOUNDS of the true keys, running top-2 per
// slice and sequence.  The winner is final only if its lower bound beats the runner-up's upper bound.
// Otherwise the workgroup that arrives last settles the sequence in float64: first among the few
// elements whose upper bound reaches the winner's lower bound (found from the per-slice records, a
// slice with two such elements is scanned again), and only if that is still too close to call, or the
// winner's mass is not certain, over the whole row (exact path).
#include "sample_device.h"

namespace adasd {

namespace {

using namespace sampling;

template <int DT, int MODE>
__device__ __forceinline__ void scan_slice(const char* prow, const char* qrow, int V, int s, int S,
                                           float cp, float cq, int excluded, int col0, uint32_t c1, uint32_t c2,
                                           uint32_t c3, uint32_t k0, uint32_t k1, Top2& best, bool& poison) {
  // col0: vocabulary index of the row's first element (0 unless the row is a column slice); indices,
  // the excluded token and the noise counters are in vocabulary indices.
  // kExclude gives a key to every finite logit but the excluded one, also to those whose probability is 0
  // in float64 (which the float64 path skips).  Such an element cannot win: this mode only runs after the
  // match test rejected the excluded token x, i.e. ln u1 >= ln p(x) with u1 < 1 - 2^-25, so the rest of the
  // row holds a mass of at least 3e-8 and some element at least 3e-8 / V of it; its key is above -50 nats
  // whatever its noise, the key of an element with p < 5e-324 below -720.
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
        const int base = col0 + idx * EPV;
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
    const int gv = col0 + v;
    const U4 r = philox4x32_10((uint32_t)gv >> 2, c1, c2, c3, k0, k1);
    const float a = load_elem<DT>(prow, v);
    if (MODE == kPlain) poison |= !(a < INFINITY);
    float k = key_ub<RESIDUAL>(a, RESIDUAL ? load_elem<DT>(qrow, v) : 0.f, cp, cq, pick_word(r, gv));
    top2_push(best, (MODE == kExclude && gv == excluded) ? -INFINITY : k, gv);
  }
}

template <int DT>
__global__ void __launch_bounds__(kBlock, 5) k_sample(SampleArgs a, int S, Workspace ws) {
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
    scan_slice<DT, kResidual>(prow, qrow, V, s, S, cp, cq, -1, 0, c1, c2, c3, a.seed_lo, a.seed_hi, best, poison);
  else if (plan.residual == kExclude)
    scan_slice<DT, kExclude>(prow, qrow, V, s, S, cp, cq, plan.excluded, 0, c1, c2, c3, a.seed_lo, a.seed_hi, best, poison);
  else
    scan_slice<DT, kPlain>(prow, qrow, V, s, S, cp, cq, -1, 0, c1, c2, c3, a.seed_lo, a.seed_hi, best, poison);

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
    int ticket = atomicAdd(&ws.ticket3[b * ticket_stride(a.map.B, kTicket3Len)], 1);
    sh_mode = (ticket == S - 1) ? 1 : 0;
  }
  __syncthreads();
  if (!sh_mode) return;

  // ---- last workgroup of this sequence: fold the S partial top-2 sets
  // modes: 1 final; 2 settle among the close candidates; 3 broken bonus row; 4 whole row in float64
  __shared__ float sh_tau;
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
        mode = 4;   // nothing had (certain) mass
      } else {
        float margin = kGuard;
        if (plan.residual == kResidual) {
          float p = ex2(fmaf(load_elem<DT>(prow, t.i1), kLog2e, -cp));
          float q = ex2(fmaf(load_elem<DT>(qrow, t.i1), kLog2e, -cq));
          float err = kErrRel * (p + q), w = p - q;
          // true key >= key_ub - log2((w+err)/(w-err)); for err/w < 1/2 that is < 3 log2(e) err/w
          if (!(w > 2.f * err)) mode = 4;
          else margin += 3.f * kLog2e * err / w;
        }
        // an element whose upper bound stays below the winner's lower bound cannot be the true winner
        if (mode == 1 && !(t.k1 - t.k2 > margin)) {
          mode = 2;
          sh_tau = t.k1 - margin;
        }
      }
      if (mode == 1) a.next_token[b] = t.i1;
      sh_mode = mode;
      __hip_atomic_store(&ws.ticket3[b * ticket_stride(a.map.B, kTicket3Len)], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  __syncthreads();
  int mode = sh_mode;
  if (mode == 1) return;
  if (mode == 3) {
    if (tid == 0) {
      a.next_token[b] = -1;
      a.status[b] |= ADASD_ST_NONFINITE;
    }
    return;
  }
  uint32_t bits = ADASD_ST_EXACT_PATH;
  const int excluded = plan.residual == kExclude ? plan.excluded : -1;
  int tok = -1;
  if (mode == 2) {
    __shared__ RefineShared sh_refine;
    tok = sample_refine<DT>(prow, qrow, plan.residual, excluded, V, b, S, sh_tau, cp, cq, plan.lse2_p,
                            plan.lse2_q, c1, c2, c3, a.seed_lo, a.seed_hi, ws, sh_red, sh_refine);
  }
  if (tok < 0)
    tok = sample_exact<DT>(prow, qrow, plan.residual == kResidual, excluded, V, c1, c2, c3, a.seed_lo,
                           a.seed_hi, sh_red, &bits);
  if (tid == 0) {
    a.next_token[b] = tok;
    a.status[b] |= bits;
  }
}

// ---------------------------------------------------------------------------------------------
// Column-sharded sampling.  Every holder scans its columns under the plan of the (replicated) decision
// stage and exports one record per sequence (best key, its vocabulary index, runner-up key, margin of
// the best); the records of all holders give the winner, or a threshold below which nothing can win;
// the holders then export the few elements above it and the refined normaliser sums of their columns,
// and the float64 keys decide.
// ---------------------------------------------------------------------------------------------
constexpr int kShardCand = 8;          // candidates a holder exports per sequence
struct ShardCand {                     // 128 bytes
  double sum_p, sum_q;                 // sum of 2^(z log2 e - c) over the holder's columns, c = the plan's normalisers
  int32_t n, flags;                    // flags: 1 more candidates than the record holds, 2 the sums are float64-exact
  struct Cand { int32_t idx; float zp, zq; } c[kShardCand];
  int32_t pad[2];
};
static_assert(sizeof(ShardCand) == 128, "exchange record of the sharded refinement");

template <int DT>
__global__ void __launch_bounds__(kBlock, 5) k_shard_scan(SampleArgs a, int S, int col0, Workspace ws) {
  const int b = blockIdx.y, s = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const SamplePlan plan = ws.plan[b];
  if (!plan.valid) return;
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
    scan_slice<DT, kResidual>(prow, qrow, V, s, S, cp, cq, -1, col0, c1, c2, c3, a.seed_lo, a.seed_hi, best, poison);
  else if (plan.residual == kExclude)
    scan_slice<DT, kExclude>(prow, qrow, V, s, S, cp, cq, plan.excluded, col0, c1, c2, c3, a.seed_lo, a.seed_hi, best, poison);
  else
    scan_slice<DT, kPlain>(prow, qrow, V, s, S, cp, cq, -1, col0, c1, c2, c3, a.seed_lo, a.seed_hi, best, poison);
  __shared__ Top2 sh_top[kWaves];
  __shared__ int sh_flag[kWaves];
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
    t.i2 = flag ? -2 : -1;
    ws.part3[(size_t)b * kMaxSampleSplit + s] = t;      // read by the next kernel
  }
}

// One wavefront per sequence: the holder's record (k1, index, k2, margin of its best element).
template <int DT>
__global__ void __launch_bounds__(kBlock) k_shard_fold_top(SampleArgs a, int S, int col0, Workspace ws, float4* out) {
  const int lane = threadIdx.x & 63, b = blockIdx.x * kWaves + (threadIdx.x >> 6);
  if (b >= a.map.B) return;
  const SamplePlan plan = ws.plan[b];
  if (!plan.valid) {
    if (lane == 0) out[b] = make_float4(-INFINITY, __int_as_float(-1), -INFINITY, 0.f);
    return;
  }
  Top2 t{-INFINITY, -1, -INFINITY, -1};
  int flag = 0;
  for (int j = lane; j < S; j += 64) {
    Top2 o = ws.part3[(size_t)b * kMaxSampleSplit + j];
    if (o.i2 == -2) { flag = 1; o.i2 = -1; }
    t = top2_merge(t, o);
  }
  t = top2_wave_reduce(t);
  flag = __any(flag);
  if (lane != 0) return;
  float margin = 0.f;
  if (t.i1 >= 0 && plan.residual == kResidual) {
    const char* prow = a.map.base[0] + ((int64_t)b * a.map.seq_stride[0] +
                                        (int64_t)plan.row * a.map.pos_stride[0]) * Elem<DT>::bytes;
    const char* qrow = a.map.base[1] + ((int64_t)b * a.map.seq_stride[1] +
                                        (int64_t)plan.row * a.map.pos_stride[1]) * Elem<DT>::bytes;
    const float p = ex2(fmaf(load_elem<DT>(prow, t.i1 - col0), kLog2e, -(float)plan.lse2_p));
    const float q = ex2(fmaf(load_elem<DT>(qrow, t.i1 - col0), kLog2e, -(float)plan.lse2_q));
    const float err = kErrRel * (p + q), w = p - q;
    margin = (w > 2.f * err) ? 3.f * kLog2e * err / w : INFINITY;     // INFINITY: the mass of the best is not certain
  }
  out[b] = make_float4(t.k1, __int_as_float(flag ? -2 : t.i1), t.k2, margin);
}

// Replicated.  One wavefront per sequence, one lane per holder: the winner if it is certain, else the
// provisional winner and the threshold tau that a candidate's upper-bound key has to reach.
__global__ void __launch_bounds__(kBlock) k_shard_pick(int B, int G, const float4* top_all, Workspace ws,
                                                       int32_t* next_token, uint32_t* status, float* tau_out) {
  const int lane = threadIdx.x & 63, b = blockIdx.x * kWaves + (threadIdx.x >> 6);
  if (b >= B) return;
  const SamplePlan plan = ws.plan[b];
  float4 rec = make_float4(-INFINITY, __int_as_float(-1), -INFINITY, 0.f);
  if (lane < G) rec = top_all[(size_t)lane * B + b];
  const int idx = __float_as_int(rec.y);
  const int poison = __any(idx == -2);
  Top2 t{rec.x, idx < 0 ? -1 : idx, rec.z, -1};
  if (idx < 0) t.k1 = -INFINITY;
  t = top2_wave_reduce(t);
  const unsigned long long owner = __ballot(t.i1 >= 0 && idx == t.i1);
  const float margin_owner = __shfl(rec.w, owner ? __ffsll((long long)owner) - 1 : 0);
  if (lane != 0) return;
  float tau = INFINITY;                 // nothing to refine
  if (!plan.valid) {
    next_token[b] = -1;                 // the status already says why
  } else if (poison) {
    next_token[b] = -1;
    status[b] |= ADASD_ST_NONFINITE;
  } else if (t.i1 < 0 || !(margin_owner < INFINITY)) {
    next_token[b] = t.i1;               // no element with certain mass: this path cannot settle it
    status[b] |= ADASD_ST_UNSETTLED;
  } else {
    const float margin = kGuard + margin_owner;
    next_token[b] = t.i1;
    if (!(t.k1 - t.k2 > margin)) tau = t.k1 - margin;
  }
  tau_out[b] = tau;
}

// One workgroup per sequence still open (finite tau): the holder's candidates and refined sums.
template <int DT>
__global__ void __launch_bounds__(kBlock) k_shard_refine(SampleArgs a, int S, int col0, const float* tau_in, int exact,
                                                         Workspace ws, ShardCand* out) {
  const int b = blockIdx.x, tid = threadIdx.x;
  const float tau = tau_in[b];
  ShardCand* rec = out + b;
  if (!(tau < INFINITY)) {
    if (tid == 0) {
      rec->sum_p = rec->sum_q = 0.0;
      rec->n = rec->flags = 0;
    }
    return;
  }
  const SamplePlan plan = ws.plan[b];
  const int V = a.map.V;
  const char* prow = a.map.base[0] + ((int64_t)b * a.map.seq_stride[0] +
                                      (int64_t)plan.row * a.map.pos_stride[0]) * Elem<DT>::bytes;
  const char* qrow = a.map.base[1] + ((int64_t)b * a.map.seq_stride[1] +
                                      (int64_t)plan.row * a.map.pos_stride[1]) * Elem<DT>::bytes;
  const uint32_t c1 = (uint32_t)plan.row | (1u << 16);
  const uint32_t c2 = a.round ? a.round[b] : a.round0;
  const uint32_t c3 = a.seq_id ? a.seq_id[b] : (uint32_t)b;
  const bool residual = plan.residual == kResidual;
  __shared__ RefineShared R;
  __shared__ double sh_red[kWaves];
  const bool ok = refine_gather<DT>(prow, qrow, residual, plan.residual == kExclude ? plan.excluded : -1, V, col0, b, S,
                                    tau, (float)plan.lse2_p, (float)plan.lse2_q, c1, c2, c3, a.seed_lo, a.seed_hi, ws, R);
  double sum_p = 0.0, sum_q = 0.0;
  if (residual && exact) {           // every term in float64 (a second attempt after overlapping bounds)
    double ap = 0.0, aq = 0.0;
    for (int v = tid; v < V; v += kBlock) {
      ap += exp((double)load_elem<DT>(prow, v) - plan.lse2_p * 0.69314718055994530942);
      aq += exp((double)load_elem<DT>(qrow, v) - plan.lse2_q * 0.69314718055994530942);
    }
    sum_p = block_sum_d(ap, sh_red);
    sum_q = block_sum_d(aq, sh_red);
  } else if (residual) {
    sum_p = row_pow2_sum_refined<DT>(prow, V, plan.lse2_p, sh_red);
    sum_q = row_pow2_sum_refined<DT>(qrow, V, plan.lse2_q, sh_red);
  }
  const int n = R.n_cand;
  if (tid == 0) {
    rec->sum_p = sum_p;
    rec->sum_q = sum_q;
    rec->n = min(n, kShardCand);
    rec->flags = ((!ok || n > kShardCand) ? 1 : 0) | (exact ? 2 : 0);
  }
  if (tid < min(n, kShardCand)) {
    const int gv = R.cand[tid];
    rec->c[tid].idx = gv;
    rec->c[tid].zp = load_elem<DT>(prow, gv - col0);
    rec->c[tid].zq = residual ? load_elem<DT>(qrow, gv - col0) : 0.f;
  }
}

// Replicated.  One wavefront per sequence: float64 keys of all holders' candidates; the best is final if
// no other can overtake it within the error bounds of the refined normalisers.
__global__ void __launch_bounds__(kBlock) k_shard_settle(SampleArgs a, int G, float* tau_in, const ShardCand* all,
                                                         Workspace ws) {
  const int lane = threadIdx.x & 63, b = blockIdx.x * kWaves + (threadIdx.x >> 6), B = a.map.B;
  if (b >= B) return;
  if (!(tau_in[b] < INFINITY)) return;
  const SamplePlan plan = ws.plan[b];
  const bool residual = plan.residual == kResidual;
  const uint32_t c1 = (uint32_t)plan.row | (1u << 16);
  const uint32_t c2 = a.round ? a.round[b] : a.round0;
  const uint32_t c3 = a.seq_id ? a.seq_id[b] : (uint32_t)b;
  double sp = 0.0, sq = 0.0;
  int overflow = 0, total = 0, exact = 2;
  for (int g = 0; g < G; ++g) {                 // same order on every replica
    const ShardCand* r = all + (size_t)g * B + b;
    sp += r->sum_p;
    sq += r->sum_q;
    overflow |= r->flags & 1;
    exact &= r->flags;
    total += r->n;
  }
  // what the remaining error of the normalisers can do to ln w, per unit of (p + q) / w: one float ulp
  // per term of the refined sums, rounding of float64 sums over the vocabulary for the exact ones
  const double bound = exact ? 0x1p-40 : 0x1p-21;
  const double lse_p = residual ? (plan.lse2_p + log(sp) * 1.44269504088896340736) * 0.69314718055994530942 : 0.0;
  const double lse_q = residual ? (plan.lse2_q + log(sq) * 1.44269504088896340736) * 0.69314718055994530942 : 0.0;
  // candidate number `lane`, `lane + 64`, ... in holder order; float64 key of one of them
  auto key_of = [&](const ShardCand::Cand& e, double* err, uint32_t* word) {
    const int v = e.idx;
    const U4 w4 = philox4x32_10((uint32_t)v >> 2, c1, c2, c3, a.seed_lo, a.seed_hi);
    *word = pick_word(w4, v);
    const double u = ((double)*word + 0.5) * (1.0 / 4294967296.0);
    const double gn = log(-log(u));
    *err = 0.0;
    if (!residual) return (double)e.zp - gn;
    const double p = exp((double)e.zp - lse_p), q = exp((double)e.zq - lse_q);
    const double w = p - q;
    *err = w > 0.0 ? bound * (p + q) / w : INFINITY;
    return w > 0.0 ? log(w) - gn : -INFINITY;
  };
  // pass 1: the best key (lowest index among equal ones), with the inputs it was formed from
  double best_key = -INFINITY, best_err = 0.0;
  int best_idx = 0x7fffffff, uncertain = 0;
  float best_zp = 0.f, best_zq = 0.f;
  uint32_t best_word = 0u;
  int seen = 0;
  for (int g = 0; g < G; ++g) {
    const ShardCand* r = all + (size_t)g * B + b;
    for (int c = 0; c < r->n; ++c, ++seen) {
      if ((seen & 63) != lane) continue;
      double err;
      uint32_t word;
      const double key = key_of(r->c[c], &err, &word);
      if (residual && !(err < 0.25)) uncertain = 1;
      const int v = r->c[c].idx;
      if (key > best_key || (key == best_key && v < best_idx)) {
        best_key = key;
        best_err = err;
        best_idx = v;
        best_zp = r->c[c].zp;
        best_zq = r->c[c].zq;
        best_word = word;
      }
    }
  }
  double wk = best_key;
  int wi = best_idx;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const double ok = __shfl_xor(wk, off);
    const int oi = __shfl_xor(wi, off);
    if (ok > wk || (ok == wk && oi < wi)) { wk = ok; wi = oi; }
  }
  const unsigned long long owner_mask = __ballot(best_idx == wi && best_key == wk);
  const int owner = owner_mask ? __ffsll((long long)owner_mask) - 1 : 0;
  const double werr = __shfl(best_err, owner);
  const float wzp = __shfl(best_zp, owner), wzq = __shfl(best_zq, owner);
  const uint32_t wword = (uint32_t)__shfl((int)best_word, owner);
  // pass 2: the largest upper end among the others.  A candidate formed from the very same logits and the
  // very same noise word as the winner has the winner's key whatever the normalisers are: an exact tie,
  // which the lower index wins, not a close call.
  double others = -INFINITY;
  seen = 0;
  for (int g = 0; g < G; ++g) {
    const ShardCand* r = all + (size_t)g * B + b;
    for (int c = 0; c < r->n; ++c, ++seen) {
      if ((seen & 63) != lane || r->c[c].idx == wi) continue;
      double err;
      uint32_t word;
      const double key = key_of(r->c[c], &err, &word);
      if (word == wword && r->c[c].zp == wzp && r->c[c].zq == wzq) continue;
      others = fmax(others, key + err);
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) others = fmax(others, __shfl_xor(others, off));
  uncertain = __any(uncertain);
  if (lane != 0) return;
  if (total == 0 || overflow || uncertain || wi == 0x7fffffff || (residual && !(wk - werr > others))) {
    // the provisional token of the pick stage stays; tau stays finite, so another refine + settle
    // with exact sums can still close it
    a.status[b] |= ADASD_ST_UNSETTLED;
  } else {
    a.next_token[b] = wi;
    a.status[b] = (a.status[b] & ~(uint32_t)ADASD_ST_UNSETTLED) | ADASD_ST_EXACT_PATH;
    tau_in[b] = INFINITY;
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

hipError_t launch_shard_sample(const SampleArgs& a, int S, int col0, const Workspace& ws, float4* top_out, hipStream_t st) {
  if (a.map.B <= 0) return hipSuccess;
  const dim3 grid(S, a.map.B), block(kBlock), fold((a.map.B + kWaves - 1) / kWaves);
  if (a.dt == ADASD_BF16) {
    launch_kernel(k_shard_scan<ADASD_BF16>, grid, block, st, a, S, col0, ws);
    launch_kernel(k_shard_fold_top<ADASD_BF16>, fold, block, st, a, S, col0, ws, top_out);
  } else {
    launch_kernel(k_shard_scan<ADASD_F32>, grid, block, st, a, S, col0, ws);
    launch_kernel(k_shard_fold_top<ADASD_F32>, fold, block, st, a, S, col0, ws, top_out);
  }
  return hipGetLastError();
}

hipError_t launch_shard_pick(int B, int G, const float4* top_all, const Workspace& ws, int32_t* next_token,
                             uint32_t* status, float* tau_out, hipStream_t st) {
  if (B <= 0) return hipSuccess;
  launch_kernel(k_shard_pick, dim3((B + kWaves - 1) / kWaves), dim3(kBlock), st, B, G, top_all, ws, next_token, status, tau_out);
  return hipGetLastError();
}

hipError_t launch_shard_refine(const SampleArgs& a, int S, int col0, const float* tau, int exact, const Workspace& ws,
                               void* cand_out, hipStream_t st) {
  if (a.map.B <= 0) return hipSuccess;
  if (a.dt == ADASD_BF16)
    launch_kernel(k_shard_refine<ADASD_BF16>, dim3(a.map.B), dim3(kBlock), st, a, S, col0, tau, exact, ws, static_cast<ShardCand*>(cand_out));
  else
    launch_kernel(k_shard_refine<ADASD_F32>, dim3(a.map.B), dim3(kBlock), st, a, S, col0, tau, exact, ws, static_cast<ShardCand*>(cand_out));
  return hipGetLastError();
}

hipError_t launch_shard_settle(const SampleArgs& a, int G, float* tau, const void* cand_all, const Workspace& ws,
                               hipStream_t st) {
  if (a.map.B <= 0) return hipSuccess;
  launch_kernel(k_shard_settle, dim3((a.map.B + kWaves - 1) / kWaves), dim3(kBlock), st, a, G, tau,
                static_cast<const ShardCand*>(cand_all), ws);
  return hipGetLastError();
}

}  // namespace adasd
