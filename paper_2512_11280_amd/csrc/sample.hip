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

template <int DT>
__global__ void __launch_bounds__(kBlock, 6) k_sample(SampleArgs a, int S, Workspace ws) {
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

}  // namespace

hipError_t launch_sample(const SampleArgs& a, int S, const Workspace& ws, hipStream_t st) {
  if (a.map.B <= 0) return hipSuccess;
  dim3 grid(S, a.map.B), block(kBlock);
  if (a.dt == ADASD_BF16) launch_kernel(k_sample<ADASD_BF16>, grid, block, st, a, S, ws);
  else launch_kernel(k_sample<ADASD_F32>, grid, block, st, a, S, ws);
  return hipGetLastError();
}

}  // namespace adasd
