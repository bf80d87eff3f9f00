// The drafting calls of the generation loop of Algorithm 1, each ONE launch and one pass over the
// logits: entropy of the draft row (Appendix A), stop rule H(q_i) > T_G (Section 4.3) and, for
// adasd_draft_step, the token x_i ~ q_i.  The Gumbel-max key of an element, ln q_v - ln(-ln u_v),
// differs from z_v - ln(-ln u_v) only by the row's normaliser, so the argmax needs no second pass: the
// scan forms the entropy sums and the keys from the same registers.  The workgroup that takes the
// last ticket of a row folds the row's slice records and settles close calls of the argmax in float64.
#include "sample_device.h"
#include "stats_device.h"

namespace adasd {

namespace {

using namespace sampling;

template <int DT>
__device__ __forceinline__ void key_push(Top2& best, float z, bool in, int index, uint32_t word) {
  const float k = key_ub<false>(z, 0.f, 0.f, 0.f, word);
  top2_push(best, in ? k : -INFINITY, index);
}

// Fold of the slice records of one row as fold_row does it, read with agent-scope loads: the records
// were written by other workgroups of the same kernel.
__device__ __forceinline__ RowResult fold_row_shared(const Workspace& ws, int rho, int S) {
  const int lane = threadIdx.x & 63;
  Lse t = lse_empty();
  if (lane < S) {
    const float* p = reinterpret_cast<const float*>(&ws.part1[(size_t)rho * kMaxSplit + lane]);
    t = Lse{ld_agent(p), ld_agent(p + 1), ld_agent(p + 2)};
  }
  const float M = wave_max_f(t.m), d = t.m - M, f = ex2(d);
  const float sw = wave_sum_f(t.s * f), uw = wave_sum_f((t.u + d * t.s) * f);
  const bool ok = (sw > 0.f) && (sw < INFINITY) && (fabsf(uw) < INFINITY) && (M > kNegHuge) && (M < INFINITY);
  RowResult res;
  if (ok) {
    const double l2s = log2_acc(sw);
    res.lse2 = (double)M + l2s;
    res.H = fmaxf((float)(kLn2 * (l2s - (double)uw / (double)sw)), 0.f);   // (a one-hot row: a few 1e-8 either side of 0)
    res.bad = 0;
  } else {
    res.lse2 = NAN;
    res.H = NAN;
    res.bad = 1;
  }
  return res;
}

// One launch per drafting call, grid (slices, rows).  Every workgroup scans its slice; the one that
// takes the last ticket of a row folds the row's slice records: entropy and stop flag, and with DRAW
// the token (a winner that does not lead by more than the rounding guard is settled in float64).
template <int DT, int NB, bool DRAW>   // NB: vectors per thread and batch
__global__ void __launch_bounds__(kBlock) k_draft(RowMap map, int S, Workspace ws, DraftOut dout, DraftDraw dr) {
  warm_kernargs<sizeof(RowMap) + sizeof(int) + sizeof(Workspace) + sizeof(DraftOut) + sizeof(DraftDraw)>();
  constexpr int EPV = Elem<DT>::per_vec;
  const int rho = blockIdx.y, s = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const RowRef r = locate_row<DT>(map, rho);
  if (!r.active) {
    if (s == 0 && tid == 0) {
      dout.H_out[rho] = 0.f;
      if (dout.stop_out) dout.stop_out[rho] = 0;
      if (DRAW) {
        dr.token_out[rho] = -1;
        if (dr.status) dr.status[rho] = 0;
      }
    }
    return;
  }
  const int V = map.V;
  const uint32_t c1 = dr.step | (2u << 16);
  const uint32_t c2 = DRAW ? (dr.round ? dr.round[rho] : dr.round0) : 0u;
  const uint32_t c3 = DRAW ? (dr.seq_id ? dr.seq_id[rho] : (uint32_t)rho) : 0u;

  float M = kNegHuge, s0 = 0.f, s1 = 0.f, u0 = 0.f, u1 = 0.f;
  Lse extra = lse_empty();
  Top2 best{-INFINITY, -1, -INFINITY, -1};
  if (aligned16(r.ptr)) {
    const int nv = V / EPV;
    const int chunk = (nv + S - 1) / S, v0 = min(s * chunk, nv), v1 = min(v0 + chunk, nv);
    const uint4* vec = reinterpret_cast<const uint4*>(r.ptr);
    const uint4 neutral = neutral_vec<DT>();
    for (int base = v0; base < v1; base += NB * kBlock) {
      uint4 v[NB];
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        const int idx = base + tid + j * kBlock;
        const bool in = idx < v1;
        const uint4 x = vec[in ? idx : v1 - 1];
        v[j] = make_uint4(in ? x.x : neutral.x, in ? x.y : neutral.y, in ? x.z : neutral.z, in ? x.w : neutral.w);
      }
      const float mb = wave_max_f(vecs_max<DT, NB>(v));
      if (mb > M) {                       // wave-uniform
        const float d = M - mb, f = ex2(d);
        u0 = (u0 + d * s0) * f;
        u1 = (u1 + d * s1) * f;
        s0 *= f;
        s1 *= f;
        M = mb;
      }
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        lse_accum<DT>(v[j], M, s0, s1, u0, u1);
        if (!DRAW) continue;
        const int idx = base + tid + j * kBlock;
        const bool in = idx < v1;
        if (!in) continue;        // whole wavefronts beyond the slice skip the key arithmetic
        float z[EPV];
        unpack<DT>(v[j], z);
#pragma unroll
        for (int g = 0; g < EPV / 4; ++g) {
          const U4 w = philox4x32_10((uint32_t)((idx * EPV) >> 2) + g, c1, c2, c3, dr.seed_lo, dr.seed_hi);
#pragma unroll
          for (int e = 0; e < 4; ++e) key_push<DT>(best, z[4 * g + e], in, idx * EPV + 4 * g + e, w.w[e]);
        }
      }
    }
    if (s == S - 1 && tid == 0)
      for (int v = nv * EPV; v < V; ++v) {
        const float z = load_elem<DT>(r.ptr, v);
        lse_push(extra, z);
        if (DRAW) {
          const U4 w = philox4x32_10((uint32_t)v >> 2, c1, c2, c3, dr.seed_lo, dr.seed_hi);
          key_push<DT>(best, z, true, v, pick_word(w, v));
        }
      }
  } else {
    const int e0 = (int)(((int64_t)s * V) / S), e1 = (int)(((int64_t)(s + 1) * V) / S);
    for (int v = e0 + tid; v < e1; v += kBlock) {
      const float z = load_elem<DT>(r.ptr, v);
      lse_push(extra, z);
      if (DRAW) {
        const U4 w = philox4x32_10((uint32_t)v >> 2, c1, c2, c3, dr.seed_lo, dr.seed_hi);
        key_push<DT>(best, z, true, v, pick_word(w, v));
      }
    }
  }
  // wavefront fold: common reference, then plain sums; winner and runner-up
  Lse st = lse_merge(Lse{M, s0 + s1, u0 + u1}, extra);
  {
    const float Mw = wave_max_f(st.m), d = st.m - Mw, f = ex2(d);
    const float sw = wave_sum_f(st.s * f), uw = wave_sum_f((st.u + d * st.s) * f);
    st = Lse{Mw, sw, uw};
  }
  if (DRAW) best = top2_wave_reduce(best);

  __shared__ Lse sh[kWaves];
  __shared__ Top2 sh_top[kWaves];
  __shared__ int sh_mode;      // 0 not the last workgroup of the row; 1 final; 2 settle among the close candidates;
                               // 3 broken row; 4 whole row in float64
  __shared__ float sh_tau;
  __shared__ double sh_red[kWaves];
  if (lane == 0) {
    sh[wave] = st;
    if (DRAW) sh_top[wave] = best;
  }
  __syncthreads();
  if (tid == 0) {
    Lse t = sh[0];
    Top2 b = sh_top[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) {
      t = lse_merge(t, sh[w]);
      if (DRAW) b = top2_merge(b, sh_top[w]);
    }
    float* p1 = reinterpret_cast<float*>(&ws.part1[(size_t)rho * kMaxSplit + s]);
    st_agent(p1, t.m); st_agent(p1 + 1, t.s); st_agent(p1 + 2, t.u);
    if (DRAW) {
      Top2* dst = &ws.part3[(size_t)rho * kMaxSampleSplit + s];
      st_agent(&dst->k1, b.k1); st_agent(&dst->i1, b.i1); st_agent(&dst->k2, b.k2);
    }
    publish_barrier();
    const int ticket = atomicAdd(&ws.ticket1[rho * ticket_stride(map.B, kTicket1Len)], 1);
    sh_mode = ticket == S - 1 ? 1 : 0;
  }
  __syncthreads();
  if (!sh_mode) return;

  // ---- last workgroup of the row
  if (wave == 0) {
    const RowResult res = fold_row_shared(ws, rho, S);
    Top2 t{-INFINITY, -1, -INFINITY, -1};
    if (DRAW) {
      if (lane < S) {
        const Top2* src = &ws.part3[(size_t)rho * kMaxSampleSplit + lane];
        t.k1 = ld_agent(&src->k1); t.i1 = ld_agent(&src->i1); t.k2 = ld_agent(&src->k2);
      }
      t = top2_wave_reduce(t);
    }
    if (lane == 0) {
      ws.rows[rho] = res;
      dout.H_out[rho] = res.H;
      if (dout.stop_out) {
        const bool over = dout.T_G ? (res.H > dout.T_G[rho]) : false;
        dout.stop_out[rho] = (uint8_t)(over || dout.force_stop || res.bad);
      }
      int mode = 1;
      if (DRAW) {
        if (res.bad) mode = 3;
        else if (t.i1 < 0) mode = 4;
        else if (!(t.k1 - t.k2 > kGuard)) {
          mode = 2;
          sh_tau = t.k1 - kGuard;
        }
        if (mode == 1) {
          dr.token_out[rho] = t.i1;
          if (dr.status) dr.status[rho] = 0;
        } else if (mode == 3) {
          dr.token_out[rho] = -1;
          if (dr.status) dr.status[rho] = ADASD_ST_NONFINITE;
        }
      }
      sh_mode = mode;
      __hip_atomic_store(&ws.ticket1[rho * ticket_stride(map.B, kTicket1Len)], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  if (!DRAW) return;
  __syncthreads();
  const int mode = sh_mode;
  if (mode == 1 || mode == 3) return;
  uint32_t bits = ADASD_ST_EXACT_PATH;
  int tok = -1;
  if (mode == 2) {
    __shared__ RefineShared sh_refine;
    tok = sample_refine<DT>(r.ptr, nullptr, kPlain, -1, V, rho, S, sh_tau, 0.f, 0.f, 0.0, 0.0, c1, c2, c3,
                            dr.seed_lo, dr.seed_hi, ws, sh_red, sh_refine);
  }
  if (tok < 0)
    tok = sample_exact<DT>(r.ptr, nullptr, false, -1, V, c1, c2, c3, dr.seed_lo, dr.seed_hi, sh_red, &bits);
  if (tid == 0) {
    dr.token_out[rho] = tok;
    if (dr.status) dr.status[rho] = bits;
  }
}

}  // namespace

// Slices per row of a drafting call: one vector per thread and slice where the row is long enough
// (the key arithmetic is the cost of the scan, so no thread should carry a second, mostly empty batch),
// fewer when there are many rows.
int pick_draft_split(int rows, int V, int dt) {
  const int nv = V / (dt == ADASD_BF16 ? 8 : 4);
  int S = (nv + kBlock - 1) / kBlock;
  if (S > kMaxSplit) S = kMaxSplit;
  while (S > 1 && (int64_t)S * rows > 16384) S = (S + 1) / 2;
  return S < 1 ? 1 : S;
}

hipError_t launch_draft_step(const RowMap& map, int dt, int S, const Workspace& ws, const DraftOut& dout,
                             const DraftDraw* draw, hipStream_t st) {
  if (map.B <= 0) return hipSuccess;
  const dim3 grid(S, map.B), block(kBlock);
  const int nv = map.V / (dt == ADASD_BF16 ? 8 : 4);
  const int chunk = (nv + S - 1) / S, per_thread = (chunk + kBlock - 1) / kBlock;
  const int nb = per_thread > 1 ? 2 : 1;
  const DraftDraw dr = draw ? *draw : DraftDraw{};
#define ADASD_DRAFT_CASE(DTV, NBV)                                                                      \
  if (dt == DTV && nb == NBV) {                                                                         \
    if (draw) launch_kernel((k_draft<DTV, NBV, true>), grid, block, st, map, S, ws, dout, dr);          \
    else launch_kernel((k_draft<DTV, NBV, false>), grid, block, st, map, S, ws, dout, dr);              \
  }
  ADASD_DRAFT_CASE(ADASD_BF16, 1) ADASD_DRAFT_CASE(ADASD_BF16, 2)
  ADASD_DRAFT_CASE(ADASD_F32, 1) ADASD_DRAFT_CASE(ADASD_F32, 2)
#undef ADASD_DRAFT_CASE
  return hipGetLastError();
}

}  // namespace adasd
