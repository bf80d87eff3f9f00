// Vocabulary-wide statistics: softmax normalisers + Shannon entropy of every row (Appendix A of
// the paper) and the Jensen-Shannon distance of every (target, draft) row pair (Section 2.2).
//
// Two-kernel split-vocabulary form: each row is cut into S slices, one workgroup per slice.  The
// first kernel leaves one (reference, sum, sum x*e) per row and slice in the workspace; every workgroup
// of the second kernel folds the slices of its two rows itself (same code, same order, so the same
// normalisers everywhere) and leaves one partial JS sum per position and slice, which the decision
// kernel adds up in slice order.  Kernel boundaries are the only synchronisation.
#include <type_traits>

#include "stats_device.h"

namespace adasd {

namespace {

template <int DT>
__device__ __forceinline__ void lse_push_vec(Lse& st, const uint4& q) {
  constexpr int N = Elem<DT>::per_vec;
  float z[N];
  unpack<DT>(q, z);
  float vmax = z[0];
#pragma unroll
  for (int e = 1; e < N; ++e) vmax = fmaxf(vmax, z[e]);
  lse_raise(st, vmax * kLog2e);   // NaN-free max: a NaN logit surfaces through lse_add instead
#pragma unroll
  for (int e = 0; e < N; ++e) lse_add(st, z[e]);
}

// ---------------------------------------------------------------------------------------------
// Pass 1: partial (m, s, u) of one slice of one row.
// ---------------------------------------------------------------------------------------------
template <int DT, int kRowBatch>   // kRowBatch: vectors per thread and batch
__global__ void __launch_bounds__(kBlock, 8)   // 64 registers: eight wavefronts per SIMD, 4096 workgroups in exactly two rounds
k_rowstats(RowMap map, int S, Workspace ws) {
  warm_kernargs<sizeof(RowMap) + sizeof(int) + sizeof(Workspace)>();
  constexpr int EPV = Elem<DT>::per_vec;
  const int s = blockIdx.x, tid = threadIdx.x;
  int rho = blockIdx.y;
  if (map.K > 0) {
    const int p = position_of_slot(map, blockIdx.y >> 1);
    if (p < 0) return;
    rho = 2 * p + (blockIdx.y & 1);
  }
  const RowRef r = locate_row<DT>(map, rho);
  if (!r.active) return;
  const int V = map.V;
  // Vector path: batches of kRowBatch vectors per thread are loaded up front (all loads of a batch in
  // flight at once), the batch's largest finite logit becomes the wavefront's reference if it exceeds
  // the current one, and every element then costs one exp and a handful of multiply-adds: no
  // per-element rescaling, no divergent branch.  (Working through a batch vector by vector as the loads
  // come back, with a reference from the first of them, measured 7 us slower on 512 rows of 128256
  // logits: a wavefront that waits for its whole batch and then runs through it leaves early, and its
  // successor's loads are on their way sooner.)  Elements outside whole vectors (unaligned rows, the
  // last V mod EPV logits) take the one-at-a-time online form in `extra`.
  float M = kNegHuge, s0 = 0.f, s1 = 0.f, u0 = 0.f, u1 = 0.f;
  Lse extra = lse_empty();
  if (aligned16(r.ptr)) {
    const int nv = V / EPV;
    const int chunk = slice_vectors(nv, S), v0 = min(s * chunk, nv), v1 = min(v0 + chunk, nv);
    const uint4* vec = reinterpret_cast<const uint4*>(r.ptr);
    const uint4 neutral = neutral_vec<DT>();
    for (int base = v0; base < v1; base += kRowBatch * kBlock) {
      uint4 v[kRowBatch];
      if (base + kRowBatch * kBlock <= v1) {          // (uniform) a whole batch: every lane has its vectors
#pragma unroll
        for (int j = 0; j < kRowBatch; ++j) v[j] = vec[base + tid + j * kBlock];
      } else {
#pragma unroll
        for (int j = 0; j < kRowBatch; ++j) {
          const int idx = base + tid + j * kBlock;
          const bool in = idx < v1;
          const uint4 x = vec[in ? idx : v1 - 1];
          v[j] = make_uint4(in ? x.x : neutral.x, in ? x.y : neutral.y, in ? x.z : neutral.z, in ? x.w : neutral.w);
        }
      }
      const float mb = wave_max_f(vecs_max<DT, kRowBatch>(v));
      if (mb > M) {                       // wave-uniform
        const float d = M - mb, f = ex2(d);
        u0 = (u0 + d * s0) * f;
        u1 = (u1 + d * s1) * f;
        s0 *= f;
        s1 *= f;
        M = mb;
      }
#pragma unroll
      for (int j = 0; j < kRowBatch; ++j) lse_accum<DT>(v[j], M, s0, s1, u0, u1);
    }
    if (s == S - 1 && tid == 0)
      for (int v = nv * EPV; v < V; ++v) lse_push(extra, load_elem<DT>(r.ptr, v));
  } else {
    const int e0 = (int)(((int64_t)s * V) / S), e1 = (int)(((int64_t)(s + 1) * V) / S);
    for (int v = e0 + tid; v < e1; v += kBlock) lse_push(extra, load_elem<DT>(r.ptr, v));
  }
  // wavefront fold: common reference, then plain sums
  Lse st = lse_merge(Lse{M, s0 + s1, u0 + u1}, extra);
  {
    const float Mw = wave_max_f(st.m), d = st.m - Mw, f = ex2(d);
    const float sw = wave_sum_f(st.s * f), uw = wave_sum_f((st.u + d * st.s) * f);
    st = Lse{Mw, sw, uw};
  }

  __shared__ Lse sh[kWaves];
  const int lane = tid & 63, wave = tid >> 6;
  if (lane == 0) sh[wave] = st;
  __syncthreads();
  if (tid == 0) {
    Lse t = sh[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) t = lse_merge(t, sh[w]);
    ws.part1[(size_t)rho * kMaxSplit + s] = make_float4(t.m, t.s, t.u, 0.f);   // folded by the next kernel
  }
}

// ---------------------------------------------------------------------------------------------
// Pass 2: JS divergence (the per-element term is jsd_push in stats_device.h).
// ---------------------------------------------------------------------------------------------
template <int DT, int kJsdBatch>   // kJsdBatch: vector pairs per thread and batch
__global__ void __launch_bounds__(kBlock)
k_jsd(RowMap map, int S, int S_fold, Workspace ws, VerifyOut vout) {
  warm_kernargs<sizeof(RowMap) + 2 * sizeof(int) + sizeof(Workspace) + sizeof(VerifyOut)>();
  constexpr int EPV = Elem<DT>::per_vec;
  // Full windows: the positions in reverse storage order.  The first kernel went through them forwards, so
  // what it read last (and what the XCDs' L2 caches may still hold) is asked for first (-0.6 us measured).
  const int slot = map.draft_len ? (int)blockIdx.y : (int)(gridDim.y - 1 - blockIdx.y);
  const int pos = position_of_slot(map, slot), s = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  __shared__ RowResult sh_row[2];
  __shared__ float sha[kWaves];
  if (pos < 0) return;
  const RowRef rp = locate_row<DT>(map, 2 * pos), rq = locate_row<DT>(map, 2 * pos + 1);
  if (!rp.active) return;
  const int V = map.V;
  const bool vec_path = aligned16(rp.ptr) && aligned16(rq.ptr);
  const int nv = V / EPV;
  const int chunk = slice_vectors(nv, S), v0 = min(s * chunk, nv), v1 = min(v0 + chunk, nv);
  const uint4* vp = reinterpret_cast<const uint4*>(rp.ptr);
  const uint4* vq = reinterpret_cast<const uint4*>(rq.ptr);
  const uint4 neutral = neutral_vec<DT>();
  uint4 xp[kJsdBatch], xq[kJsdBatch];
  // one batch of vector pairs: all loads in flight at once; a pair masked in both rows contributes 0
  auto load_batch = [&](int base) {
    if (base + kJsdBatch * kBlock <= v1) {          // (uniform) a whole batch: every lane has its vectors
#pragma unroll
      for (int j = 0; j < kJsdBatch; ++j) {
        xp[j] = vp[base + tid + j * kBlock];
        xq[j] = vq[base + tid + j * kBlock];
      }
      return;
    }
#pragma unroll
    for (int j = 0; j < kJsdBatch; ++j) {
      const int idx = base + tid + j * kBlock;
      const bool in = idx < v1;
      const uint4 a = vp[in ? idx : v1 - 1], b = vq[in ? idx : v1 - 1];
      xp[j] = make_uint4(in ? a.x : neutral.x, in ? a.y : neutral.y, in ? a.z : neutral.z, in ? a.w : neutral.w);
      xq[j] = make_uint4(in ? b.x : neutral.x, in ? b.y : neutral.y, in ? b.z : neutral.z, in ? b.w : neutral.w);
    }
  };
  // The position's drafted token, for the look-up of its two logits further down (one thread per
  // position).  Asked for ahead of the batch: loads come back in order, so the wait for the token then
  // does not include the batch.
  const bool gathers = s == 0 && tid == 0 && vout.tok != nullptr;
  int x = -1;
  if (gathers) x = vout.tokens[pos];
  // the first batch is requested before anything else that waits: it does not depend on the normalisers
  if (vec_path && v0 < v1) load_batch(v0);

  // both rows' slice results are folded by every workgroup of the position, the same way
  if (wave < 2) {
    const RowResult res = fold_row(ws, 2 * pos + wave, S_fold);   // S_fold records per row: this call's slices, or one per column shard
    if (lane == 0) sh_row[wave] = res;
  }
  __syncthreads();
  const RowResult resp = sh_row[0], resq = sh_row[1];
  const bool bad = resp.bad || resq.bad;
  uint32_t zx_p = 0u, zx_q = 0u;      // their bits: turned into floats where they are stored, at the very end
  if (gathers && x >= 0 && x < V) {
    zx_p = load_elem_bits<DT>(rp.ptr, x);
    zx_q = load_elem_bits<DT>(rq.ptr, x);
  }
  const JsNorm n = js_norm(resp, resq);
  float acc = 0.f;
  // (the same loops twice: rows whose normalisers are far apart take the longer form of the term)
  auto add_up = [&](auto far_tag) {
    constexpr bool FAR = decltype(far_tag)::value;
    if (vec_path) {
      float acc1 = 0.f;
      for (int base = v0; base < v1; base += kJsdBatch * kBlock) {
        if (base != v0) load_batch(base);
#pragma unroll
        for (int j = 0; j < kJsdBatch; ++j) {
          float zp[EPV], zq[EPV];
          unpack<DT>(xp[j], zp);
          unpack<DT>(xq[j], zq);
#pragma unroll
          for (int e = 0; e < EPV; e += 2) {
            jsd_push<FAR>(zp[e], zq[e], n, acc);
            jsd_push<FAR>(zp[e + 1], zq[e + 1], n, acc1);
          }
        }
      }
      acc += acc1;
      if (s == S - 1 && tid == 0)
        for (int v = nv * EPV; v < V; ++v)
          jsd_push<FAR>(load_elem<DT>(rp.ptr, v), load_elem<DT>(rq.ptr, v), n, acc);
    } else {
      const int e0 = (int)(((int64_t)s * V) / S), e1 = (int)(((int64_t)(s + 1) * V) / S);
      for (int v = e0 + tid; v < e1; v += kBlock)
        jsd_push<FAR>(load_elem<DT>(rp.ptr, v), load_elem<DT>(rq.ptr, v), n, acc);
    }
  };
  if (bad) {
    // nothing to add up: the decision kernel reports the distance as NaN
  } else if (n.far) {
    add_up(std::true_type{});
  } else {
    add_up(std::false_type{});
  }

  acc = wave_sum_f(acc);
  if (lane == 0) sha[wave] = acc;
  __syncthreads();
  if (tid == 0) {
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) t += sha[w];
    // partial sum of this slice: added up, corrected and turned into the distance by the decision kernel
    reinterpret_cast<float*>(&ws.part2[(size_t)pos * kMaxSplit + s])[0] = t;
    if (s == 0) {        // the position's rows and entropies, once
      ws.rows[2 * pos] = resp;
      ws.rows[2 * pos + 1] = resq;
      if (vout.H_p) vout.H_p[pos] = resp.H;
      if (vout.H_q) vout.H_q[pos] = resq.H;
      if (vout.tok) {
        asm volatile("" : "+v"(zx_p), "+v"(zx_q));   // keeps the conversion, and with it the wait for the two loads, down here
        vout.tok[pos] = make_float2(elem_from_bits<DT>(zx_p), elem_from_bits<DT>(zx_q));
      }
    }
  }
}

}  // namespace

namespace {

// One workgroup (as many wavefronts as 64 sequences each, at most 16): for every window position i in turn,
// the sequences whose window holds it, ranked by a ballot per wavefront and the wavefronts' counts.
__global__ void __launch_bounds__(1024) k_pack_slots(const int32_t* __restrict__ draft_len, int B, int K,
                                                     int32_t* __restrict__ slots) {
  __shared__ int sh_cnt[16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nt = blockDim.x, nw = nt >> 6;
  int base = 0;                                   // (every thread keeps the same count)
  for (int b0 = 0; b0 < B; b0 += nt) {            // (more sequences than threads: their chunks one after the other)
    const int b = b0 + tid;
    const int kb = b < B ? min(max(draft_len[b], 0), K) : 0;
    for (int i = 0; i < K; ++i) {
      const bool in = i < kb;
      const unsigned long long m = __ballot(in);
      if (nw > 1) {
        __syncthreads();                          // (the counts of the previous turn have been read)
        if (lane == 0) sh_cnt[wave] = __popcll(m);
        __syncthreads();
      }
      int before = base, total = 0;
      if (nw > 1) {
        for (int w = 0; w < nw; ++w) {
          before += w < wave ? sh_cnt[w] : 0;
          total += sh_cnt[w];
        }
      } else {
        total = __popcll(m);
      }
      if (in) slots[before + __popcll(m & ((1ull << lane) - 1ull))] = b * K + i;
      base += total;
    }
  }
  for (int m = base + tid; m < B * K; m += nt) slots[m] = -1;
}

}  // namespace

hipError_t launch_pack_slots(const int32_t* draft_len, int B, int K, int32_t* slots, hipStream_t st) {
  if (B <= 0 || K <= 0) return hipSuccess;
  int threads = (B + 63) / 64 * 64;
  if (threads > 1024) threads = 1024;
  launch_kernel(k_pack_slots, dim3(1), dim3(threads), st, draft_len, B, K, slots);
  return hipGetLastError();
}

int pick_split(int rows, int V, int dt) {
  const int epv = dt == ADASD_BF16 ? 8 : 4;
  const int nv = V / epv;
  int S = (4096 + rows - 1) / (rows > 0 ? rows : 1);
  int cap = nv / kBlock;            // at least one vector per thread and slice
  if (S > cap) S = cap;
  if (S > kMaxSplit) S = kMaxSplit;
  if (S < 1) S = 1;
  return S;
}

// vectors per thread and batch: the smallest power of two that covers a slice in one batch, up to `most`
static int pick_batch(int V, int dt, int S, int most) {
  const int nv = V / (dt == ADASD_BF16 ? 8 : 4);
  const int chunk = (nv + S - 1) / S, per_thread = (chunk + kBlock - 1) / kBlock;
  int nb = 1;
  while (nb < per_thread && nb < most) nb *= 2;
  return nb;
}

hipError_t launch_rowstats(const RowMap& map, int dt, int rows, int S, const Workspace& ws, hipStream_t st) {
  if (rows <= 0) return hipSuccess;
  dim3 grid(S, rows), block(kBlock);
  const int nb = pick_batch(map.V, dt, S, 8);
#define ADASD_ROW_CASE(DTV, NB) \
  if (dt == DTV && nb == NB) launch_kernel((k_rowstats<DTV, NB>), grid, block, st, map, S, ws);
  ADASD_ROW_CASE(ADASD_BF16, 1) ADASD_ROW_CASE(ADASD_BF16, 2) ADASD_ROW_CASE(ADASD_BF16, 4) ADASD_ROW_CASE(ADASD_BF16, 8)
  ADASD_ROW_CASE(ADASD_F32, 1) ADASD_ROW_CASE(ADASD_F32, 2) ADASD_ROW_CASE(ADASD_F32, 4) ADASD_ROW_CASE(ADASD_F32, 8)
#undef ADASD_ROW_CASE
  return hipGetLastError();
}

hipError_t launch_jsd(const RowMap& map, int dt, int S, int S_fold, const Workspace& ws, const VerifyOut& vout,
                      hipStream_t st) {
  const int positions = map.B * map.K;
  if (positions <= 0) return hipSuccess;
  dim3 grid(S, positions), block(kBlock);
  const int nb = pick_batch(map.V, dt, S, 4);
#define ADASD_JSD_CASE(DTV, NB) \
  if (dt == DTV && nb == NB) launch_kernel((k_jsd<DTV, NB>), grid, block, st, map, S, S_fold, ws, vout);
  ADASD_JSD_CASE(ADASD_BF16, 1) ADASD_JSD_CASE(ADASD_BF16, 2) ADASD_JSD_CASE(ADASD_BF16, 4)
  ADASD_JSD_CASE(ADASD_F32, 1) ADASD_JSD_CASE(ADASD_F32, 2) ADASD_JSD_CASE(ADASD_F32, 4)
#undef ADASD_JSD_CASE
  return hipGetLastError();
}

}  // namespace adasd
