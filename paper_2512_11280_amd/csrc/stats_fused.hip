// Single-read statistics kernel: normalisers, entropies and JS distance of every (target, draft) row
// pair with ONE read of the logits (Appendix A and Section 2.2 of the paper).
//
// The JS distance needs both normalisers before its first term can be formed, so the computation is
// inherently two-phase.  Instead of streaming the rows twice, every thread keeps its few 16-byte
// vectors of the row pair in registers across the two phases.  A work item is one slice of one
// position (T threads x NB vectors per row); a workgroup runs phase 1 on it (reference, sum, weighted
// sum of both rows), publishes the slice's result, waits for the other slices of the position, folds
// all of them (every workgroup of a position the same way, so the same normalisers everywhere) and
// runs phase 2 (the JS sum) on the registers it still holds.
//
// One workgroup per item, T threads, NB vectors per thread and row held in registers from the load to
// the end of phase 2.  The kernel is bound by the vector ALU (about 43 issued instructions per logit pair,
// 36 of them the arithmetic itself and five of those transcendental, against two bytes of bf16 each), so
// what matters is the instruction count per pair -- many pairs per thread, because the reductions and the
// exchange cost a fixed number of instructions per item -- and enough wavefronts per SIMD to keep it
// issuing while other workgroups load or wait: with four vectors per thread and row the kernel fits 64
// registers, i.e. eight wavefronts per SIMD.  (Also built and measured: persistent workgroups with two and
// with three register buffers, the loads and the exchange of the next items in flight behind the arithmetic
// of the current one.  They need about a hundred registers, i.e. four wavefronts per SIMD, and the folds
// that one wavefront does for its workgroup between two barriers then stand in the open: 56-80 us against 47.)
//
// Hand-off between the workgroups of a position: self-validating 64-bit words (two floats, valid flag
// in the low mantissa bit of the low float; a cleared word is 0) written and read with agent-scope
// atomic accesses: no fence, no separate flag, no read-modify-write, and since every word carries its
// own validity no ordering between different words is relied on.  The decision kernel, which runs
// next, clears the words of the positions it handles.  The slices of a position are consecutive
// workgroups of the grid and workgroups are dispatched in order, so whenever one waits, the ones it waits
// for are resident or next in line; all the same every wait is bounded: after `wait_polls` polls the
// workgroup recomputes the other slices' results itself from memory with the very same code
// (bit-identical), so every wave exits whatever the dispatch order is.
#include "stats_device.h"

namespace adasd {

namespace {

__device__ __forceinline__ float flagged(float v) { return __uint_as_float(__float_as_uint(v) | 1u); }
__device__ __forceinline__ void put_pair(uint64_t* p, float lo_flagged, float hi) {
  const uint64_t w = ((uint64_t)__float_as_uint(hi) << 32) | (uint64_t)__float_as_uint(lo_flagged);
  __hip_atomic_store(p, w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t get_word(const uint64_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float lo_float(uint64_t w) { return __uint_as_float((uint32_t)w); }
__device__ __forceinline__ float hi_float(uint64_t w) { return __uint_as_float((uint32_t)(w >> 32)); }

struct FusedGeom {
  int S;           // slices (work items) per position
  int nv;          // 16-byte vectors per row
  int chunk;       // vectors per slice
  int wait_polls;  // polls before a workgroup stops waiting and recomputes what is missing
};

struct SliceRecord {   // phase-1 result of one slice of a row pair; the references carry the valid flag
  float mp, sp, up, mq, sq, uq;
};

template <int W> struct FusedShared {
  SliceRecord wave[W];            // per-wavefront results of the slice in hand
  SliceRecord redo[kMaxSplit];    // recomputed slices (only after an expired wait)
  JsNorm norm;
  RowResult row[2];
  int bad, expired;
  float acc[W];
};

// Workgroup barrier that waits for LDS traffic only (outstanding global loads stay in flight).
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// The vectors of slice s that this thread holds: vector j is number v0 + tid + j*T of the row.  Loads are
// issued unconditionally (lanes past the end re-read the slice's last vector); mask_slice then puts -inf
// where a lane is past the end.  The two are separate so that the masking can wait until the values are
// needed: the loads of an item are issued a turn ahead of their use.
template <int DT, int T, int NB>
__device__ __forceinline__ void load_slice(const char* prow, const char* qrow, int s, const FusedGeom& g,
                                           uint4 (&xp)[NB], uint4 (&xq)[NB]) {
  const int v0 = min(s * g.chunk, g.nv), v1 = min(v0 + g.chunk, g.nv), tid = threadIdx.x;
  const uint4* vp = reinterpret_cast<const uint4*>(prow);
  const uint4* vq = reinterpret_cast<const uint4*>(qrow);
  const int last = max(v1 - 1, 0);     // (an empty slice reads vector 0, all of it masked afterwards)
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    const int idx = min(v0 + tid + j * T, last);
    xp[j] = vp[idx];
    xq[j] = vq[idx];
  }
}
template <int DT, int T, int NB>
__device__ __forceinline__ void mask_slice(int s, const FusedGeom& g, uint4 (&xp)[NB], uint4 (&xq)[NB]) {
  const int v0 = min(s * g.chunk, g.nv), v1 = min(v0 + g.chunk, g.nv), tid = threadIdx.x;
  if (v0 + NB * T <= v1) return;       // (uniform) a whole slice: every lane has its vectors
  const uint4 neutral = neutral_vec<DT>();
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    const bool in = v0 + tid + j * T < v1;
    xp[j] = make_uint4(in ? xp[j].x : neutral.x, in ? xp[j].y : neutral.y, in ? xp[j].z : neutral.z, in ? xp[j].w : neutral.w);
    xq[j] = make_uint4(in ? xq[j].x : neutral.x, in ? xq[j].y : neutral.y, in ? xq[j].z : neutral.z, in ? xq[j].w : neutral.w);
  }
}

// Phase 1 of the slice held in (xp, xq) by the whole workgroup.  Wavefront 0 returns the slice's record
// (wave-uniform); the other wavefronts return their own.  One workgroup barrier.
template <int DT, int T, int NB>
__device__ __forceinline__ SliceRecord phase1(const uint4 (&xp)[NB], const uint4 (&xq)[NB],
                                              FusedShared<T / 64>& sh) {
  constexpr int W = T / 64;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  SliceRecord r;
  r.mp = flagged(wave_max_f(vecs_max<DT, NB>(xp)));
  r.mq = flagged(wave_max_f(vecs_max<DT, NB>(xq)));
  float ps0 = 0.f, ps1 = 0.f, pu0 = 0.f, pu1 = 0.f, qs0 = 0.f, qs1 = 0.f, qu0 = 0.f, qu1 = 0.f;
  float neg_mp = -r.mp, neg_mq = -r.mq;
  asm volatile("" : "+v"(neg_mp), "+v"(neg_mq));   // in vector registers, once
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    lse_accum_neg<DT>(xp[j], neg_mp, ps0, ps1, pu0, pu1);
    lse_accum_neg<DT>(xq[j], neg_mq, qs0, qs1, qu0, qu1);
    __builtin_amdgcn_sched_barrier(0);     // one vector pair at a time: keeps the number of unpacked values in flight small
  }
  r.sp = wave_sum_f(ps0 + ps1);
  r.up = wave_sum_f(pu0 + pu1);
  r.sq = wave_sum_f(qs0 + qs1);
  r.uq = wave_sum_f(qu0 + qu1);
  if (lane == 0) sh.wave[wave] = r;
  lds_barrier();
  if (wave != 0) return r;
  // the W wavefront results, one per lane: common reference, plain sums
  Lse tp = lse_empty(), tq = lse_empty();
  if (lane < W) {
    const SliceRecord o = sh.wave[lane];
    tp = Lse{o.mp, o.sp, o.up};
    tq = Lse{o.mq, o.sq, o.uq};
  }
  SliceRecord f;
  {
    const float M = wave_max_f(tp.m), d = tp.m - M, e = ex2(d);
    f.mp = M;
    f.sp = wave_sum_f(tp.s * e);
    f.up = wave_sum_f((tp.u + d * tp.s) * e);
  }
  {
    const float M = wave_max_f(tq.m), d = tq.m - M, e = ex2(d);
    f.mq = M;
    f.sq = wave_sum_f(tq.s * e);
    f.uq = wave_sum_f((tq.u + d * tq.s) * e);
  }
  return f;
}

template <int DT, int NB, bool FAR>
__device__ __forceinline__ float phase2(const uint4 (&xp)[NB], const uint4 (&xq)[NB], const JsNorm& n) {
  constexpr int EPV = Elem<DT>::per_vec;
  float acc0 = 0.f, acc1 = 0.f;
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    // (an opaque copy: without it the unpacking, common to the two forms of this function, is moved up in
    // front of the branch between them, and every unpacked value of the buffer is live at once)
    uint4 vp = xp[j], vq = xq[j];
    asm volatile("" : "+v"(vp.x), "+v"(vp.y), "+v"(vp.z), "+v"(vp.w));
    asm volatile("" : "+v"(vq.x), "+v"(vq.y), "+v"(vq.z), "+v"(vq.w));
    float zp[EPV], zq[EPV];
    unpack<DT>(vp, zp);
    unpack<DT>(vq, zq);
#pragma unroll
    for (int e = 0; e < EPV; e += 2) {
      jsd_push<FAR>(zp[e], zq[e], n, acc0);
      if (FAR) __builtin_amdgcn_sched_barrier(0);
      jsd_push<FAR>(zp[e + 1], zq[e + 1], n, FAR ? acc0 : acc1);   // (the long form gets by with one register less)
      if (FAR) __builtin_amdgcn_sched_barrier(0);   // (the long form, rarely taken, must not set the kernel's register count)
    }
    __builtin_amdgcn_sched_barrier(0);     // one vector pair at a time: keeps the number of unpacked values in flight small
  }
  return acc0 + acc1;
}

__device__ __forceinline__ void publish(const Workspace& ws, int pos, int s, const SliceRecord& r) {
  uint64_t* w = ws.xchg + ((size_t)pos * kMaxSplit + s) * kXchgWords;
  put_pair(w + 0, r.mp, r.sp);
  put_pair(w + 1, r.mq, r.sq);
  put_pair(w + 2, flagged(r.up), r.uq);
}

// Wavefront 0: the rows' results and what phase 2 needs of them, from one slice record per lane.
__device__ __forceinline__ void fold_position(const Lse& tp, const Lse& tq, JsNorm& norm, RowResult (&row)[2], int& bad) {
  const RowResult resp = fold_lanes(tp), resq = fold_lanes(tq);
  if ((threadIdx.x & 63) == 0) {
    norm = js_norm(resp, resq);
    row[0] = resp;
    row[1] = resq;
    bad = resp.bad || resq.bad;
  }
}

template <int DT, int T, int NB>
__global__ void __launch_bounds__(T, NB <= 4 ? 8 : 4)
k_stats_fused(RowMap map, FusedGeom g, Workspace ws, VerifyOut vout) {
  warm_kernargs<sizeof(RowMap) + sizeof(FusedGeom) + sizeof(Workspace) + sizeof(VerifyOut)>();
  constexpr int W = T / 64;
  __shared__ FusedShared<W> sh;
  const int s = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int pos = position_of_slot(map, (int)blockIdx.y);
  if (pos < 0) return;
  const RowRef rp = locate_row<DT>(map, 2 * pos), rq = locate_row<DT>(map, 2 * pos + 1);
  if (!rp.active) return;

  // the drafted token of the position (its two logits are looked up further down by one thread)
  const bool gathers = s == 0 && tid == 0 && vout.tok != nullptr;
  int x = -1;
  if (gathers) x = vout.tokens[pos];

  uint4 xp[NB], xq[NB];
  load_slice<DT, T, NB>(rp.ptr, rq.ptr, s, g, xp, xq);
  mask_slice<DT, T, NB>(s, g, xp, xq);
  const SliceRecord mine = phase1<DT, T, NB>(xp, xq, sh);

  if (wave == 0) {
    const bool need = lane < g.S;
    bool ok = true;
    Lse tp = lse_empty(), tq = lse_empty();
    if (g.S > 1) {
      if (lane == 0) publish(ws, pos, s, mine);
      // every slice of the position, one per lane (this workgroup's own words come back the same way)
      const uint64_t* src = ws.xchg + ((size_t)pos * kMaxSplit + (need ? lane : 0)) * kXchgWords;
      uint64_t w0, w1, w2;
      int polls = 0;
      while (true) {
        w0 = get_word(src + 0);
        w1 = get_word(src + 1);
        w2 = get_word(src + 2);
        ok = __all(!need || ((w0 & w1 & w2 & 1ull) != 0));
        if (ok || ++polls > g.wait_polls) break;
        __builtin_amdgcn_s_sleep(4);
      }
      if (need) {
        tp = Lse{lo_float(w0), hi_float(w0), lo_float(w2)};
        tq = Lse{lo_float(w1), hi_float(w1), hi_float(w2)};
      }
    } else if (lane == 0) {              // one slice per position: nothing travels through memory
      tp = Lse{mine.mp, mine.sp, flagged(mine.up)};
      tq = Lse{mine.mq, mine.sq, mine.uq};
    }
    if (ok) fold_position(tp, tq, sh.norm, sh.row, sh.bad);
    if (lane == 0) sh.expired = ok ? 0 : 1;
  }
  lds_barrier();
  if (sh.expired) {                        // (uniform) the bounded wait ran out: every slice from memory
    if (tid == 0) sh.redo[s] = mine;
    for (int o = 0; o < g.S; ++o) {
      if (o == s) continue;
      lds_barrier();                       // (sh.wave of the previous turn has been read)
      load_slice<DT, T, NB>(rp.ptr, rq.ptr, o, g, xp, xq);
      mask_slice<DT, T, NB>(o, g, xp, xq);
      const SliceRecord other = phase1<DT, T, NB>(xp, xq, sh);
      if (tid == 0) sh.redo[o] = other;
    }
    lds_barrier();
    if (wave == 0) {
      Lse tp = lse_empty(), tq = lse_empty();
      if (lane < g.S) {
        const SliceRecord o = sh.redo[lane];
        // (what travels through the words: the weighted sum of the target row carries the flag)
        tp = Lse{o.mp, o.sp, flagged(o.up)};
        tq = Lse{o.mq, o.sq, o.uq};
      }
      fold_position(tp, tq, sh.norm, sh.row, sh.bad);
    }
    // (the slice number goes through an opaque copy: otherwise the addresses of the loads at the top of the
    // kernel are kept in registers all the way down here, sixteen of them per thread)
    int s_again = s;
    asm volatile("" : "+s"(s_again));
    load_slice<DT, T, NB>(rp.ptr, rq.ptr, s_again, g, xp, xq);
    mask_slice<DT, T, NB>(s_again, g, xp, xq);
    lds_barrier();
  }

  const JsNorm n = sh.norm;
  const bool bad = sh.bad != 0;
  uint32_t zx_p = 0u, zx_q = 0u;
  if (gathers && x >= 0 && x < map.V) {
    zx_p = load_elem_bits<DT>(rp.ptr, x);
    zx_q = load_elem_bits<DT>(rq.ptr, x);
  }
  float acc = 0.f;
  if (!bad) acc = n.far ? phase2<DT, NB, true>(xp, xq, n) : phase2<DT, NB, false>(xp, xq, n);
  acc = wave_sum_f(acc);
  if (lane == 0) sh.acc[wave] = acc;
  lds_barrier();
  if (tid == 0) {
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < W; ++w) t += sh.acc[w];
    // partial sum of this slice: added up, corrected and turned into the distance by the decision kernel
    reinterpret_cast<float*>(&ws.part2[(size_t)pos * kMaxSplit + s])[0] = t;
    if (s == 0) {        // the position's rows and entropies, once
      const RowResult resp = sh.row[0], resq = sh.row[1];
      ws.rows[2 * pos] = resp;
      ws.rows[2 * pos + 1] = resq;
      if (vout.H_p) vout.H_p[pos] = resp.H;
      if (vout.H_q) vout.H_q[pos] = resq.H;
      if (vout.tok) vout.tok[pos] = make_float2(elem_from_bits<DT>(zx_p), elem_from_bits<DT>(zx_q));
    }
  }
}

}  // namespace

// Can the single-read kernel take this call, and with which tiling?  Requirements: every row starts on
// a 16-byte boundary, the vocabulary is a whole number of vectors, and at most kMaxSplit slices of at
// most eight vectors per thread and row.
bool fused_plan(const RowMap& map, int dt, int* T_out, int* NB_out, int* S_out) {
  const int es = dt == ADASD_BF16 ? 2 : 4, epv = 16 / es;
  if (map.K <= 0 || map.V % epv != 0) return false;
  for (int w = 0; w < 2; ++w) {
    if (reinterpret_cast<uintptr_t>(map.base[w]) % 16 != 0) return false;
    if ((map.seq_stride[w] * es) % 16 != 0 || (map.pos_stride[w] * es) % 16 != 0) return false;
  }
  const int nv = map.V / epv;
  int T = 512, NB = 4;
  while (T > 256 && nv <= (T / 2) * NB) T /= 2;                 // small vocabularies: smaller workgroups
  while (NB > 1 && nv <= T * (NB / 2)) NB /= 2;
  while (NB < 8 && (nv + T * NB - 1) / (T * NB) > kMaxSplit) NB *= 2;   // very large ones: more vectors per thread
  const int S = (nv + T * NB - 1) / (T * NB);
  if (S > kMaxSplit) return false;
  *T_out = T;
  *NB_out = NB;
  *S_out = S;
  return true;
}

hipError_t launch_stats_fused(const RowMap& map, int dt, int T, int NB, int S, int wait_polls,
                              const Workspace& ws, const VerifyOut& vout, hipStream_t st) {
  const int positions = map.B * map.K;
  if (positions <= 0) return hipSuccess;
  FusedGeom g;
  g.S = S;
  g.nv = map.V / (dt == ADASD_BF16 ? 8 : 4);
  g.chunk = (g.nv + S - 1) / S;
  g.chunk = (g.chunk + 63) / 64 * 64;          // whole wavefronts of vectors (the last slice takes what is left)
  if ((int64_t)g.chunk * (S - 1) >= g.nv) g.chunk = (g.nv + S - 1) / S;
  g.wait_polls = wait_polls;
  if (g.chunk > T * NB) return hipErrorInvalidValue;
  const dim3 grid(S, positions);
#define ADASD_FUSED_CASE(DTV, TV, NBV) \
  if (dt == DTV && T == TV && NB == NBV) { \
    launch_kernel((k_stats_fused<DTV, TV, NBV>), grid, dim3(TV), st, map, g, ws, vout); \
    return hipGetLastError(); \
  }
#define ADASD_FUSED_DT(DTV) \
  ADASD_FUSED_CASE(DTV, 256, 1) ADASD_FUSED_CASE(DTV, 256, 2) ADASD_FUSED_CASE(DTV, 256, 4) ADASD_FUSED_CASE(DTV, 256, 8) \
  ADASD_FUSED_CASE(DTV, 512, 1) ADASD_FUSED_CASE(DTV, 512, 2) ADASD_FUSED_CASE(DTV, 512, 4) ADASD_FUSED_CASE(DTV, 512, 8) \
  ADASD_FUSED_CASE(DTV, 1024, 2) ADASD_FUSED_CASE(DTV, 1024, 4)
  ADASD_FUSED_DT(ADASD_BF16)
  ADASD_FUSED_DT(ADASD_F32)
#undef ADASD_FUSED_DT
#undef ADASD_FUSED_CASE
  return hipErrorInvalidValue;
}

}  // namespace adasd
