// Single-read statistics kernel: normalisers, entropies and JS distance of every (target, draft) row
// pair with ONE read of the logits from HBM (Appendix A and Section 2.2 of the paper).
//
// The JS distance needs both normalisers before its first term can be formed, so the computation
// is inherently two-phase.  Instead of streaming the rows twice, a workgroup keeps its slice of the
// row pair in registers (raw 128-bit vectors: 8 bf16 or 4 fp32 logits each), runs phase 1 on them,
// exchanges the per-wavefront (reference, sum) pairs with the other workgroups working on the same
// position through the workspace, and runs phase 2 on the same registers.
//
// Structure: persistent workgroups of four wavefronts, each looping over work items
// (position, slice) with a three-deep software pipeline over three register buffers:
//     tick n:   phase 1 of item n+1, the loads of item n+2 issued between its chunks | phase 2 of item n
// so HBM has loads in flight while the vector ALU works, and a whole tick passes between publishing
// a slice's results and needing the siblings'.  Memory results return in issue order, so what a tick
// reads from other workgroups is requested BEFORE the tick's prefetch is issued, and the workgroup
// barrier waits for LDS traffic only, never for the prefetch.
//
// Item order: consecutive workgroup ids are dealt round-robin to the 8 XCDs, so item k is decoded as
// (xcd = k % 8, local = k / 8): the S slices of one position get consecutive `local` values on ONE
// XCD and, because the grid size is a multiple of 8*S, are processed in the same tick by different
// workgroups, all of them resident.
//
// Hand-off between workgroups uses self-validating 64-bit words (two floats, valid flag in the low
// mantissa bit of the low float) written and read with agent-scope atomic accesses: no fence, no
// separate flag, no read-modify-write atomics.  Every wait is bounded: after `spin_limit` polls a
// workgroup recomputes the siblings' results itself from memory with the very same code
// (bit-identical), so all waves exit whatever the dispatch order is.  A second small kernel finalises
// the positions in double precision and clears the words.
//
// On gfx950 this kernel is bound by the vector ALU, not by HBM (about 48 lane-instructions per logit
// pair against a budget of 20 at the HBM roofline), which is why reading the rows once does not pay
// here: the two-kernel path is the default and this one is selected explicitly.
#include "internal.h"

namespace adasd {

namespace {

constexpr int kXcd = 8;
constexpr int kWave = 64;

// Hand-off words: two floats per 64-bit word; the LOW float carries the valid flag in the least
// significant bit of its mantissa (a cleared word is 0, a published one never is).
__device__ __forceinline__ float flagged(float v) { return __uint_as_float(__float_as_uint(v) | 1u); }
__device__ __forceinline__ void put_pair(uint64_t* p, float lo_flagged, float hi) {
  const uint64_t w = ((uint64_t)__float_as_uint(hi) << 32) | (uint64_t)__float_as_uint(lo_flagged);
  __hip_atomic_store(p, w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t get_word(const uint64_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void clear_word(uint64_t* p) {
  __hip_atomic_store(p, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float lo_float(uint64_t w) { return __uint_as_float((uint32_t)w); }
__device__ __forceinline__ float hi_float(uint64_t w) { return __uint_as_float((uint32_t)(w >> 32)); }

// Fold of up to 128 triples held two per lane: common reference first, then plain sums.
__device__ __forceinline__ Lse wave_fold(const Lse& a, const Lse& b) {
  Lse r;
  r.m = wave_max_f(fmaxf(a.m, b.m));
  const float da = a.m - r.m, db = b.m - r.m;
  const float fa = ex2(da), fb = ex2(db);
  r.s = wave_sum_f(a.s * fa + b.s * fb);
  r.u = wave_sum_f((a.u + da * a.s) * fa + (b.u + db * b.s) * fb);
  return r;
}

struct PipeGeom {
  int S;           // workgroup slices per row
  int nv;          // 16-byte vectors per row
  int P;           // positions (B * k_max)
  int items;       // padded item count: ceil(P / 8) * 8 * S
  int chunk;       // vectors per slice: ceil(nv / S)
  int pos_step;    // positions between a workgroup's items of consecutive ticks: grid / S
  int spin_limit;  // polls before a wavefront stops waiting and recomputes what is missing
};

struct Item {
  int pos, s;
  bool valid;
  const char* prow;
  const char* qrow;
};

// Decoding an item reads the sequence's draft length from memory; it is split in two so that the
// read is issued a tick before its result is needed.
struct Seed {
  int pos, s, b, i, kb;
  bool in_range;
};

// The grid is a multiple of 8*S workgroups, so a workgroup keeps its XCD and its slice through all
// ticks and its position advances by a constant step: no division by S in the loop.
__device__ __forceinline__ Seed decode_begin(const RowMap& map, const PipeGeom& g, int tick) {
  const int xcd = blockIdx.x % kXcd, local0 = blockIdx.x / kXcd;
  Seed sd;
  sd.s = local0 % g.S;
  sd.pos = (local0 / g.S) * kXcd + xcd + tick * g.pos_step;
  sd.in_range = sd.pos < g.P;
  sd.b = sd.in_range ? sd.pos / map.K : 0;
  sd.i = sd.pos - sd.b * map.K;
  sd.kb = map.draft_len ? map.draft_len[sd.b] : map.K;
  return sd;
}

template <int DT>
__device__ __forceinline__ Item decode_end(const RowMap& map, const Seed& sd) {
  Item it;
  it.valid = sd.in_range && sd.i < min(max(sd.kb, 0), map.K);
  it.pos = it.valid ? sd.pos : 0;
  it.s = it.valid ? sd.s : 0;
  // items that are not valid still load and compute (nothing is published): their pointers name the
  // first position's rows
  const int b = it.valid ? sd.b : 0, i = it.valid ? sd.i : 0;
  it.prow = map.base[0] + ((int64_t)b * map.seq_stride[0] + (int64_t)i * map.pos_stride[0]) * Elem<DT>::bytes;
  it.qrow = map.base[1] + ((int64_t)b * map.seq_stride[1] + (int64_t)i * map.pos_stride[1]) * Elem<DT>::bytes;
  return it;
}

// Loads are issued unconditionally and without branches (out-of-range lanes re-read the slice's last
// vector and then substitute -inf): only straight-line load sequences let the compiler keep exact
// track of how many loads may still be in flight when an older buffer is consumed.
struct SliceRange {
  int v0, v1;
};
__device__ __forceinline__ SliceRange slice_range(int s, const PipeGeom& g) {
  const int v0 = min(s * g.chunk, g.nv);
  return SliceRange{v0, min(v0 + g.chunk, g.nv)};
}
template <int DT>
__device__ __forceinline__ uint4 load_vec(const char* row, const SliceRange& r, int j) {
  const uint4* src = reinterpret_cast<const uint4*>(row);
  const uint4 neutral = neutral_vec<DT>();
  const int idx = r.v0 + (int)threadIdx.x + j * kBlock;
  const bool in = idx < r.v1;
  const uint4 x = src[in ? idx : r.v1 - 1];
  return make_uint4(in ? x.x : neutral.x, in ? x.y : neutral.y, in ? x.z : neutral.z, in ? x.w : neutral.w);
}

template <int NV> struct Buf {
  uint4 p[NV], q[NV];
};

template <int DT, int NV>
__device__ __forceinline__ void load_item(const Item& it, const PipeGeom& g, Buf<NV>& b) {
  const SliceRange r = slice_range(it.s, g);
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    b.p[j] = load_vec<DT>(it.prow, r, j);
    b.q[j] = load_vec<DT>(it.qrow, r, j);
  }
}

// Per-lane sums of phase 1 for both rows of an item.
struct P1Sums {
  float ps0 = 0.f, ps1 = 0.f, pu0 = 0.f, pu1 = 0.f, qs0 = 0.f, qs1 = 0.f, qu0 = 0.f, qu1 = 0.f;
};
template <int DT, int NV>
__device__ __forceinline__ void p1_chunk(const Buf<NV>& b, int j, float ref_p, float ref_q, P1Sums& a) {
  lse_accum<DT>(b.p[j], ref_p, a.ps0, a.ps1, a.pu0, a.pu1);
  __builtin_amdgcn_sched_barrier(0);     // keeps the number of unpacked values in flight small
  lse_accum<DT>(b.q[j], ref_q, a.qs0, a.qs1, a.qu0, a.qu1);
}
__device__ __forceinline__ void p1_reduce(const P1Sums& a, Lse& lp, Lse& lq) {
  lp.s = wave_sum_f(a.ps0 + a.ps1);
  lp.u = wave_sum_f(a.pu0 + a.pu1);
  lq.s = wave_sum_f(a.qs0 + a.qs1);
  lq.u = wave_sum_f(a.qu0 + a.qu1);
}
// References of the part of a row pair held by a wavefront (wave-uniform; they travel in flagged
// words, so they are flagged before they are used).  FIRST_ONLY takes the maximum over the first vector
// of each row only, the one whose load was issued first: any reference within about 2^100 of the true
// maximum gives the same sums up to rounding, and a part whose first 512 logits are all masked, or
// whose logits span more than that, shows as a sum that is not finite and is then redone exactly.
template <int DT, int NV, bool FIRST_ONLY>
__device__ __forceinline__ void p1_refs(const Buf<NV>& b, float& ref_p, float& ref_q) {
  if (FIRST_ONLY) {
    const uint4 fp[1] = {b.p[0]}, fq[1] = {b.q[0]};
    ref_p = flagged(wave_max_f(vecs_max<DT, 1>(fp)));
    ref_q = flagged(wave_max_f(vecs_max<DT, 1>(fq)));
  } else {
    ref_p = flagged(wave_max_f(vecs_max<DT, NV>(b.p)));
    ref_q = flagged(wave_max_f(vecs_max<DT, NV>(b.q)));
  }
}
// A mean exponent u/s well above zero means that a token well above the cheap reference carries most of the
// part's mass: then the weighted sum is one large term plus the small ones that hold the entropy, and float
// loses those (an absolute error of about (maximum - reference) x 2^-24 nats on the row's entropy).  Such
// parts are redone with their true maximum as well (with that, every term is <= 0).  Ordinary rows, whose
// mass sits within a few units of the part's maximum, stay below the mark.
__device__ __forceinline__ bool p1_suspect(const Lse& lp, const Lse& lq) {
  return !(lp.s < INFINITY) || !(lq.s < INFINITY) || !(fabsf(lp.u) < INFINITY) || !(fabsf(lq.u) < INFINITY) ||
         lp.u > 4.f * lp.s || lq.u > 4.f * lq.s;
}
// Phase 1 in one piece with exact references.
template <int DT, int NV>
__device__ __forceinline__ void phase1_exact(const Buf<NV>& b, Lse& lp, Lse& lq) {
  p1_refs<DT, NV, false>(b, lp.m, lq.m);
  P1Sums a;
#pragma unroll
  for (int j = 0; j < NV; ++j) p1_chunk<DT, NV>(b, j, lp.m, lq.m, a);
  p1_reduce(a, lp, lq);
}
// The same from memory, as a real call: taken only for parts whose cheap references failed.
template <int DT, int NV>
__device__ __noinline__ void redo_exact(const char* prow, const char* qrow, int s, int chunk, int nv,
                                        float* out /* m_p s_p u_p m_q s_q u_q, per lane */) {
  PipeGeom g;
  g.chunk = chunk;
  g.nv = nv;
  Item one;
  one.prow = prow;
  one.qrow = qrow;
  one.s = s;
  Buf<NV> tmp;
  load_item<DT, NV>(one, g, tmp);
  Lse lp, lq;
  phase1_exact<DT, NV>(tmp, lp, lq);
  out[0] = lp.m; out[1] = lp.s; out[2] = lp.u; out[3] = lq.m; out[4] = lq.s; out[5] = lq.u;
}
template <int DT, int NV>
__device__ __forceinline__ void fix_suspect(const Item& it, const PipeGeom& g, Lse& lp, Lse& lq) {
  if (p1_suspect(lp, lq)) {        // wave-uniform
    float r[6];
    redo_exact<DT, NV>(it.prow, it.qrow, it.s, g.chunk, g.nv, r);
    lp = Lse{r[0], r[1], r[2]};
    lq = Lse{r[3], r[4], r[5]};
  }
}
// Phase 1 in one piece (prologue and recomputation); the pipeline runs the same steps spread out.
template <int DT, int NV>
__device__ __forceinline__ void phase1(const Item& it, const PipeGeom& g, const Buf<NV>& b, Lse& lp, Lse& lq) {
  p1_refs<DT, NV, true>(b, lp.m, lq.m);
  P1Sums a;
#pragma unroll
  for (int j = 0; j < NV; ++j) p1_chunk<DT, NV>(b, j, lp.m, lq.m, a);
  p1_reduce(a, lp, lq);
  fix_suspect<DT, NV>(it, g, lp, lq);
}

// One element of the JS sum (the algebra is explained above jsd_push in stats.hip).
__device__ __forceinline__ void jsd_term(float zp, float zq, float cp, float cq, float dc, float& acc) {
  float yp = fmaf(zp, kLog2e, -cp), yq = fmaf(zq, kLog2e, -cq);
  float b = ex2(fmaxf(yp, yq));
  float delta = fmaf(zq - zp, kLog2e, -dc);
  float nd = fmaxf(-fabsf(delta), -126.0f);
  float r = ex2(nd);
  float h = fmaf(r, 0.5f, 0.5f);
  float t = fmaf(-2.0f, h * lg2(h), r * nd);
  acc = fmaf(b, t, acc);
}

template <int DT, int NV>
__device__ __forceinline__ float slice_jsd(const uint4 (&vp)[NV], const uint4 (&vq)[NV], float cp,
                                           float cq, float dc) {
  constexpr int EPV = Elem<DT>::per_vec;
  float acc0 = 0.f, acc1 = 0.f;
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    float zp[EPV], zq[EPV];
    unpack<DT>(vp[j], zp);
    unpack<DT>(vq[j], zq);
#pragma unroll
    for (int e = 0; e < EPV; e += 2) {
      jsd_term(zp[e], zq[e], cp, cq, dc, acc0);
      jsd_term(zp[e + 1], zq[e + 1], cp, cq, dc, acc1);
    }
    __builtin_amdgcn_sched_barrier(0);   // keeps the number of unpacked values in flight small
  }
  return acc0 + acc1;     // per lane; the caller reduces over the wavefront
}

// Hand-off words are kept per wavefront: wave w of slice s owns entry s*4 + w of its position.
// word 0: (m_p flagged, s_p)   word 1: (m_q flagged, s_q)   word 2: (u_p flagged, u_q)
// word 3: (phase-2 partial sum flagged, 0)
__device__ __forceinline__ uint64_t* slot_of(const Workspace& ws, int pos, int entry) {
  return ws.fused_slots + ((size_t)pos * kMaxFusedSplit + entry) * kSlotWords;
}

struct LdsBlock {
  float part[2][kWaves][4];   // [tick parity][wave][m_p, s_p, m_q, s_q] folded over a quarter of the entries
  int part_ok[2][kWaves];     // 1: fetched; 0: the bounded wait expired
  float redo[kMaxFusedSplit][4];   // recomputed (m_p, s_p, m_q, s_q) (only used after an expired wait)
};

// Workgroup barrier that waits for LDS traffic only (outstanding global loads stay in flight).
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

struct Norm {     // what phase 2 needs, identical in every workgroup of a position
  float cp, cq, dc;
  bool ok;
};

__device__ __forceinline__ bool ms_ok(float m, float s) {
  return (s > 0.f) && (s < INFINITY) && (m > kNegHuge) && (m < INFINITY);
}
__device__ __forceinline__ bool lse_ok(const Lse& t) { return ms_ok(t.m, t.s) && (fabsf(t.u) < INFINITY); }

__device__ __forceinline__ Norm make_norm(float mp, float sp, float mq, float sq) {
  Norm n;
  const float l2p = lg2(sp), l2q = lg2(sq);
  n.cp = mp + l2p;                              // log2-sum-exp of p, float
  n.cq = mq + l2q;
  n.dc = (mq - mp) + (l2q - l2p);               // their difference, formed from the small parts
  n.ok = ms_ok(mp, sp) && ms_ok(mq, sq);
  return n;
}

// Folding the 4S published (m, s) pairs of a position is shared by the four wavefronts: wave w looks
// after entries [w*S, (w+1)*S), lanes 0..31 take their target-row word, lanes 32..63 the draft-row word.
__device__ __forceinline__ const uint64_t* fetch_address(const Item& it, const PipeGeom& g, const Workspace& ws) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, idx = lane & 31;
  return slot_of(ws, it.pos, wave * g.S + (idx < g.S ? idx : 0)) + (lane >> 5);
}
// Fold of one quarter: every lane passes the (m, s) of its entry (or an empty one); the results are
// wave-uniform.  Rows of 16 lanes are folded by rotations, the two rows of each half through scalars.
__device__ __forceinline__ void fold_quarter(float m, float s, float (&out)[4]) {
  float v = m;
  v = fmaxf(v, dpp_rot<0x121>(v));
  v = fmaxf(v, dpp_rot<0x122>(v));
  v = fmaxf(v, dpp_rot<0x124>(v));
  v = fmaxf(v, dpp_rot<0x128>(v));
  const float Mp = fmaxf(lane_value(v, 0), lane_value(v, 16)), Mq = fmaxf(lane_value(v, 32), lane_value(v, 48));
  const float M = (threadIdx.x & 32) ? Mq : Mp;
  float t = s * ex2(m - M);
  t += dpp_rot<0x121>(t);
  t += dpp_rot<0x122>(t);
  t += dpp_rot<0x124>(t);
  t += dpp_rot<0x128>(t);
  out[0] = Mp;
  out[1] = lane_value(t, 0) + lane_value(t, 16);
  out[2] = Mq;
  out[3] = lane_value(t, 32) + lane_value(t, 48);
}
// The word of this lane was not valid when first looked at: poll (bounded).  False if it still is not.
__device__ __forceinline__ bool fetch_retry(const Item& it, const PipeGeom& g, const Workspace& ws, uint64_t& w) {
  const bool need = (threadIdx.x & 31) < g.S;
  int spins = 0;
  while (true) {
    if (++spins > g.spin_limit) return false;
    __builtin_amdgcn_s_sleep(8);
    w = get_word(fetch_address(it, g, ws));
    if (__all(!need || (w & 1ull))) return true;
  }
}
// The four quarters are merged the same way wherever it is done.
__device__ __forceinline__ void merge4(const float (&part)[kWaves][4], float (&ms)[4]) {
  float M[2] = {kNegHuge, kNegHuge};
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    M[0] = fmaxf(M[0], part[w][0]);
    M[1] = fmaxf(M[1], part[w][2]);
  }
  float S[2] = {0.f, 0.f};
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    S[0] += part[w][1] * ex2(part[w][0] - M[0]);
    S[1] += part[w][3] * ex2(part[w][2] - M[1]);
  }
  ms[0] = M[0]; ms[1] = S[0]; ms[2] = M[1]; ms[3] = S[1];
}
// After the barrier every wavefront merges the quarters left in LDS (wave-uniform results).
__device__ __forceinline__ bool merge_quarters(const LdsBlock& sh, int par, float (&ms)[4]) {
  float part[kWaves][4];
  bool ok = true;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
#pragma unroll
    for (int x = 0; x < 4; ++x) part[w][x] = lane_value(sh.part[par][w][x], 0);
    ok = ok && __builtin_amdgcn_readfirstlane(sh.part_ok[par][w]) != 0;
  }
  merge4(part, ms);
  return ok;
}

// Bounded wait expired: the whole workgroup recomputes every wavefront's (m, s) pair of the position
// from memory, with the code the owners run (same values, same rounding), and folds them the same way.
template <int DT, int NV>
__device__ __noinline__ float4 recompute_norm(const char* prow, const char* qrow, int S, int chunk, int nv,
                                                 LdsBlock* shp, int par) {
  // a real call with everything passed by value: this path is almost never taken and must not cost
  // the pipeline registers or stack traffic
  LdsBlock& sh = *shp;
  PipeGeom g;
  g.S = S;
  g.chunk = chunk;
  g.nv = nv;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int o = 0; o < g.S; ++o) {
    Item one;
    one.prow = prow;
    one.qrow = qrow;
    one.s = o;
    Buf<NV> tmp;
    load_item<DT, NV>(one, g, tmp);
    Lse wp, wq;
    phase1<DT, NV>(one, g, tmp, wp, wq);
    if (lane == 0) {
      float* r = sh.redo[o * kWaves + wave];
      r[0] = wp.m; r[1] = wp.s; r[2] = wq.m; r[3] = wq.s;
    }
  }
  lds_barrier();
  const int idx = lane & 31, half = lane >> 5;
  const bool need = idx < g.S;
  const float* r = sh.redo[wave * g.S + (need ? idx : 0)];
  float out[4];
  fold_quarter(need ? r[2 * half] : kNegHuge, need ? r[2 * half + 1] : 0.f, out);
  if (lane == 0) {
#pragma unroll
    for (int x = 0; x < 4; ++x) sh.part[par][wave][x] = out[x];
    sh.part_ok[par][wave] = 1;
  }
  lds_barrier();
  float ms[4];
  merge_quarters(sh, par, ms);
  lds_barrier();                                   // sh.redo and sh.part[par] may be rewritten
  return make_float4(ms[0], ms[1], ms[2], ms[3]);
}

// Makes the compiler forget what it knows about the buffer's registers (no instruction is emitted).
// Without it the values unpacked in phase 1 are kept alive for phase 2, a tick later, instead of being
// unpacked again from the raw vectors: twice the registers across the hand-off.
template <int NV> __device__ __forceinline__ void forget(Buf<NV>& b) {
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    asm volatile("" : "+v"(b.p[j].x), "+v"(b.p[j].y), "+v"(b.p[j].z), "+v"(b.p[j].w));
    asm volatile("" : "+v"(b.q[j].x), "+v"(b.q[j].y), "+v"(b.q[j].z), "+v"(b.q[j].w));
  }
}

// What a wavefront carries from one tick to the next.
struct Carry {
  float ref_p, ref_q;   // phase-1 references of the item that is `nxt` in the coming tick
  float acc;            // per-lane phase-2 sum of the item that was `cur` in the last tick
  int acc_pos, acc_s;
  bool acc_valid;
};

__device__ __forceinline__ void publish_sum(const Carry& c, float A, const Workspace& ws) {
  if (c.acc_valid && (threadIdx.x & 63) == 0)
    put_pair(slot_of(ws, c.acc_pos, c.acc_s * kWaves + (threadIdx.x >> 6)) + 3, flagged(A), 0.f);
}

// One tick of the pipeline.  `cur` has been through phase 1 (buffer bc), `nxt` is loaded (buffer bn)
// and its references are known, `far` (decoded from `seed`) gets its loads issued into bf between
// the chunks of phase 1.
//
// The cross-lane reductions are long chains of dependent instructions, so each is placed next to
// element-wise work of another phase that it does not depend on, for the instruction scheduler to
// interleave: the fold of the siblings' results of `cur` next to the last chunk of phase 1 of `nxt`,
// the phase-1 sums of `nxt` next to phase 2 of `cur`, the phase-2 sum of `cur` next to the first
// chunk of phase 1 in the following tick.  Results are published in one place per tick.
//
// A position is finalised by the workgroup that owns slice (tick mod S) of it, two ticks after its
// phase 2: the duty moves from workgroup to workgroup, so nobody falls behind its siblings.
template <int DT, int NV>
__device__ __forceinline__ void tick(const RowMap& map, const PipeGeom& g, const Workspace& ws,
                                     LdsBlock& sh, Seed& seed,
                                     const Item& cur, const Buf<NV>& bc, const Item& nxt,
                                     Buf<NV>& bn, Item& far, Buf<NV>& bf, Carry& c, int tick_no) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, par = tick_no & 1;
  // what this tick reads from other workgroups is requested first, ahead of the prefetch
  uint64_t fw = 1ull;
  if (cur.valid) fw = get_word(fetch_address(cur, g, ws));
  far = decode_end<DT>(map, seed);
  seed = decode_begin(map, g, tick_no + 3);
  const SliceRange fr = slice_range(far.s, g);
  const bool need = (lane & 31) < g.S;

  // ---- phase 1 of `nxt`, chunk by chunk, with the loads of `far` in between
  P1Sums sums;
  float A_prev = 0.f, quarter[4] = {0.f, 0.f, 0.f, 0.f};
  bool fetched = true;
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    bf.p[j] = load_vec<DT>(far.prow, fr, j);
    bf.q[j] = load_vec<DT>(far.qrow, fr, j);
    __builtin_amdgcn_sched_barrier(0);
    p1_chunk<DT, NV>(bn, j, c.ref_p, c.ref_q, sums);
    if (j == 0) A_prev = wave_sum_f(c.acc);
    if (j == NV - 1) {
      fetched = __all(!need || (fw & 1ull));
      fold_quarter(need ? lo_float(fw) : kNegHuge, need ? hi_float(fw) : 0.f, quarter);
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  forget(bn);
  if (cur.valid) {
    bool got = true;
    if (!fetched) {
      got = fetch_retry(cur, g, ws, fw);
      fold_quarter(need ? lo_float(fw) : kNegHuge, need ? hi_float(fw) : 0.f, quarter);
    }
    if (lane == 0) {
#pragma unroll
      for (int x = 0; x < 4; ++x) sh.part[par][wave][x] = quarter[x];
      sh.part_ok[par][wave] = got ? 1 : 0;
    }
  }
  lds_barrier();
  // Two workgroups share a compute unit and the instruction arbiter favours the older wavefront: left
  // alone, one workgroup races ahead and the other is starved, then finishes on its own at a fraction
  // of the machine.  Raising the priority in one half of the tick makes the two take turns.
  __builtin_amdgcn_s_setprio(2);

  // ---- phase 2 of `cur`; the phase-1 sums of `nxt` are reduced alongside
  Norm n;
  n.cp = n.cq = n.dc = 0.f;
  n.ok = false;
  if (cur.valid) {
    float ms[4];
    if (!merge_quarters(sh, par, ms)) {
      const float4 r = recompute_norm<DT, NV>(cur.prow, cur.qrow, g.S, g.chunk, g.nv, &sh, par);
      ms[0] = r.x; ms[1] = r.y; ms[2] = r.z; ms[3] = r.w;
    }
    n = make_norm(ms[0], ms[1], ms[2], ms[3]);
  }
  Lse lp, lq;
  lp.m = c.ref_p;
  lq.m = c.ref_q;
  p1_reduce(sums, lp, lq);
  fix_suspect<DT, NV>(nxt, g, lp, lq);
  float acc = slice_jsd<DT, NV>(bc.p, bc.q, n.cp, n.cq, n.dc);
  acc = n.ok ? acc : 0.f;
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_setprio(0);

  // ---- everything this tick hands to other workgroups
  publish_sum(c, A_prev, ws);
  if (nxt.valid && lane == 0) {
    uint64_t* w = slot_of(ws, nxt.pos, nxt.s * kWaves + wave);
    put_pair(w + 0, lp.m, lp.s);
    put_pair(w + 1, lq.m, lq.s);
    put_pair(w + 2, flagged(lp.u), lq.u);
  }
  c.acc = acc;
  c.acc_pos = cur.pos;
  c.acc_s = cur.s;
  c.acc_valid = cur.valid;
  // references for the next tick's phase 1 (the loads of `far` are the youngest: last)
  p1_refs<DT, NV, true>(bf, c.ref_p, c.ref_q);
}

template <int DT, int NV>
__global__ void __launch_bounds__(kBlock, NV == 2 ? 3 : 2)
k_stats_pipe(RowMap map, PipeGeom g, Workspace ws) {
  warm_kernargs<sizeof(RowMap) + sizeof(PipeGeom) + sizeof(Workspace)>();
  __shared__ LdsBlock sh;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int ticks = (g.items + (int)gridDim.x - 1) / (int)gridDim.x;
  Buf<NV> b0, b1, b2;
  Item i0 = decode_end<DT>(map, decode_begin(map, g, 0));
  Item i1 = decode_end<DT>(map, decode_begin(map, g, 1)), i2;
  Seed seed = decode_begin(map, g, 2);
  Carry c;
  c.acc = 0.f;
  c.acc_pos = c.acc_s = 0;
  c.acc_valid = false;
  load_item<DT, NV>(i0, g, b0);
  load_item<DT, NV>(i1, g, b1);
  {
    Lse lp, lq;
    phase1<DT, NV>(i0, g, b0, lp, lq);
    if (i0.valid && lane == 0) {
      uint64_t* w = slot_of(ws, i0.pos, i0.s * kWaves + wave);
      put_pair(w + 0, lp.m, lp.s);
      put_pair(w + 1, lq.m, lq.s);
      put_pair(w + 2, flagged(lp.u), lq.u);
    }
  }
  forget(b0);
  __builtin_amdgcn_sched_barrier(0);
  p1_refs<DT, NV, true>(b1, c.ref_p, c.ref_q);
  for (int tick_no = 0; tick_no < ticks; tick_no += 3) {
    tick<DT, NV>(map, g, ws, sh, seed, i0, b0, i1, b1, i2, b2, c, tick_no);
    tick<DT, NV>(map, g, ws, sh, seed, i1, b1, i2, b2, i0, b0, c, tick_no + 1);
    tick<DT, NV>(map, g, ws, sh, seed, i2, b2, i0, b0, i1, b1, c, tick_no + 2);
  }
  publish_sum(c, wave_sum_f(c.acc), ws);
}

// Finalisation, one wavefront per position, after the pipeline kernel has finished: fold the 4S
// published results, form entropies and the distance in double precision, clear the position's words
// for the next call.  The float normalisers that weighted the phase-2 sums are formed again with the
// pipeline's own folding code (same values), for the first-order correction of the common scale.
__global__ void __launch_bounds__(kBlock) k_stats_finish(RowMap map, PipeGeom g, Workspace ws, VerifyOut vout) {
  warm_kernargs<sizeof(RowMap) + sizeof(PipeGeom) + sizeof(Workspace) + sizeof(VerifyOut)>();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, E = g.S * kWaves;
  const int pos = blockIdx.x * kWaves + wave;
  if (pos >= g.P) return;
  const int b = pos / map.K, i = pos - b * map.K;
  const int kb = map.draft_len ? min(max(map.draft_len[b], 0), map.K) : map.K;
  if (i >= kb) return;
  // the normalisers as phase 2 saw them
  float part[kWaves][4];
  const int idx = lane & 31;
  const bool need = idx < g.S;
  bool complete = true;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    const uint64_t x = get_word(slot_of(ws, pos, w * g.S + (need ? idx : 0)) + (lane >> 5));
    complete = complete && __all(!need || (x & 1ull));
    fold_quarter(need ? lo_float(x) : kNegHuge, need ? hi_float(x) : 0.f, part[w]);
  }
  float ms[4];
  merge4(part, ms);
  const Norm n = make_norm(ms[0], ms[1], ms[2], ms[3]);
  // full triples and the phase-2 sum
  Lse tp[2], tq[2];
  double sum = 0.0;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int e = lane + h * kWave;
    uint64_t w[4];
    uint64_t* src = slot_of(ws, pos, e < E ? e : 0);
#pragma unroll
    for (int x = 0; x < 4; ++x) w[x] = get_word(src + x);
    const bool valid = (w[0] & w[1] & w[2] & w[3] & 1ull) != 0;
    complete = complete && __all(e >= E || valid);
    const bool have = e < E && valid;
    tp[h] = have ? Lse{lo_float(w[0]), hi_float(w[0]), lo_float(w[2])} : lse_empty();
    tq[h] = have ? Lse{lo_float(w[1]), hi_float(w[1]), hi_float(w[2])} : lse_empty();
    sum += have ? (double)lo_float(w[3]) : 0.0;
    if (e < E) {
#pragma unroll
      for (int x = 0; x < 4; ++x) clear_word(src + x);
    }
  }
  const Lse fp = wave_fold(tp[0], tp[1]), fq = wave_fold(tq[0], tq[1]);
  const double A = wave_sum(sum);
  if (lane != 0) return;
  RowResult rp, rq;
  float d_out = NAN;
  const bool okp = lse_ok(fp) && complete, okq = lse_ok(fq) && complete;
  const double l2p = log2((double)fp.s), l2q = log2((double)fq.s);
  rp.lse2 = okp ? (double)fp.m + l2p : NAN;
  rq.lse2 = okq ? (double)fq.m + l2q : NAN;
  rp.H = okp ? (float)(kLn2 * (l2p - (double)fp.u / (double)fp.s)) : NAN;
  rq.H = okq ? (float)(kLn2 * (l2q - (double)fq.u / (double)fq.s)) : NAN;
  rp.bad = !okp;
  rq.bad = !okq;
  if (okp && okq && n.ok) {
    const double a = kLn2 * (rp.lse2 - (double)n.cp), a2 = kLn2 * (rq.lse2 - (double)n.cq);
    double D = 0.5 * A * (1.0 - 0.5 * (a + a2));
    D = fmin(fmax(D, 0.0), 1.0);
    d_out = (float)sqrt(D);
  }
  ws.rows[2 * pos] = rp;
  ws.rows[2 * pos + 1] = rq;
  if (vout.H_p) vout.H_p[pos] = rp.H;
  vout.H_q[pos] = rq.H;
  vout.d_js[pos] = d_out;
}

template <int DT, int NV> int max_resident_groups() {
  static int cached = 0;
  if (!cached) {
    int dev = 0, per_cu = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_stats_pipe<DT, NV>, kBlock, 0) != hipSuccess)
      return 0;
    cached = per_cu * prop.multiProcessorCount;
  }
  return cached;
}

template <int DT, int NV>
hipError_t launch_pipe(const RowMap& map, PipeGeom g, const Workspace& ws, const VerifyOut& vout, hipStream_t st) {
  const int unit = kXcd * g.S;                         // siblings must share a tick
  int cap = max_resident_groups<DT, NV>();
  int G = cap / unit * unit;
  if (G < unit) G = unit;
  if (G > g.items) G = g.items;
  // balance: same number of ticks, smallest grid that achieves it
  const int ticks = (g.items + G - 1) / G;
  const int need = (g.items + ticks - 1) / ticks;
  G = (need + unit - 1) / unit * unit;
  g.pos_step = G / g.S;
  launch_kernel((k_stats_pipe<DT, NV>), dim3(G), dim3(kBlock), st, map, g, ws);
  launch_kernel(k_stats_finish, dim3((g.P + kWaves - 1) / kWaves), dim3(kBlock), st, map, g, ws, vout);
  return hipGetLastError();
}

}  // namespace

// Can the fused kernel take this call, and with which tiling?  Requirements: every row starts on a
// 16-byte boundary, the vocabulary is a whole number of vectors, and at most kMaxFusedSplit slices.
bool fused_plan(const RowMap& map, int dt, int* NV_out, int* S_out) {
  const int es = dt == ADASD_BF16 ? 2 : 4, epv = 16 / es;
  if (map.K <= 0 || map.V % epv != 0) return false;
  for (int w = 0; w < 2; ++w) {
    if (reinterpret_cast<uintptr_t>(map.base[w]) % 16 != 0) return false;
    if ((map.seq_stride[w] * es) % 16 != 0 || (map.pos_stride[w] * es) % 16 != 0) return false;
  }
  const int nv = map.V / epv;
  int NV = 4;
  int S = (nv + NV * kBlock - 1) / (NV * kBlock);
  while (S * kWaves > kMaxFusedSplit && NV < 8) {
    NV *= 2;
    S = (nv + NV * kBlock - 1) / (NV * kBlock);
  }
  if (S * kWaves > kMaxFusedSplit) return false;
  *NV_out = NV;
  *S_out = S;
  return true;
}

hipError_t launch_stats_fused(const RowMap& map, int dt, int NV, int S, int spin_limit,
                              const Workspace& ws, const VerifyOut& vout, hipStream_t st) {
  PipeGeom g;
  g.S = S;
  g.nv = map.V / (dt == ADASD_BF16 ? 8 : 4);
  g.P = map.B * map.K;
  g.items = (g.P + kXcd - 1) / kXcd * kXcd * S;
  g.chunk = (g.nv + S - 1) / S;
  g.pos_step = 0;
  g.spin_limit = spin_limit;
  if (g.P <= 0) return hipSuccess;
#define ADASD_PIPE_CASE(DTV, NVV) \
  if (dt == DTV && NV == NVV) return launch_pipe<DTV, NVV>(map, g, ws, vout, st);
  ADASD_PIPE_CASE(ADASD_BF16, 2) ADASD_PIPE_CASE(ADASD_BF16, 4) ADASD_PIPE_CASE(ADASD_BF16, 8)
  ADASD_PIPE_CASE(ADASD_F32, 2) ADASD_PIPE_CASE(ADASD_F32, 4) ADASD_PIPE_CASE(ADASD_F32, 8)
#undef ADASD_PIPE_CASE
  return hipErrorInvalidValue;
}

}  // namespace adasd
