// Device helpers of the vocabulary-wide statistics (Appendix A of the paper: softmax and entropy),
// shared by the statistics kernels and the drafting step.
#pragma once
#include "internal.h"

namespace adasd {

struct RowRef {
  const char* ptr;
  int b, i, which;
  bool active;
};

template <int DT>
__device__ __forceinline__ RowRef locate_row(const RowMap& map, int rho) {
  RowRef r;
  if (map.K > 0) {
    r.which = rho & 1;
    int pos = rho >> 1;
    r.b = pos / map.K;
    r.i = pos - r.b * map.K;
    int kb = map.K;
    if (map.draft_len && !map.slots) kb = min(max(map.draft_len[r.b], 0), map.K);   // (a packed slot list only names positions inside their windows)
    r.active = r.i < kb;
  } else {
    r.which = 0;
    r.b = rho;
    r.i = 0;
    r.active = map.active ? (map.active[rho] != 0) : true;
  }
  int64_t off = (int64_t)r.b * map.seq_stride[r.which] + (int64_t)r.i * map.pos_stride[r.which];
  r.ptr = map.base[r.which] + off * Elem<DT>::bytes;
  return r;
}

// The candidate position that the m-th position slot of a launch works on, or -1 for none.  With ragged
// windows (draft_len given) the positions past a window's end have no work and their workgroups leave at
// once; in storage order they recur with period k_max, and the placement of consecutive workgroups on
// consecutive compute units turns that period into compute units without work (measured: the JS kernel
// took as long for half-length windows as for full ones).  So the slots either follow a packed list of
// the positions that have work (map.slots), or, without one, run over the sequences first and the
// window position second, which at least moves the empty positions to the end of the dispatch order.
__device__ __forceinline__ int position_of_slot(const RowMap& map, int m) {
  if (!map.draft_len) return m;
  if (map.slots) return map.slots[m];
  const int i = m / map.B, b = m - i * map.B;
  return b * map.K + i;
}

// Vectors per slice of a row of nv vectors cut into S slices: a multiple of the workgroup size where the
// last slice then still has work, so that all slices but the last consist of whole batches (no lane is
// ever past the end there, and the loads need neither clamping nor masking).
__device__ __forceinline__ int slice_vectors(int nv, int S) {
  const int chunk = (nv + S - 1) / S;
  const int rounded = (chunk + kBlock - 1) / kBlock * kBlock;
  return (int64_t)rounded * (S - 1) < nv ? rounded : chunk;
}

__device__ __forceinline__ bool aligned16(const void* p) {
  return (reinterpret_cast<uintptr_t>(p) & 15u) == 0;
}

// One element of the row joins the running state (reference raised first if needed).
__device__ __forceinline__ void lse_push(Lse& st, float z) {
  lse_raise(st, z * kLog2e);
  lse_add(st, z);
}

// Fold of up to 64 partial states of one row held one per lane (an empty state in the other lanes), by
// one wavefront; all lanes return the same: common reference, plain sums, then the row's log2-sum-exp
// and entropy in double precision.
__device__ __forceinline__ RowResult fold_lanes(const Lse& t) {
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

// Fold of the S slice results that the first statistics kernel left for one row.
__device__ __forceinline__ RowResult fold_row(const Workspace& ws, int rho, int S) {
  const int lane = threadIdx.x & 63;
  Lse t = lse_empty();
  if (lane < S) {
    const float4 p = ws.part1[(size_t)rho * kMaxSplit + lane];
    t = Lse{p.x, p.y, p.z};
  }
  return fold_lanes(t);
}

// What the JS sum of a position needs of its two rows' normalisers: their float roundings (the weights
// are formed with those; the decision stage corrects the common scale afterwards) and their difference.
// Softmax does not see a row's offset, so the two rows may carry very different ones; `far` marks such a
// position (normalisers more than 8 units of log2 apart).  There the element's log ratio, a small number
// where it matters, must not be formed as the difference of two large ones: each logit is first taken
// relative to its own row's offset (op, oq: the row's log-sum-exp in nats rounded to float, 0 for a row
// whose offset is below 32: next to a large offset z - o is exact for every element of any weight), the
// difference of the two is kept with its rounding error (two floats), and so is the rest of the
// normalisers' difference.  The factor log2(e) is the SAME float constant everywhere, in the normalisers
// (which are log2 sum 2^(z k) with k that constant) and in the element's log ratio: what comes out is the
// log ratio of the two distributions at a temperature k / log2(e) = 1 - 1.3e-8, a relative change of that
// size.  (Correcting the constant in one place only, e.g. with its low part here, would put 1.3e-8 of a
// row's offset into every log ratio: 3.7e-6 at an offset of 193 nats, which showed in the distance of two
// one-hot rows that far apart.)
struct JsNorm {
  float cp, cq, dc_hi, dc_lo, op, oq;
  int far;
};
__device__ __forceinline__ JsNorm js_norm(const RowResult& rp, const RowResult& rq) {
  JsNorm n;
  n.cp = (float)rp.lse2;
  n.cq = (float)rq.lse2;
  double dc = rq.lse2 - rp.lse2;
  n.far = !(fabs(dc) <= 8.0);
  n.op = n.oq = 0.f;
  if (n.far) {
    const double lp = rp.lse2 * kLn2, lq = rq.lse2 * kLn2;
    n.op = fabs(lp) >= 32.0 ? (float)lp : 0.f;
    n.oq = fabs(lq) >= 32.0 ? (float)lq : 0.f;
    dc -= ((double)n.oq - (double)n.op) * (double)kLog2e;   // (the float constant: see below)
  }
  n.dc_hi = (float)dc;
  n.dc_lo = n.far ? (float)(dc - (double)n.dc_hi) : 0.f;
  return n;
}

// ---------------------------------------------------------------------------------------------
// One element of the Jensen-Shannon sum (Section 2.2 of the paper), in bits.  With b = max(p,q),
// delta = log2 q - log2 p and r = min(p,q)/max(p,q) = 2^-|delta|,
//     p log2(p/m) + q log2(q/m) = b * ( r * log2 r - (1 + r) * log2((1 + r)/2) ),   m = (p+q)/2,
// which is non-negative, symmetric in (p,q), never overflows (r <= 1) and keeps every logarithm at
// magnitude <= 1.  delta is formed from the exact logit difference.  For small |delta| the bracket is
// the difference of two nearly equal numbers (it is ~ (ln2/4) delta^2) and the rounding of (1+r)/2
// alone leaves an absolute error of ~1e-7: there it is taken from its series instead.  With
// s = |delta| ln2 / 2 the bracket equals (1 + r) (s tanh s - ln cosh s) / ln 2, and
//     s tanh s - ln cosh s = s^2/2 - s^4/4 + s^6/9 - ...      (next term 4e-8 relative at |delta| = 1/4)
// is a polynomial in the exactly formed delta^2, so the term keeps RELATIVE accuracy however close the
// two rows are (identical rows give exactly 0).
// ---------------------------------------------------------------------------------------------
constexpr float kJsC0 = 0.17328679513998632735f;     // 2 * ln2 / 8        (the 2: 1 + r = 2 h below)
constexpr float kJsC1 = -0.010407020374654045f;      // -2 * ln2^3 / 64
constexpr float kJsC2 = 0.0005555649227678517f;      // 2 * ln2^5 / 576
constexpr float kJsSmall = 0.25f;


template <bool FAR>
__device__ __forceinline__ void jsd_push(float zp, float zq, const JsNorm& n, float& acc) {
  const float yp = fmaf(zp, kLog2e, -n.cp), yq = fmaf(zq, kLog2e, -n.cq);   // log2 p, log2 q
  const float b = ex2(fmaxf(yp, yq));
  float delta;
  if (FAR) {
    const float a = zq - n.oq, c = n.op - zp;               // delta = (a + c) log2(e) - dc
    const float hi = a + c, t = hi - a;
    const float lo = (a - (hi - t)) + (c - t);              // a + c = hi + lo exactly
    delta = fmaf(hi, kLog2e, -n.dc_hi) + fmaf(lo, kLog2e, -n.dc_lo);
  } else {
    delta = fmaf(zq - zp, kLog2e, -n.dc_hi);
  }
  const float nd = fmaxf(-fabsf(delta), -126.0f);   // masked logits (delta = +-inf or NaN) end up at r = 2^-126
  const float r = ex2(nd);
  const float h = fmaf(r, 0.5f, 0.5f);
  const float t_log = fmaf(-2.0f, h * lg2(h), r * nd);
  const float d2 = nd * nd;
  const float t_series = fmaf(d2, fmaf(d2, kJsC2, kJsC1), kJsC0) * d2 * h;
  acc = fmaf(b, nd > -kJsSmall ? t_series : t_log, acc);
}

}  // namespace adasd
