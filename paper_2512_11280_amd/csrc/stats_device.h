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

// Fold of the S slice results of one row by one wavefront (all lanes return the same): common
// reference, plain sums, then the row's log2-sum-exp and entropy in double precision.
__device__ __forceinline__ RowResult fold_row(const Workspace& ws, int rho, int S) {
  const int lane = threadIdx.x & 63;
  Lse t = lse_empty();
  if (lane < S) {
    const float4 p = ws.part1[(size_t)rho * kMaxSplit + lane];
    t = Lse{p.x, p.y, p.z};
  }
  const float M = wave_max_f(t.m), d = t.m - M, f = ex2(d);
  const float sw = wave_sum_f(t.s * f), uw = wave_sum_f((t.u + d * t.s) * f);
  const bool ok = (sw > 0.f) && (sw < INFINITY) && (fabsf(uw) < INFINITY) && (M > kNegHuge) && (M < INFINITY);
  RowResult res;
  if (ok) {
    const double l2s = log2_acc(sw);
    res.lse2 = (double)M + l2s;
    res.H = (float)(kLn2 * (l2s - (double)uw / (double)sw));
    res.bad = 0;
  } else {
    res.lse2 = NAN;
    res.H = NAN;
    res.bad = 1;
  }
  return res;
}


}  // namespace adasd
