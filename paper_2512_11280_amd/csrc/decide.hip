// Acceptance decisions of one round (Section 2.1.3, Section 4.4 and the verification loop of
// Algorithm 1 of the paper) and the update of the adaptive state (Section 4.3; update lines).
#include "decide_device.h"
#include "internal.h"

namespace adasd {

namespace {

template <int DT>
__global__ void __launch_bounds__(kBlock) k_decide(DecideArgs a, Workspace ws) {
  warm_kernargs<sizeof(DecideArgs) + sizeof(Workspace)>();
  __shared__ DecideShared sh;
  decide_sequence<DT>(a, ws, blockIdx.x, sh);
}

// ---------------------------------------------------------------------------------------------
// Update step: one wavefront per sequence, one lane per candidate position (k_max <= 64).  Every lane
// reads its position's distance at once; accepted positions that pass the open-interval filter are
// appended in position order (rank = number of passing positions before it, from a ballot).
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(64) k_update(UpdateArgs a) {
  warm_kernargs<sizeof(UpdateArgs)>();
  const int b = blockIdx.x, lane = threadIdx.x;
  int kb = a.K;
  if (a.draft_len) kb = min(max(a.draft_len[b], 0), a.K);
  const int r = min(max(a.n_accept[b], 0), kb);
  const int nA = a.nA[b], nR = a.nR[b];
  const float lo = a.d_eps, hi = 1.0f - a.d_eps;
  float d = 0.f, H = 0.f;
  if (lane <= r && lane < kb) d = a.d_js[(size_t)b * a.K + lane];
  if (lane == r && r < kb) H = a.H_q[(size_t)b * a.K + r];
  const bool pass = d > lo && d < hi;                       // NaN fails both comparisons
  uint32_t st = 0;
  // accepted positions 0 .. r-1
  const unsigned long long acc = __ballot(pass && lane < r);
  if (pass && lane < r) {
    const int slot = nA + __popcll(acc & ((1ull << lane) - 1ull));
    if (slot < a.cap) a.LA[(size_t)b * a.cap + slot] = d;
  }
  const int nA_new = min(nA + __popcll(acc), a.cap);
  if (nA + __popcll(acc) > a.cap) st |= ADASD_ST_OVERFLOW;
  // the lane of the rejected position finishes the sequence (with all 64 positions accepted: the last lane)
  if (lane != (r < 64 ? r : 63)) return;
  int nR_new = nR;
  if (r < kb) {
    if (isfinite(H)) {
      a.ent_sum[b] += (double)H;
      a.ent_cnt[b] += 1;
    }
    if (pass) {
      if (nR < a.cap) a.LR[(size_t)b * a.cap + nR_new++] = d;
      else st |= ADASD_ST_OVERFLOW;
    }
  }
  a.nA[b] = nA_new;
  a.nR[b] = nR_new;
  const int cnt = a.ent_cnt[b];
  a.T_G[b] = cnt > 0 ? (float)(a.ent_sum[b] / (double)cnt) : 0.f;
  if (a.status && st) a.status[b] |= st;
}

__global__ void __launch_bounds__(64) k_state_init(UpdateArgs a) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= a.B) return;
  a.T_G[b] = 0.f;
  a.ent_sum[b] = 0.0;
  a.ent_cnt[b] = 0;
  a.nA[b] = 0;
  a.nR[b] = 0;
}

__global__ void __launch_bounds__(256) k_zero(uint32_t* p, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = 0u;
}

}  // namespace

hipError_t launch_decide(const DecideArgs& a, const Workspace& ws, hipStream_t st) {
  if (a.map.B <= 0) return hipSuccess;
  if (a.dt == ADASD_BF16)
    launch_kernel(k_decide<ADASD_BF16>, dim3(a.map.B), dim3(kBlock), st, a, ws);
  else
    launch_kernel(k_decide<ADASD_F32>, dim3(a.map.B), dim3(kBlock), st, a, ws);
  return hipGetLastError();
}

hipError_t launch_update(const UpdateArgs& a, hipStream_t st) {
  if (a.B <= 0) return hipSuccess;
  launch_kernel(k_update, dim3(a.B), dim3(64), st, a);
  return hipGetLastError();
}

hipError_t launch_state_init(const UpdateArgs& a, hipStream_t st) {
  if (a.B <= 0) return hipSuccess;
  launch_kernel(k_state_init, dim3((a.B + 63) / 64), dim3(64), st, a);
  return hipGetLastError();
}

hipError_t launch_zero(void* p, size_t bytes, hipStream_t st) {
  const size_t n = bytes / 4;
  if (n == 0) return hipSuccess;
  int blocks = (int)((n + 255) / 256);
  if (blocks > 1024) blocks = 1024;
  launch_kernel(k_zero, dim3(blocks), dim3(256), st, (uint32_t*)p, n);
  return hipGetLastError();
}

}  // namespace adasd
