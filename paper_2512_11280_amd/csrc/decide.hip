// Acceptance decisions of one round (Section 2.1.3, Section 4.4 and the verification loop of
// Algorithm 1 of the paper) and the update of the adaptive state (Section 4.3; update lines).
#include "decide_device.h"
#include "internal.h"

namespace adasd {

namespace {

template <int DT, bool INLOOP>
__global__ void __launch_bounds__(kBlock) k_decide(DecideArgs a, UpdateArgs upd, Workspace ws) {
  warm_kernargs<sizeof(DecideArgs) + sizeof(UpdateArgs) + sizeof(Workspace)>();
  __shared__ DecideShared sh;
  decide_sequence<DT, INLOOP>(a, ws, blockIdx.x, sh);
  // the round applied to the state right away (the lists were only read above)
  if (upd.B > 0 && threadIdx.x < 64) update_sequence_shared(upd, blockIdx.x, threadIdx.x, sh.first_reject, sh.k_b, sh);
}

// Long histories: one workgroup per candidate position.  The workgroup of position 0 does all the work of
// a sequence whose lists are still short and the others leave at once, so with more workgroups than the
// chip holds at a time those of position 0 have to come first in dispatch order or they queue behind the
// idle ones: grid (sequences, k_max).  A launch that gives every workgroup a compute unit of its own
// measured 0.4 us faster the other way round (grid (k_max, sequences)); `seq_first` says which it is.
template <int DT, bool INLOOP>
__global__ void __launch_bounds__(kBlock) k_decide_wide(DecideArgs a, UpdateArgs upd, Workspace ws, int seq_first) {
  warm_kernargs<sizeof(DecideArgs) + sizeof(UpdateArgs) + sizeof(Workspace) + sizeof(int)>();
  __shared__ DecideShared sh;
  __shared__ WideShared wsh;
  const int b = seq_first ? blockIdx.x : blockIdx.y, pos = seq_first ? blockIdx.y : blockIdx.x;
  // The launch is sized for long lists (the host only knows their capacity); a sequence whose lists are
  // still short is cheaper in the one-workgroup form, so its first workgroup takes that and the others leave.
  const int n_long = min(max(max(a.nA[b], a.nR[b]), 0), a.cap);
  if (n_long < kWideMin) {
    if (pos != 0) return;
    decide_sequence<DT, INLOOP>(a, ws, b, sh);
    if (upd.B > 0 && threadIdx.x < 64) update_sequence_shared(upd, b, threadIdx.x, sh.first_reject, sh.k_b, sh);
    return;
  }
  decide_position_wide<DT, INLOOP>(a, upd, ws, ws.pos_rec, b, pos, sh, wsh);
}

// ---------------------------------------------------------------------------------------------
// Update step: one wavefront per sequence, one lane per candidate position (k_max <= 64).  Every lane
// reads its position's distance at once; accepted positions that pass the open-interval filter are
// appended in position order (rank = number of passing positions before it, from a ballot).
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(64) k_update(UpdateArgs a) {
  warm_kernargs<sizeof(UpdateArgs)>();
  const int b = blockIdx.x;
  int kb = a.K;
  if (a.draft_len) kb = min(max(a.draft_len[b], 0), a.K);
  const int r = min(max(a.n_accept[b], 0), kb);
  update_sequence(a, b, threadIdx.x, r, kb);
}

__global__ void __launch_bounds__(64) k_state_init(UpdateArgs a) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= a.B) return;
  a.T_G[b] = 0.f;
  a.ent_sum[b] = 0.0;
  a.ent_cnt[b] = 0;
  a.nA[b] = 0;
  a.nR[b] = 0;
  if (a.mom)
    for (int x = 0; x < 4; ++x) a.mom[4 * b + x] = 0.0;
}

// Running sums of both lists of one sequence from scratch (one workgroup per sequence).
__global__ void __launch_bounds__(kBlock) k_state_refresh(UpdateArgs a) {
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nA = min(max(a.nA[b], 0), a.cap), nR = min(max(a.nR[b], 0), a.cap);
  const float* LA = a.LA + (size_t)b * a.cap;
  const float* LR = a.LR + (size_t)b * a.cap;
  const double cA = nA > 0 ? (double)LA[0] : 0.0, cR = nR > 0 ? (double)LR[0] : 0.0;
  double m[4] = {0.0, 0.0, 0.0, 0.0};
  for (int j = tid; j < nA; j += kBlock) {
    const double e = (double)LA[j] - cA;
    m[0] += e;
    m[1] += e * e;
  }
  for (int j = tid; j < nR; j += kBlock) {
    const double e = (double)LR[j] - cR;
    m[2] += e;
    m[3] += e * e;
  }
  __shared__ double sh[kWaves][4];
#pragma unroll
  for (int x = 0; x < 4; ++x) {
    m[x] = half_sum_d(m[x]);
    m[x] += __shfl_xor(m[x], 32);
  }
  if (lane == 0)
    for (int x = 0; x < 4; ++x) sh[wave][x] = m[x];
  __syncthreads();
  if (tid < 4) a.mom[4 * b + tid] = (sh[0][tid] + sh[1][tid]) + (sh[2][tid] + sh[3][tid]);
}

__global__ void __launch_bounds__(256) k_zero(uint32_t* p, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = 0u;
}

}  // namespace

hipError_t launch_decide(const DecideArgs& a, const UpdateArgs& upd, const Workspace& ws, hipStream_t st) {
  if (a.map.B <= 0) return hipSuccess;
  const dim3 block(kBlock);
  if (a.cap >= kWideCap && a.map.K > 0 && !a.relaxed_off && a.LA && a.LR && a.nA && a.nR) {
    const int lead = a.map.B * a.map.K > 256 ? 1 : 0;   // (256 compute units)
    const dim3 grid(lead ? a.map.B : a.map.K, lead ? a.map.K : a.map.B);
    if (a.dt == ADASD_BF16) {
      if (a.list_update) launch_kernel(k_decide_wide<ADASD_BF16, true>, grid, block, st, a, upd, ws, lead);
      else launch_kernel(k_decide_wide<ADASD_BF16, false>, grid, block, st, a, upd, ws, lead);
    } else {
      if (a.list_update) launch_kernel(k_decide_wide<ADASD_F32, true>, grid, block, st, a, upd, ws, lead);
      else launch_kernel(k_decide_wide<ADASD_F32, false>, grid, block, st, a, upd, ws, lead);
    }
    return hipGetLastError();
  }
  const dim3 grid(a.map.B);
  if (a.dt == ADASD_BF16) {
    if (a.list_update) launch_kernel(k_decide<ADASD_BF16, true>, grid, block, st, a, upd, ws);
    else launch_kernel(k_decide<ADASD_BF16, false>, grid, block, st, a, upd, ws);
  } else {
    if (a.list_update) launch_kernel(k_decide<ADASD_F32, true>, grid, block, st, a, upd, ws);
    else launch_kernel(k_decide<ADASD_F32, false>, grid, block, st, a, upd, ws);
  }
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

hipError_t launch_state_refresh(const UpdateArgs& a, hipStream_t st) {
  if (a.B <= 0 || !a.mom) return hipSuccess;
  launch_kernel(k_state_refresh, dim3(a.B), dim3(kBlock), st, a);
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
