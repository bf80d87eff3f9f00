// Host-side declarations shared by the translation units of libadasd.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/adasd.h"
#include <hip/hip_ext.h>

#include "device_common.h"

namespace adasd {

constexpr int kWideCap = 512;       // list capacity from which the decision stage is launched with a workgroup per position
constexpr int kSumsMin = 4096;      // list length from which the state's running sums are kept and used
constexpr int kWideMin = 384;       // list length from which a sequence actually uses them
constexpr int kNarrowMax = kWideCap; // so the one-workgroup form never sees a longer list: it stages both in shared memory
constexpr int kMaxSplit = 64;        // vocabulary slices per row (statistics kernels)
constexpr int kMaxSampleSplit = 128; // vocabulary slices per sequence (sampling kernel)
constexpr int kXchgWords = 3;        // 64-bit hand-off words per (position, slice) of the single-read statistics kernel
constexpr int kWaitPolls = 16384;    // polls (about 25 ms) before a workgroup of that kernel stops waiting for the others

// Where the rows of one call live.  which = 0: target, 1: draft.
struct RowMap {
  const char* base[2];
  int64_t seq_stride[2], pos_stride[2];  // elements
  const int32_t* draft_len;              // [B] or null
  const uint8_t* active;                 // [B] or null (draft-entropy mode)
  const int32_t* slots;                  // [B*K] or null: the candidate positions inside their windows, packed
                                         // (window position first, sequence second), -1 behind them
  int32_t K;                             // k_max; 0 selects draft-entropy mode (one row per sequence)
  int32_t B, V;
};

struct Workspace {
  float4* part1;      // [rows][kMaxSplit]   (m, s, u, -) partial log-sum-exp states
  int32_t* ticket1;   // [kTicket1Len]       arrival counters of the drafting kernel (row rho at rho * ticket_stride), zero between calls
  RowResult* rows;    // [rows]
  float2* part2;      // [positions][kMaxSplit] partial KL sums (p side, q side), log2 units
  int32_t* ticket2;   // [kTicket2Len]       arrival counters of the long-history decision kernel, zero between calls
  SamplePlan* plan;   // [B]
  Top2* part3;        // [B][kMaxSampleSplit]
  int32_t* ticket3;   // [kTicket3Len]       arrival counters of the sampling kernel, zero between calls
  uint64_t* xchg;     // [positions][kMaxSplit][kXchgWords] self-validating hand-off words of the single-read statistics
                      // kernel (two floats each, valid flag in the lowest mantissa bit of the low one), zero between calls
  PosRecord* pos_rec; // [positions] outcomes of the positions (long-history decision kernel)
  float2* tok;        // [positions] logits of the drafted tokens (looked up by the JS kernel or by the column shards)
  int32_t* slots;     // [positions] packed list of the positions inside their windows (ragged calls)
  size_t bytes;
};

// Region offsets depend only on the size of the workspace (not on the shape of the call), so calls of
// different shapes can share one workspace: counters and hand-off words are always found where the
// previous call left them zeroed.  Returns the number of positions the workspace can serve.
size_t workspace_bytes_for(size_t positions);
size_t workspace_layout(size_t ws_bytes, Workspace* ws, void* base);

// Arrival counters of different rows / sequences sit on different 128-byte lines while the array is long
// enough (read-modify-writes on one line are served one after the other, whatever word they hit).
__host__ __device__ inline int ticket_stride(int count, int capacity) {
  int st = count > 0 ? capacity / count : 32;
  return st > 32 ? 32 : (st < 1 ? 1 : st);
}
constexpr int kTicket1Len = 65536, kTicket2Len = 32768, kTicket3Len = 32768;

struct DraftOut {     // draft-entropy epilogue
  const float* T_G;
  float* H_out;
  uint8_t* stop_out;
  int32_t force_stop; // step + 1 >= k_max
};

struct DraftDraw {    // token draw of a drafting step (x_i ~ q_i)
  uint32_t seed_lo, seed_hi;
  const uint32_t* seq_id;
  const uint32_t* round;
  uint32_t round0;
  uint32_t step;
  int32_t* token_out;
  uint32_t* status;   // may be null
};
// One drafting call: entropy and stop flag of each row, and with `draw` the drawn token (one kernel)
int pick_draft_split(int rows, int V, int dt);
hipError_t launch_draft_step(const RowMap& map, int dt, int S, const Workspace& ws, const DraftOut& dout,
                             const DraftDraw* draw /* or null */, hipStream_t st);

struct VerifyOut {
  float* H_p;
  float* H_q;
  float* d_js;
  // With both set, the JS kernel also looks up the two logits of each position's drafted token and leaves
  // them in tok[position], so the decision kernel does not start with a chain of two dependent loads.
  const int32_t* tokens;   // [positions] or null
  float2* tok;             // [positions] or null
};

// Kernel launches go through launch_kernel: while kernel timing is enabled and a timing scope is open,
// the launch carries a pair of events that the dispatch itself stamps at its start and end (the same
// timestamps a profiler reports), so the measured durations hold no launch or queueing time.
bool profile_take_events(hipEvent_t* start, hipEvent_t* stop);
template <class Kernel, class... Args>
inline void launch_kernel(Kernel kernel, dim3 grid, dim3 block, hipStream_t st, Args... args) {
  hipEvent_t e0, e1;
  if (profile_take_events(&e0, &e1))
    hipExtLaunchKernelGGL(kernel, grid, block, 0, st, e0, e1, 0, args...);
  else
    hipLaunchKernelGGL(kernel, grid, block, 0, st, args...);
}

int pick_split(int rows, int V, int dt);

// Ragged windows: the positions i < draft_len[b] of all sequences, packed into slots[0 .. n) in the order
// (window position, sequence), -1 in the remaining slots up to B*K (one small kernel).
hipError_t launch_pack_slots(const int32_t* draft_len, int B, int K, int32_t* slots, hipStream_t st);

// plain streaming read (diagnostics): one word per workgroup goes to `sink`
size_t stream_read_groups(size_t bytes);
hipError_t launch_stream_read(const void* src, size_t bytes, uint32_t* sink, hipStream_t st);

hipError_t launch_rowstats(const RowMap& map, int dt, int rows, int S, const Workspace& ws, hipStream_t st);
// Single-read statistics kernel: T threads per workgroup, NB vectors per thread and row, S slices per position.
// It leaves what the two-kernel path leaves (rows, entropies, per-slice JS sums, the drafted tokens' logits)
// plus the hand-off words of the positions it worked on, which the decision kernel clears (DecideArgs::xchg_split).
bool fused_plan(const RowMap& map, int dt, int* T_out, int* NB_out, int* S_out);
hipError_t launch_stats_fused(const RowMap& map, int dt, int T, int NB, int S, int wait_polls,
                              const Workspace& ws, const VerifyOut& vout, hipStream_t st);

struct UpdateArgs {
  int32_t B, K, cap;
  float* T_G;
  double* ent_sum;
  int32_t* ent_cnt;
  float* LA;
  float* LR;
  int32_t* nA;
  int32_t* nR;
  double* mom;          // [B,4] running sums of the lists about their first elements, or null
  const int32_t* n_accept;
  const int32_t* draft_len;
  const float* H_q;
  const float* d_js;
  float d_eps;
  uint32_t* status;
};
struct DecideArgs {
  RowMap map;
  int32_t dt;
  int32_t jsd_split;   // > 0: the distances are still per-slice partial sums of the JS kernel (that many per position)
  int32_t xchg_split;  // > 0: the single-read statistics kernel ran with that many slices: its hand-off words are cleared here
  const int32_t* draft_tokens;
  // state (device pointers, may be null)
  int32_t cap;
  const float* LA;
  const float* LR;
  const int32_t* nA;
  const int32_t* nR;
  const double* mom;    // [B,4] running sums of the lists about their first elements, or null: add them up here
  uint32_t seed_lo, seed_hi;
  const uint32_t* seq_id;
  const uint32_t* round;
  uint32_t round0;
  int32_t reject_rule, kde_min_n, bw_rule, relaxed_off;
  const float2* tok;    // non-null: (z_p(x), z_q(x)) of every position's drafted token; the logits are then not read
  int32_t base_test;    // 1: match test of the verification loop, replacement from p without the drafted token
  int32_t list_update;  // 1: the accepted list grows inside the loop
  float d_eps;          // filter of the in-loop appends
  // outputs
  int32_t* n_accept;
  float* H_p;
  float* H_q;
  float* d_js;
  float* p_accept;
  uint8_t* accept_mask;
  uint32_t* status;
};
// upd.B > 0: the round is also applied to the state (the update step) by the same kernel
hipError_t launch_decide(const DecideArgs& a, const UpdateArgs& upd, const Workspace& ws, hipStream_t st);
// JS distance: per-slice partial sums (the decision kernel adds them up), rows and entropies
// S_fold: slice records per row that the kernel folds into the normalisers (S for a whole-vocabulary call)
hipError_t launch_jsd(const RowMap& map, int dt, int S, int S_fold, const Workspace& ws, const VerifyOut& vout,
                      hipStream_t st);

// ---- column-sharded verification: records exchanged between the shards (float4 each)
hipError_t launch_shard_fold_rows(const RowMap& map, int S, const Workspace& ws, float4* triples_out, hipStream_t st);
hipError_t launch_shard_scatter_rows(const float4* triples_all, int G, int rows, const Workspace& ws, hipStream_t st);
hipError_t launch_shard_fold_pos(const RowMap& map, int dt, int S, const Workspace& ws, const int32_t* draft_tokens,
                                 int col_begin, float4* pos_out, hipStream_t st);
hipError_t launch_shard_prepare(const RowMap& map, const float4* pos_all, int G, const Workspace& ws, float* H_p,
                                float* H_q, hipStream_t st);

struct SampleArgs {
  RowMap map;
  int32_t dt;
  uint32_t seed_lo, seed_hi;
  const uint32_t* seq_id;
  const uint32_t* round;
  uint32_t round0;
  int32_t* next_token;
  uint32_t* status;
};
hipError_t launch_shard_sample(const SampleArgs& a, int S, int col0, const Workspace& ws, float4* top_out, hipStream_t st);
hipError_t launch_shard_pick(int B, int G, const float4* top_all, const Workspace& ws, int32_t* next_token,
                             uint32_t* status, float* tau_out, hipStream_t st);
hipError_t launch_shard_refine(const SampleArgs& a, int S, int col0, const float* tau, int exact, const Workspace& ws,
                               void* cand_out, hipStream_t st);
hipError_t launch_shard_settle(const SampleArgs& a, int G, float* tau, const void* cand_all, const Workspace& ws,
                               hipStream_t st);
hipError_t launch_sample(const SampleArgs& a, int S, const Workspace& ws, hipStream_t st);

hipError_t launch_update(const UpdateArgs& a, hipStream_t st);
hipError_t launch_state_refresh(const UpdateArgs& a, hipStream_t st);
hipError_t launch_state_init(const UpdateArgs& a, hipStream_t st);
hipError_t launch_state_refresh(const UpdateArgs& a, hipStream_t st);
hipError_t launch_zero(void* p, size_t bytes, hipStream_t st);

}  // namespace adasd
