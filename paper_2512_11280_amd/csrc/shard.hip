// Column-sharded verification: the vocabulary of every row is split over G holders of V/G columns each
// (a tensor-parallel output layer), and the statistics of Appendix A and Section 2.2 are formed from
// per-shard partial results: one (reference, sum, sum x*e) triple per row and shard, then one partial
// Jensen-Shannon sum per position and shard.  The kernels here turn the slice records of a shard's own
// launch into those exchange records, and the gathered records of all shards back into the workspace
// layout the whole-vocabulary kernels read.
#include "stats_device.h"

namespace adasd {

namespace {

__device__ __forceinline__ bool row_is_active(const RowMap& map, int rho) {
  const int pos = rho >> 1, b = pos / map.K, i = pos - b * map.K;
  int kb = map.K;
  if (map.draft_len) kb = min(max(map.draft_len[b], 0), map.K);
  return i < kb;
}

// One wavefront per row: the S slice records of this shard's launch -> one triple (reference, sum, sum x*e).
__global__ void __launch_bounds__(kBlock) k_shard_fold_rows(RowMap map, int S, Workspace ws, float4* out) {
  const int lane = threadIdx.x & 63, rho = blockIdx.x * kWaves + (threadIdx.x >> 6);
  const int rows = map.B * map.K * 2;
  if (rho >= rows) return;
  Lse t = lse_empty();
  if (row_is_active(map, rho) && lane < S) {
    const float4 p = ws.part1[(size_t)rho * kMaxSplit + lane];
    t = Lse{p.x, p.y, p.z};
  }
  const float M = wave_max_f(t.m), d = t.m - M, f = ex2(d);
  const float sw = wave_sum_f(t.s * f), uw = wave_sum_f((t.u + d * t.s) * f);
  if (lane == 0) out[rho] = make_float4(M, sw, uw, 0.f);
}

// The gathered triples of all shards become the "slices" of each row.
__global__ void __launch_bounds__(kBlock) k_shard_scatter_rows(const float4* all, int G, int rows, Workspace ws) {
  const int idx = blockIdx.x * kBlock + threadIdx.x;
  if (idx >= G * rows) return;
  const int g = idx / rows, rho = idx - g * rows;
  ws.part1[(size_t)rho * kMaxSplit + g] = all[idx];
}

// One thread per position: this shard's partial Jensen-Shannon sum (slices added in order) and, if the
// drafted token's column lives here, its two logits.
template <int DT>
__global__ void __launch_bounds__(kBlock) k_shard_fold_pos(RowMap map, int S, Workspace ws, const int32_t* draft_tokens,
                                                           int col_begin, float4* out) {
  const int pos = blockIdx.x * kBlock + threadIdx.x;
  if (pos >= map.B * map.K) return;
  float t = 0.f;
  if (row_is_active(map, 2 * pos))
    for (int s = 0; s < S; ++s) t += ws.part2[(size_t)pos * kMaxSplit + s].x;
  const int b = pos / map.K, i = pos - b * map.K;
  const int x = draft_tokens[pos] - col_begin;
  float zp = 0.f, zq = 0.f, has = 0.f;
  if (x >= 0 && x < map.V) {
    const char* prow = map.base[0] + ((int64_t)b * map.seq_stride[0] + (int64_t)i * map.pos_stride[0]) * Elem<DT>::bytes;
    const char* qrow = map.base[1] + ((int64_t)b * map.seq_stride[1] + (int64_t)i * map.pos_stride[1]) * Elem<DT>::bytes;
    zp = load_elem<DT>(prow, x);
    zq = load_elem<DT>(qrow, x);
    has = 1.f;
  }
  out[pos] = make_float4(t, zp, zq, has);
}

// One wavefront per row, after the scatter: normaliser and entropy of the row from the G triples; the
// wavefront of a position's target row also lays out the G partial sums and the token's logits.
__global__ void __launch_bounds__(kBlock) k_shard_prepare(RowMap map, const float4* pos_all, int G, Workspace ws,
                                                          float* H_p, float* H_q) {
  const int lane = threadIdx.x & 63, rho = blockIdx.x * kWaves + (threadIdx.x >> 6);
  const int P = map.B * map.K;
  if (rho >= 2 * P) return;
  const RowResult res = fold_row(ws, rho, G);
  const int pos = rho >> 1;
  if (lane == 0) {
    ws.rows[rho] = res;
    float* H = (rho & 1) ? H_q : H_p;
    if (H) H[pos] = res.H;
  }
  if (rho & 1) return;
  float4 rec = make_float4(0.f, 0.f, 0.f, 0.f);
  if (lane < G) {
    rec = pos_all[(size_t)lane * P + pos];
    reinterpret_cast<float*>(&ws.part2[(size_t)pos * kMaxSplit + lane])[0] = rec.x;
  }
  const unsigned long long owners = __ballot(lane < G && rec.w != 0.f);
  const int owner = owners ? __ffsll((long long)owners) - 1 : 0;
  const float zp = __shfl(rec.y, owner), zq = __shfl(rec.z, owner);
  if (lane == 0) ws.tok[pos] = owners ? make_float2(zp, zq) : make_float2(0.f, 0.f);
}

}  // namespace

hipError_t launch_shard_fold_rows(const RowMap& map, int S, const Workspace& ws, float4* triples_out, hipStream_t st) {
  const int rows = map.B * map.K * 2;
  if (rows <= 0) return hipSuccess;
  launch_kernel(k_shard_fold_rows, dim3((rows + kWaves - 1) / kWaves), dim3(kBlock), st, map, S, ws, triples_out);
  return hipGetLastError();
}

hipError_t launch_shard_scatter_rows(const float4* triples_all, int G, int rows, const Workspace& ws, hipStream_t st) {
  if (rows <= 0) return hipSuccess;
  launch_kernel(k_shard_scatter_rows, dim3((G * rows + kBlock - 1) / kBlock), dim3(kBlock), st, triples_all, G, rows, ws);
  return hipGetLastError();
}

hipError_t launch_shard_fold_pos(const RowMap& map, int dt, int S, const Workspace& ws, const int32_t* draft_tokens,
                                 int col_begin, float4* pos_out, hipStream_t st) {
  const int P = map.B * map.K;
  if (P <= 0) return hipSuccess;
  const dim3 grid((P + kBlock - 1) / kBlock), block(kBlock);
  if (dt == ADASD_BF16) launch_kernel(k_shard_fold_pos<ADASD_BF16>, grid, block, st, map, S, ws, draft_tokens, col_begin, pos_out);
  else launch_kernel(k_shard_fold_pos<ADASD_F32>, grid, block, st, map, S, ws, draft_tokens, col_begin, pos_out);
  return hipGetLastError();
}

hipError_t launch_shard_prepare(const RowMap& map, const float4* pos_all, int G, const Workspace& ws, float* H_p,
                                float* H_q, hipStream_t st) {
  const int rows = map.B * map.K * 2;
  if (rows <= 0) return hipSuccess;
  launch_kernel(k_shard_prepare, dim3((rows + kWaves - 1) / kWaves), dim3(kBlock), st, map, pos_all, G, ws, H_p, H_q);
  return hipGetLastError();
}

}  // namespace adasd
