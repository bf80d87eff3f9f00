// C ABI of libadasd: argument validation, workspace carving and kernel enqueue.
#include <mutex>
#include <vector>

#include "internal.h"

namespace adasd {

namespace {

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

bool aligned_to(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// ---- optional kernel timing ----------------------------------------------------------------
constexpr int kClasses = 7;
struct Profiler {
  std::mutex mu;
  bool on = false;
  int cap = 0;
  std::vector<hipEvent_t> start[kClasses], stop[kClasses];
  int used[kClasses] = {0, 0, 0, 0, 0, 0, 0};
} g_prof;

thread_local int t_class = -1;   // kernel class of the timing scope that is open on this thread

struct Scope {   // the kernels launched while it lives are timed under class c
  int prev;
  Scope(int c, hipStream_t) : prev(t_class) { t_class = c; }
  ~Scope() { t_class = prev; }
};

}  // namespace

bool profile_take_events(hipEvent_t* start, hipEvent_t* stop) {
  if (!g_prof.on || t_class < 0) return false;
  std::lock_guard<std::mutex> lk(g_prof.mu);
  if (g_prof.used[t_class] >= g_prof.cap) return false;
  const int slot = g_prof.used[t_class]++;
  *start = g_prof.start[t_class][slot];
  *stop = g_prof.stop[t_class][slot];
  return true;
}

namespace {
constexpr size_t kHeaderBytes = (65536 + 32768 + 32768) * sizeof(int32_t);
// bytes per position of every shape-dependent region (per-sequence regions are sized per position too)
constexpr size_t kRegionBytes[] = {
    (size_t)kMaxSplit * kXchgWords * sizeof(uint64_t),    // xchg
    2 * (size_t)kMaxSplit * sizeof(float4),               // part1
    2 * sizeof(RowResult),                                // rows
    (size_t)kMaxSplit * sizeof(float2),                   // part2
    sizeof(SamplePlan),                                   // plan
    (size_t)kMaxSampleSplit * sizeof(Top2),               // part3
    sizeof(PosRecord),                                    // pos_rec
    sizeof(float2),                                       // tok
    sizeof(int32_t),                                      // slots
};
constexpr size_t per_position_bytes() {
  size_t t = 0;
  for (size_t r : kRegionBytes) t += r;
  return t;
}
}  // namespace

size_t workspace_bytes_for(size_t positions) {
  return kHeaderBytes + (positions + 1) * per_position_bytes() + 9 * 256;
}

size_t workspace_layout(size_t ws_bytes, Workspace* ws, void* base) {
  const size_t slack = kHeaderBytes + 9 * 256;
  if (ws_bytes <= slack) return 0;
  const size_t cap = (ws_bytes - slack) / per_position_bytes();
  if (ws && cap > 0) {
    char* p = static_cast<char*>(base);
    size_t off = 0;
    auto take = [&](size_t bytes) {
      size_t at = off;
      off = align_up(off + bytes, 256);
      return p + at;
    };
    // arrival counters: fixed size, sized for the compiled limits
    ws->ticket1 = reinterpret_cast<int32_t*>(take(kTicket1Len * sizeof(int32_t)));
    ws->ticket2 = reinterpret_cast<int32_t*>(take(kTicket2Len * sizeof(int32_t)));
    ws->ticket3 = reinterpret_cast<int32_t*>(take(kTicket3Len * sizeof(int32_t)));
    ws->xchg = reinterpret_cast<uint64_t*>(take(cap * kRegionBytes[0]));
    ws->part1 = reinterpret_cast<float4*>(take(cap * kRegionBytes[1]));
    ws->rows = reinterpret_cast<RowResult*>(take(cap * kRegionBytes[2]));
    ws->part2 = reinterpret_cast<float2*>(take(cap * kRegionBytes[3]));
    ws->plan = reinterpret_cast<SamplePlan*>(take(cap * kRegionBytes[4]));
    ws->part3 = reinterpret_cast<Top2*>(take(cap * kRegionBytes[5]));
    ws->pos_rec = reinterpret_cast<PosRecord*>(take(cap * kRegionBytes[6]));
    ws->tok = reinterpret_cast<float2*>(take(cap * kRegionBytes[7]));
    ws->slots = reinterpret_cast<int32_t*>(take(cap * kRegionBytes[8]));
    ws->bytes = off;
  }
  return cap;
}

}  // namespace adasd

using namespace adasd;

extern "C" {

int adasd_version(void) { return 100; }

const char* adasd_strerror(int code) {
  switch (code) {
    case ADASD_OK: return "ok";
    case ADASD_ERR_INVALID_ARG: return "invalid argument";
    case ADASD_ERR_MISALIGNED: return "pointer below the natural alignment of its element type";
    case ADASD_ERR_UNSUPPORTED: return "option value not supported by this build";
    case ADASD_ERR_WORKSPACE: return "workspace missing or too small";
    case ADASD_ERR_CAPACITY: return "size beyond a compiled limit";
    case ADASD_ERR_HIP: return "HIP runtime error";
    default: return "unknown error code";
  }
}

static int check_shape(int B, int k_max, int V, int dt) {
  if (B < 0 || k_max < 0 || V < 1) return ADASD_ERR_INVALID_ARG;
  if (dt != ADASD_F32 && dt != ADASD_BF16) return ADASD_ERR_INVALID_ARG;
  if (k_max > ADASD_MAX_K || V > ADASD_MAX_V) return ADASD_ERR_CAPACITY;
  if ((int64_t)B * (k_max > 0 ? k_max : 1) * 2 > 65535) return ADASD_ERR_CAPACITY;
  return ADASD_OK;
}

int adasd_workspace_bytes(int B, int k_max, int V, adasd_dtype dt, size_t* bytes) {
  if (!bytes) return ADASD_ERR_INVALID_ARG;
  int rc = check_shape(B, k_max, V, (int)dt);
  if (rc) return rc;
  // large enough for a verify call of this shape and for draft-entropy calls with up to B*max(k,1) rows
  *bytes = workspace_bytes_for((size_t)B * (size_t)(k_max > 0 ? k_max : 1));
  return ADASD_OK;
}

int adasd_workspace_init(void* workspace, size_t ws_bytes, void* stream) {
  if (!workspace || ws_bytes == 0) return ADASD_ERR_WORKSPACE;
  if (!aligned_to(workspace, 256)) return ADASD_ERR_MISALIGNED;
  return launch_zero(workspace, ws_bytes, (hipStream_t)stream) == hipSuccess ? ADASD_OK : ADASD_ERR_HIP;
}

static int check_state(const adasd_state* st) {
  if (!st) return ADASD_ERR_INVALID_ARG;
  if (st->B < 0 || st->cap < 0) return ADASD_ERR_INVALID_ARG;
  if (st->B == 0) return ADASD_OK;
  if (!st->T_G || !st->ent_sum || !st->ent_cnt || !st->nA || !st->nR) return ADASD_ERR_INVALID_ARG;
  if (st->cap > 0 && (!st->LA || !st->LR)) return ADASD_ERR_INVALID_ARG;
  if (!aligned_to(st->T_G, 4) || !aligned_to(st->ent_sum, 8) || !aligned_to(st->ent_cnt, 4) ||
      !aligned_to(st->LA, 4) || !aligned_to(st->LR, 4) || !aligned_to(st->nA, 4) ||
      !aligned_to(st->nR, 4) || !aligned_to(st->mom, 8))
    return ADASD_ERR_MISALIGNED;
  return ADASD_OK;
}

static UpdateArgs state_args(const adasd_state* st) {
  UpdateArgs u{};
  u.B = st->B;
  u.cap = st->cap;
  u.T_G = st->T_G;
  u.ent_sum = st->ent_sum;
  u.ent_cnt = st->ent_cnt;
  u.LA = st->LA;
  u.LR = st->LR;
  u.nA = st->nA;
  u.nR = st->nR;
  u.mom = st->mom;
  return u;
}

int adasd_state_init(const adasd_state* st, void* stream) {
  int rc = check_state(st);
  if (rc) return rc;
  UpdateArgs u = state_args(st);
  return launch_state_init(u, (hipStream_t)stream) == hipSuccess ? ADASD_OK : ADASD_ERR_HIP;
}

int adasd_state_refresh(const adasd_state* st, void* stream) {
  int rc = check_state(st);
  if (rc) return rc;
  if (!st->mom || st->B == 0) return ADASD_OK;
  UpdateArgs u = state_args(st);
  return launch_state_refresh(u, (hipStream_t)stream) == hipSuccess ? ADASD_OK : ADASD_ERR_HIP;
}

int adasd_draft_entropy(const void* draft_logits, adasd_dtype dt, int B, int V, int64_t row_stride,
                        const float* T_G, const uint8_t* active, int step, int k_max, float* H_out,
                        uint8_t* stop_out, void* workspace, size_t ws_bytes, void* stream) {
  int rc = check_shape(B, 0, V, (int)dt);
  if (rc) return rc;
  if (B == 0) return ADASD_OK;
  if (!draft_logits || !H_out || row_stride < V || step < 0 || k_max < 1) return ADASD_ERR_INVALID_ARG;
  const size_t es = dt == ADASD_BF16 ? 2 : 4;
  if (!aligned_to(draft_logits, es) || !aligned_to(H_out, 4) || !aligned_to(T_G, 4))
    return ADASD_ERR_MISALIGNED;
  if (!workspace) return ADASD_ERR_WORKSPACE;
  if (!aligned_to(workspace, 256)) return ADASD_ERR_MISALIGNED;
  Workspace ws;
  if (workspace_layout(ws_bytes, &ws, workspace) < (size_t)B) return ADASD_ERR_WORKSPACE;

  RowMap map{};
  map.base[0] = static_cast<const char*>(draft_logits);
  map.base[1] = nullptr;
  map.seq_stride[0] = row_stride;
  map.active = active;
  map.K = 0;
  map.B = B;
  map.V = V;
  DraftOut dout{T_G, H_out, stop_out, step + 1 >= k_max ? 1 : 0};
  hipStream_t st = (hipStream_t)stream;
  const int S = pick_draft_split(B, V, (int)dt);
  Scope sc(5, st);
  return launch_draft_step(map, (int)dt, S, ws, dout, nullptr, st) == hipSuccess ? ADASD_OK : ADASD_ERR_HIP;
}

int adasd_draft_step(const void* draft_logits, adasd_dtype dt, int B, int V, int64_t row_stride,
                     const float* T_G, const uint8_t* active, int step, int k_max, uint64_t seed,
                     const uint32_t* seq_id, const uint32_t* round, uint32_t round0, float* H_out,
                     uint8_t* stop_out, int32_t* token_out, uint32_t* status_out, void* workspace,
                     size_t ws_bytes, void* stream) {
  int rc = check_shape(B, 0, V, (int)dt);
  if (rc) return rc;
  if (B == 0) return ADASD_OK;
  if (!draft_logits || !H_out || !token_out || row_stride < V || step < 0 || step >= 65536 || k_max < 1)
    return ADASD_ERR_INVALID_ARG;
  const size_t es = dt == ADASD_BF16 ? 2 : 4;
  if (!aligned_to(draft_logits, es) || !aligned_to(H_out, 4) || !aligned_to(T_G, 4) ||
      !aligned_to(token_out, 4) || !aligned_to(status_out, 4) || !aligned_to(seq_id, 4) ||
      !aligned_to(round, 4))
    return ADASD_ERR_MISALIGNED;
  if (!workspace) return ADASD_ERR_WORKSPACE;
  if (!aligned_to(workspace, 256)) return ADASD_ERR_MISALIGNED;
  Workspace ws;
  if (workspace_layout(ws_bytes, &ws, workspace) < (size_t)B) return ADASD_ERR_WORKSPACE;

  RowMap map{};
  map.base[0] = static_cast<const char*>(draft_logits);
  map.base[1] = nullptr;
  map.seq_stride[0] = row_stride;
  map.active = active;
  map.K = 0;
  map.B = B;
  map.V = V;
  DraftOut dout{T_G, H_out, stop_out, step + 1 >= k_max ? 1 : 0};
  DraftDraw draw{(uint32_t)seed, (uint32_t)(seed >> 32), seq_id, round, round0, (uint32_t)step, token_out, status_out};
  hipStream_t st = (hipStream_t)stream;
  const int S = pick_draft_split(B, V, (int)dt);
  Scope sc(5, st);
  return launch_draft_step(map, (int)dt, S, ws, dout, &draw, st) == hipSuccess ? ADASD_OK : ADASD_ERR_HIP;
}

namespace {

// Everything adasd_verify and the column-sharded entry points derive from their arguments.
struct VerifySetup {
  adasd_options opt;
  Workspace ws;
  RowMap map;
  DecideArgs d;
  UpdateArgs upd;
};
enum { kWantLogits = 1, kWantOutputs = 2, kWantToken = 4 };

// Returns ADASD_OK with `out` filled, a negative error code, or 1 for an empty batch (nothing to do).
int verify_setup(const adasd_verify_args* a, const adasd_options* opt_in, int wants, VerifySetup* out) {
  if (!a) return ADASD_ERR_INVALID_ARG;
  adasd_options opt{};
  if (opt_in) opt = *opt_in;
  int rc = check_shape(a->B, a->k_max, a->V, (int)a->dt);
  if (rc) return rc;
  if (opt.base_test != 0 && opt.base_test != 1) return ADASD_ERR_INVALID_ARG;
  if (opt.list_update != 0 && opt.list_update != 1) return ADASD_ERR_INVALID_ARG;
  if (opt.reject_rule != 0 && opt.reject_rule != 1) return ADASD_ERR_INVALID_ARG;
  if (opt.bw_rule != 0 && opt.bw_rule != 1) return ADASD_ERR_INVALID_ARG;
  if (opt.stats_path < 0 || opt.stats_path > 2) return ADASD_ERR_INVALID_ARG;
  if (opt.apply_update != 0 && opt.apply_update != 1) return ADASD_ERR_INVALID_ARG;
  if (opt.apply_update && !a->state) return ADASD_ERR_INVALID_ARG;
  if (a->B == 0) return 1;
  const int B = a->B, K = a->k_max, V = a->V;
  if ((wants & kWantLogits) && !a->target_logits) return ADASD_ERR_INVALID_ARG;
  if ((wants & kWantOutputs) && (!a->n_accept || !a->status)) return ADASD_ERR_INVALID_ARG;
  if ((wants & kWantToken) && (!a->next_token || !a->status)) return ADASD_ERR_INVALID_ARG;
  if (K > 0 && (wants & kWantLogits) && !a->draft_logits) return ADASD_ERR_INVALID_ARG;
  if (K > 0 && !a->draft_tokens) return ADASD_ERR_INVALID_ARG;
  if (K > 0 && (wants & kWantOutputs) && (!a->H_q || !a->d_js)) return ADASD_ERR_INVALID_ARG;
  if (wants & kWantLogits) {
    if (a->t_pos_stride < V || a->t_seq_stride < (int64_t)(K + 1) * V) return ADASD_ERR_INVALID_ARG;
    if (K > 0 && (a->d_pos_stride < V || a->d_seq_stride < (int64_t)K * V)) return ADASD_ERR_INVALID_ARG;
  }
  const size_t es = a->dt == ADASD_BF16 ? 2 : 4;
  if (!aligned_to(a->target_logits, es) || !aligned_to(a->draft_logits, es) ||
      !aligned_to(a->draft_tokens, 4) || !aligned_to(a->draft_len, 4) || !aligned_to(a->seq_id, 4) ||
      !aligned_to(a->round, 4) || !aligned_to(a->n_accept, 4) || !aligned_to(a->next_token, 4) ||
      !aligned_to(a->H_p, 4) || !aligned_to(a->H_q, 4) || !aligned_to(a->d_js, 4) ||
      !aligned_to(a->p_accept, 4) || !aligned_to(a->status, 4))
    return ADASD_ERR_MISALIGNED;
  if (a->state) {
    rc = check_state(a->state);
    if (rc) return rc;
    if (a->state->B < B) return ADASD_ERR_INVALID_ARG;
  }
  if (!a->workspace) return ADASD_ERR_WORKSPACE;
  if (!aligned_to(a->workspace, 256)) return ADASD_ERR_MISALIGNED;
  Workspace ws;
  if (workspace_layout(a->ws_bytes, &ws, a->workspace) < (size_t)B * (size_t)(K > 0 ? K : 1))
    return ADASD_ERR_WORKSPACE;

  RowMap map{};
  map.base[0] = static_cast<const char*>(a->target_logits);
  map.base[1] = static_cast<const char*>(a->draft_logits);
  map.seq_stride[0] = a->t_seq_stride;
  map.pos_stride[0] = a->t_pos_stride;
  map.seq_stride[1] = a->d_seq_stride;
  map.pos_stride[1] = a->d_pos_stride;
  map.draft_len = a->draft_len;
  map.active = nullptr;
  map.K = K;
  map.B = B;
  map.V = V;

  DecideArgs d{};
  d.map = map;
  d.dt = (int)a->dt;
  d.draft_tokens = a->draft_tokens;
  if (a->state) {
    d.cap = a->state->cap;
    d.LA = a->state->LA;
    d.LR = a->state->LR;
    d.nA = a->state->nA;
    d.nR = a->state->nR;
    d.mom = a->state->mom;
  }
  d.seed_lo = (uint32_t)a->seed;
  d.seed_hi = (uint32_t)(a->seed >> 32);
  d.seq_id = a->seq_id;
  d.round = a->round;
  d.round0 = a->round0;
  d.reject_rule = opt.reject_rule;
  d.kde_min_n = opt.kde_min_n;
  d.bw_rule = opt.bw_rule;
  d.relaxed_off = opt.relaxed_off;
  d.base_test = opt.base_test;
  d.list_update = opt.list_update;
  d.d_eps = opt.d_eps > 0.f ? opt.d_eps : 1e-6f;
  d.n_accept = a->n_accept;
  d.H_p = a->H_p;
  d.H_q = a->H_q;
  d.d_js = a->d_js;
  d.p_accept = a->p_accept;
  d.accept_mask = a->accept_mask;
  d.status = a->status;

  UpdateArgs upd{};            // B = 0: the state is only read
  if (opt.apply_update) {
    upd = state_args(a->state);
    upd.K = K;
    upd.n_accept = a->n_accept;
    upd.draft_len = a->draft_len;
    upd.H_q = a->H_q;
    upd.d_js = a->d_js;
    upd.d_eps = d.d_eps;
    upd.status = a->status;
  }
  out->opt = opt;
  out->ws = ws;
  out->map = map;
  out->d = d;
  out->upd = upd;
  return ADASD_OK;
}

SampleArgs sample_args(const adasd_verify_args* a, const VerifySetup& v) {
  SampleArgs s{};
  s.map = v.map;
  s.dt = (int)a->dt;
  s.seed_lo = v.d.seed_lo;
  s.seed_hi = v.d.seed_hi;
  s.seq_id = a->seq_id;
  s.round = a->round;
  s.round0 = a->round0;
  s.next_token = a->next_token;
  s.status = a->status;
  return s;
}

// about two 16-byte vectors per thread: enough workgroups to cover the chip for a handful of rows
int sample_split(int V, int dt) {
  const int nvec = V / (dt == ADASD_BF16 ? 8 : 4);
  int S3 = (nvec + 2 * kBlock - 1) / (2 * kBlock);
  if (S3 < 1) S3 = 1;
  if (S3 > kMaxSampleSplit) S3 = kMaxSampleSplit;
  return S3;
}

}  // namespace

int adasd_verify(const adasd_verify_args* a, const adasd_options* opt_in, void* stream) {
  VerifySetup v;
  int rc = verify_setup(a, opt_in, kWantLogits | kWantOutputs | kWantToken, &v);
  if (rc) return rc < 0 ? rc : ADASD_OK;
  const adasd_options& opt = v.opt;
  const Workspace& ws = v.ws;
  const RowMap& map = v.map;
  DecideArgs& d = v.d;
  const UpdateArgs& upd = v.upd;
  const int B = a->B, K = a->k_max, V = a->V;
  hipStream_t st = (hipStream_t)stream;
  VerifyOut vout{a->H_p, a->H_q, a->d_js, nullptr, nullptr};
  int fT = 0, fNB = 0, fS = 0;
  if (K > 0 && opt.stats_path != 1 && fused_plan(map, (int)a->dt, &fT, &fNB, &fS)) {
    Scope sc(0, st);
    RowMap smap = map;
    if (a->draft_len) {          // ragged windows: the positions that have work, packed
      if (launch_pack_slots(a->draft_len, B, K, ws.slots, st) != hipSuccess) return ADASD_ERR_HIP;
      smap.slots = ws.slots;
    }
    vout.tokens = a->draft_tokens;
    vout.tok = a->draft_tokens ? ws.tok : nullptr;
    const int polls = opt.wait_polls == 0 ? kWaitPolls : (opt.wait_polls < 0 ? 0 : opt.wait_polls);
    if (launch_stats_fused(smap, (int)a->dt, fT, fNB, fS, polls, ws, vout, st) != hipSuccess) return ADASD_ERR_HIP;
    d.jsd_split = fS;
    d.xchg_split = fS;
    d.tok = vout.tok;
  } else if (K > 0) {
    const int rows = B * K * 2;
    const int S = pick_split(rows, V, (int)a->dt);
    RowMap smap = map;
    {
      Scope sc(0, st);
      if (a->draft_len) {        // ragged windows: the positions that have work, packed
        if (launch_pack_slots(a->draft_len, B, K, ws.slots, st) != hipSuccess) return ADASD_ERR_HIP;
        smap.slots = ws.slots;
      }
      if (launch_rowstats(smap, (int)a->dt, rows, S, ws, st) != hipSuccess) return ADASD_ERR_HIP;
    }
    {
      Scope sc(1, st);
      vout.tokens = a->draft_tokens;
      vout.tok = a->draft_tokens ? ws.tok : nullptr;
      if (launch_jsd(smap, (int)a->dt, S, S, ws, vout, st) != hipSuccess) return ADASD_ERR_HIP;
    }
    d.jsd_split = S;
    d.tok = vout.tok;
  }
  {
    Scope sc(2, st);
    if (launch_decide(d, upd, ws, st) != hipSuccess) return ADASD_ERR_HIP;
  }

  const SampleArgs s = sample_args(a, v);
  const int S3 = sample_split(V, (int)a->dt);
  {
    Scope sc(3, st);
    if (launch_sample(s, S3, ws, st) != hipSuccess) return ADASD_ERR_HIP;
  }
  return ADASD_OK;
}

// ---- verification without a caller-provided workspace -------------------------------------------
// For callers that cannot allocate device memory (code under HIP graph capture, serving loops and harnesses
// that forbid hipMalloc): the workspace is an array in the library's own device image.  Every GPU the
// library runs on holds its own copy of the array at its own address until the process ends; the array's
// name is only a host-side handle, so its device address is looked up once per device, with that device
// current, and only that address is ever handed to a kernel.
constexpr size_t kScratchBytes = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
struct StaticScratch {
  std::mutex mu;
  void* ptr[kMaxDevices] = {};
  bool clean[kMaxDevices] = {};      // false: the counters and hand-off words have to be zeroed before the next call
} g_scratch;

// The device address of `scratch` on the current device (looked up on the first call there), zeroed on the
// caller's stream if it has never been used or if the last call on it failed half-way.
int static_scratch(void** out, hipStream_t st) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return ADASD_ERR_HIP;
  std::lock_guard<std::mutex> lk(g_scratch.mu);
  if (!g_scratch.ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return ADASD_ERR_HIP;
    g_scratch.ptr[dev] = p;
    g_scratch.clean[dev] = false;
  }
  if (!g_scratch.clean[dev]) {
    if (launch_zero(g_scratch.ptr[dev], kScratchBytes, st) != hipSuccess) return ADASD_ERR_HIP;
    g_scratch.clean[dev] = true;
  }
  *out = g_scratch.ptr[dev];
  return ADASD_OK;
}
void static_scratch_failed() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return;
  std::lock_guard<std::mutex> lk(g_scratch.mu);
  g_scratch.clean[dev] = false;
}
}  // namespace

int adasd_verify_noalloc(const adasd_verify_args* a, const adasd_options* opt, void* stream) {
  if (!a) return ADASD_ERR_INVALID_ARG;
  size_t need = 0;
  int rc = adasd_workspace_bytes(a->B, a->k_max, a->V, a->dt, &need);
  if (rc) return rc;
  if (need > kScratchBytes) return ADASD_ERR_CAPACITY;      // more positions than the built-in workspace serves
  void* ptr = nullptr;
  rc = static_scratch(&ptr, (hipStream_t)stream);
  if (rc) return rc;
  adasd_verify_args b = *a;
  b.workspace = ptr;
  b.ws_bytes = kScratchBytes;
  rc = adasd_verify(&b, opt, stream);
  if (rc == ADASD_ERR_HIP) static_scratch_failed();         // a launch failed half-way: counters may be left set
  return rc;
}

// ---- column-sharded verification ---------------------------------------------------------------
static int check_shard(const adasd_shard* sh, int V_local, bool local) {
  if (!sh) return ADASD_ERR_INVALID_ARG;
  if (sh->n_shards < 1 || sh->n_shards > ADASD_MAX_SHARDS) return ADASD_ERR_CAPACITY;
  if (sh->V_total < 1 || sh->V_total > ADASD_MAX_V) return ADASD_ERR_CAPACITY;
  if (!local) return V_local == sh->V_total ? ADASD_OK : ADASD_ERR_INVALID_ARG;
  if (sh->shard < 0 || sh->shard >= sh->n_shards) return ADASD_ERR_INVALID_ARG;
  if (sh->col_begin < 0 || (sh->col_begin & 7) || (int64_t)sh->col_begin + V_local > sh->V_total)
    return ADASD_ERR_INVALID_ARG;
  return ADASD_OK;
}

int adasd_verify_shard_stats(const adasd_verify_args* local, const adasd_shard* sh, float* triples_out, void* stream) {
  VerifySetup v;
  int rc = verify_setup(local, nullptr, kWantLogits, &v);
  if (rc) return rc < 0 ? rc : ADASD_OK;
  rc = check_shard(sh, local->V, true);
  if (rc) return rc;
  const int rows = local->B * local->k_max * 2;
  if (rows == 0) return ADASD_OK;
  if (!triples_out) return ADASD_ERR_INVALID_ARG;
  if (!aligned_to(triples_out, 16)) return ADASD_ERR_MISALIGNED;
  hipStream_t st = (hipStream_t)stream;
  const int S = pick_split(rows, local->V, (int)local->dt);
  Scope sc(0, st);
  if (launch_rowstats(v.map, (int)local->dt, rows, S, v.ws, st) != hipSuccess) return ADASD_ERR_HIP;
  if (launch_shard_fold_rows(v.map, S, v.ws, reinterpret_cast<float4*>(triples_out), st) != hipSuccess) return ADASD_ERR_HIP;
  return ADASD_OK;
}

int adasd_verify_shard_jsd(const adasd_verify_args* local, const adasd_shard* sh, const float* triples_all,
                           float* pos_out, void* stream) {
  VerifySetup v;
  int rc = verify_setup(local, nullptr, kWantLogits, &v);
  if (rc) return rc < 0 ? rc : ADASD_OK;
  rc = check_shard(sh, local->V, true);
  if (rc) return rc;
  const int rows = local->B * local->k_max * 2;
  if (rows == 0) return ADASD_OK;
  if (!triples_all || !pos_out) return ADASD_ERR_INVALID_ARG;
  if (!aligned_to(triples_all, 16) || !aligned_to(pos_out, 16)) return ADASD_ERR_MISALIGNED;
  hipStream_t st = (hipStream_t)stream;
  const int S = pick_split(rows, local->V, (int)local->dt);
  Scope sc(1, st);
  if (launch_shard_scatter_rows(reinterpret_cast<const float4*>(triples_all), sh->n_shards, rows, v.ws, st) != hipSuccess)
    return ADASD_ERR_HIP;
  const VerifyOut none{nullptr, nullptr, nullptr};
  if (launch_jsd(v.map, (int)local->dt, S, sh->n_shards, v.ws, none, st) != hipSuccess) return ADASD_ERR_HIP;
  if (launch_shard_fold_pos(v.map, (int)local->dt, S, v.ws, local->draft_tokens, sh->col_begin,
                            reinterpret_cast<float4*>(pos_out), st) != hipSuccess)
    return ADASD_ERR_HIP;
  return ADASD_OK;
}

int adasd_verify_shard_decide(const adasd_verify_args* meta, const adasd_shard* sh, const float* triples_all,
                              const float* pos_all, const adasd_options* opt, void* stream) {
  VerifySetup v;
  int rc = verify_setup(meta, opt, kWantOutputs, &v);
  if (rc) return rc < 0 ? rc : ADASD_OK;
  rc = check_shard(sh, meta->V, false);
  if (rc) return rc;
  const int rows = meta->B * meta->k_max * 2;
  if (rows > 0 && (!triples_all || !pos_all)) return ADASD_ERR_INVALID_ARG;
  if (!aligned_to(triples_all, 16) || !aligned_to(pos_all, 16)) return ADASD_ERR_MISALIGNED;
  hipStream_t st = (hipStream_t)stream;
  Scope sc(2, st);
  if (rows > 0) {
    if (launch_shard_scatter_rows(reinterpret_cast<const float4*>(triples_all), sh->n_shards, rows, v.ws, st) != hipSuccess)
      return ADASD_ERR_HIP;
    if (launch_shard_prepare(v.map, reinterpret_cast<const float4*>(pos_all), sh->n_shards, v.ws, meta->H_p, meta->H_q,
                             st) != hipSuccess)
      return ADASD_ERR_HIP;
    v.d.jsd_split = sh->n_shards;
    v.d.tok = v.ws.tok;
  }
  v.d.map.base[0] = v.d.map.base[1] = nullptr;      // no logits in this call
  if (launch_decide(v.d, v.upd, v.ws, st) != hipSuccess) return ADASD_ERR_HIP;
  return ADASD_OK;
}

int adasd_verify_shard_sample(const adasd_verify_args* local, const adasd_shard* sh, float* top_out, void* stream) {
  VerifySetup v;
  int rc = verify_setup(local, nullptr, kWantLogits, &v);
  if (rc) return rc < 0 ? rc : ADASD_OK;
  rc = check_shard(sh, local->V, true);
  if (rc) return rc;
  if (!top_out) return ADASD_ERR_INVALID_ARG;
  if (!aligned_to(top_out, 16)) return ADASD_ERR_MISALIGNED;
  hipStream_t st = (hipStream_t)stream;
  Scope sc(3, st);
  const SampleArgs s = sample_args(local, v);
  return launch_shard_sample(s, sample_split(local->V, (int)local->dt), sh->col_begin, v.ws,
                             reinterpret_cast<float4*>(top_out), st) == hipSuccess ? ADASD_OK : ADASD_ERR_HIP;
}

int adasd_verify_shard_pick(const adasd_verify_args* meta, const adasd_shard* sh, const float* top_all, float* tau_out,
                            void* stream) {
  VerifySetup v;
  int rc = verify_setup(meta, nullptr, kWantToken, &v);
  if (rc) return rc < 0 ? rc : ADASD_OK;
  rc = check_shard(sh, meta->V, false);
  if (rc) return rc;
  if (!top_all || !tau_out) return ADASD_ERR_INVALID_ARG;
  if (!aligned_to(top_all, 16) || !aligned_to(tau_out, 4)) return ADASD_ERR_MISALIGNED;
  hipStream_t st = (hipStream_t)stream;
  Scope sc(3, st);
  return launch_shard_pick(meta->B, sh->n_shards, reinterpret_cast<const float4*>(top_all), v.ws, meta->next_token,
                           meta->status, tau_out, st) == hipSuccess ? ADASD_OK : ADASD_ERR_HIP;
}

int adasd_verify_shard_refine(const adasd_verify_args* local, const adasd_shard* sh, const float* tau, int exact_sums,
                              void* cand_out, void* stream) {
  VerifySetup v;
  int rc = verify_setup(local, nullptr, kWantLogits, &v);
  if (rc) return rc < 0 ? rc : ADASD_OK;
  rc = check_shard(sh, local->V, true);
  if (rc) return rc;
  if (!tau || !cand_out || (exact_sums != 0 && exact_sums != 1)) return ADASD_ERR_INVALID_ARG;
  if (!aligned_to(tau, 4) || !aligned_to(cand_out, 16)) return ADASD_ERR_MISALIGNED;
  hipStream_t st = (hipStream_t)stream;
  Scope sc(3, st);
  const SampleArgs s = sample_args(local, v);
  return launch_shard_refine(s, sample_split(local->V, (int)local->dt), sh->col_begin, tau, exact_sums, v.ws, cand_out, st) == hipSuccess
             ? ADASD_OK : ADASD_ERR_HIP;
}

int adasd_verify_shard_settle(const adasd_verify_args* meta, const adasd_shard* sh, float* tau, const void* cand_all,
                              void* stream) {
  VerifySetup v;
  int rc = verify_setup(meta, nullptr, kWantToken, &v);
  if (rc) return rc < 0 ? rc : ADASD_OK;
  rc = check_shard(sh, meta->V, false);
  if (rc) return rc;
  if (!tau || !cand_all) return ADASD_ERR_INVALID_ARG;
  if (!aligned_to(tau, 4) || !aligned_to(cand_all, 16)) return ADASD_ERR_MISALIGNED;
  hipStream_t st = (hipStream_t)stream;
  Scope sc(3, st);
  const SampleArgs s = sample_args(meta, v);
  return launch_shard_settle(s, sh->n_shards, tau, cand_all, v.ws, st) == hipSuccess ? ADASD_OK : ADASD_ERR_HIP;
}

int adasd_update_thresholds(const adasd_state* st, int k_max, const int32_t* n_accept,
                            const int32_t* draft_len, const float* H_q, const float* d_js,
                            const adasd_options* opt, uint32_t* status, void* stream) {
  int rc = check_state(st);
  if (rc) return rc;
  if (k_max < 0) return ADASD_ERR_INVALID_ARG;
  if (k_max > ADASD_MAX_K) return ADASD_ERR_CAPACITY;
  if (st->B == 0) return ADASD_OK;
  if (!n_accept || (k_max > 0 && (!H_q || !d_js))) return ADASD_ERR_INVALID_ARG;
  if (!aligned_to(n_accept, 4) || !aligned_to(draft_len, 4) || !aligned_to(H_q, 4) ||
      !aligned_to(d_js, 4) || !aligned_to(status, 4))
    return ADASD_ERR_MISALIGNED;
  UpdateArgs u = state_args(st);
  u.K = k_max;
  u.n_accept = n_accept;
  u.draft_len = draft_len;
  u.H_q = H_q;
  u.d_js = d_js;
  u.d_eps = (opt && opt->d_eps > 0.f) ? opt->d_eps : 1e-6f;
  u.status = status;
  hipStream_t s = (hipStream_t)stream;
  Scope sc(4, s);
  return launch_update(u, s) == hipSuccess ? ADASD_OK : ADASD_ERR_HIP;
}

int adasd_stream_read(const void* src, size_t bytes, uint32_t* sink, size_t sink_words, void* stream) {
  if (bytes == 0) return ADASD_OK;
  if (!src || !sink) return ADASD_ERR_INVALID_ARG;
  if (!aligned_to(src, 16) || (bytes & 15) != 0 || !aligned_to(sink, 4)) return ADASD_ERR_MISALIGNED;
  const size_t groups = stream_read_groups(bytes);
  if (groups > 0x7fffffffu) return ADASD_ERR_CAPACITY;
  if (sink_words < groups) return ADASD_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  Scope sc(6, s);
  return launch_stream_read(src, bytes, sink, s) == hipSuccess ? ADASD_OK : ADASD_ERR_HIP;
}

int adasd_profile_enable(int max_launches) {
  if (max_launches < 1) return ADASD_ERR_INVALID_ARG;
  adasd_profile_disable();
  std::lock_guard<std::mutex> lk(g_prof.mu);
  for (int c = 0; c < kClasses; ++c) {
    g_prof.start[c].resize(max_launches);
    g_prof.stop[c].resize(max_launches);
    for (int i = 0; i < max_launches; ++i) {
      if (hipEventCreate(&g_prof.start[c][i]) != hipSuccess) return ADASD_ERR_HIP;
      if (hipEventCreate(&g_prof.stop[c][i]) != hipSuccess) return ADASD_ERR_HIP;
    }
    g_prof.used[c] = 0;
  }
  g_prof.cap = max_launches;
  g_prof.on = true;
  return ADASD_OK;
}

int adasd_profile_read(int kernel_class, double* total_ms, int* launches) {
  if (kernel_class < 0 || kernel_class >= kClasses || !total_ms || !launches) return ADASD_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lk(g_prof.mu);
  double sum = 0.0;
  const int n = g_prof.used[kernel_class];
  for (int i = 0; i < n; ++i) {
    if (hipEventSynchronize(g_prof.stop[kernel_class][i]) != hipSuccess) return ADASD_ERR_HIP;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, g_prof.start[kernel_class][i], g_prof.stop[kernel_class][i]) != hipSuccess)
      return ADASD_ERR_HIP;
    sum += ms;
  }
  *total_ms = sum;
  *launches = n;
  return ADASD_OK;
}

int adasd_profile_disable(void) {
  std::lock_guard<std::mutex> lk(g_prof.mu);
  for (int c = 0; c < kClasses; ++c) {
    for (auto e : g_prof.start[c]) (void)hipEventDestroy(e);
    for (auto e : g_prof.stop[c]) (void)hipEventDestroy(e);
    g_prof.start[c].clear();
    g_prof.stop[c].clear();
    g_prof.used[c] = 0;
  }
  g_prof.cap = 0;
  g_prof.on = false;
  return ADASD_OK;
}

}  // extern "C"
