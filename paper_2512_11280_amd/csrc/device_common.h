// Device-side helpers shared by the AdaSD kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/adasd.h"

namespace adasd {

constexpr int kBlock = 256;                 // threads per workgroup (4 wavefronts)
constexpr int kWaves = kBlock / 64;
constexpr float kLog2e = 1.44269504088896340736f;
constexpr double kLn2 = 0.693147180559945309417232;
constexpr float kNegHuge = -3.0e38f;        // finite stand-in for "no element seen yet"

// Kernel arguments are fetched with scalar loads where they are first needed, one 64-byte line at a
// time, and right after a launch every line misses all the way to memory: a kernel with a few
// hundred bytes of arguments pays that latency several times in a row before it issues its first
// load of data.  Touching every line at the very top makes those misses overlap.
template <int BYTES> __device__ __forceinline__ void warm_kernargs() {
  const __attribute__((address_space(4))) int* ka =
      (const __attribute__((address_space(4))) int*)__builtin_amdgcn_kernarg_segment_ptr();
  int t = 0;
#pragma unroll
  for (int off = 0; off < BYTES; off += 64) t ^= ka[off / 4];
  asm volatile("" ::"s"(t));
}

__device__ __forceinline__ float ex2(float x) { return __builtin_amdgcn_exp2f(x); }  // v_exp_f32
__device__ __forceinline__ float lg2(float x) { return __builtin_amdgcn_logf(x); }   // v_log_f32

// log2 of a positive finite float, as exponent + hardware log2 of the mantissa in [0.5, 1): absolute
// error about 6e-8 whatever the magnitude.  A handful of instructions, where the double-precision
// library routine is several hundred that a latency-bound kernel would have to fetch first.
__device__ __forceinline__ double log2_acc(float x) {
  int e;
  const float m = __builtin_frexpf(x, &e);
  return (double)e + (double)lg2(m);
}

// ---------------------------------------------------------------------------------------------
// Logit access.  A "vector" is 16 bytes: 8 bf16 or 4 fp32 logits.
// ---------------------------------------------------------------------------------------------
template <int DT> struct Elem;
template <> struct Elem<ADASD_BF16> { static constexpr int bytes = 2, per_vec = 8; };
template <> struct Elem<ADASD_F32> { static constexpr int bytes = 4, per_vec = 4; };

template <int DT> __device__ __forceinline__ float load_elem(const char* row, int64_t v) {
  if (DT == ADASD_BF16) {
    uint32_t w = (uint32_t)reinterpret_cast<const uint16_t*>(row)[v] << 16;
    return __uint_as_float(w);
  }
  return reinterpret_cast<const float*>(row)[v];
}

// The same in two steps, for a load whose value is only needed much later: the bits now, the float then
// (the wait for the load stands where the bits are first used).
template <int DT> __device__ __forceinline__ uint32_t load_elem_bits(const char* row, int64_t v) {
  if (DT == ADASD_BF16) return (uint32_t)reinterpret_cast<const uint16_t*>(row)[v];
  return reinterpret_cast<const uint32_t*>(row)[v];
}
template <int DT> __device__ __forceinline__ float elem_from_bits(uint32_t bits) {
  return __uint_as_float(DT == ADASD_BF16 ? bits << 16 : bits);
}

// Unpack one 16-byte vector into Elem<DT>::per_vec floats (exact conversions).
template <int DT> __device__ __forceinline__ void unpack(const uint4& q, float* z) {
  if (DT == ADASD_BF16) {
    z[0] = __uint_as_float(q.x << 16); z[1] = __uint_as_float(q.x & 0xffff0000u);
    z[2] = __uint_as_float(q.y << 16); z[3] = __uint_as_float(q.y & 0xffff0000u);
    z[4] = __uint_as_float(q.z << 16); z[5] = __uint_as_float(q.z & 0xffff0000u);
    z[6] = __uint_as_float(q.w << 16); z[7] = __uint_as_float(q.w & 0xffff0000u);
  } else {
    z[0] = __uint_as_float(q.x); z[1] = __uint_as_float(q.y);
    z[2] = __uint_as_float(q.z); z[3] = __uint_as_float(q.w);
  }
}

// ---------------------------------------------------------------------------------------------
// Online log-sum-exp state in the log2 domain: with x = z * log2(e),
//   m = reference (running max), s = sum 2^(x-m), u = sum (x-m) 2^(x-m).
// Then log2-sum-exp = m + log2 s and the entropy in nats is ln2 * (log2 s - u/s).
// ---------------------------------------------------------------------------------------------
struct Lse {
  float m, s, u;
};
__device__ __forceinline__ Lse lse_empty() { return Lse{kNegHuge, 0.f, 0.f}; }

__device__ __forceinline__ Lse lse_merge(const Lse& a, const Lse& b) {
  float m = fmaxf(a.m, b.m);
  float da = a.m - m, db = b.m - m;          // <= 0, finite unless a row holds +inf (then NaN: flagged later)
  float fa = ex2(da), fb = ex2(db);
  Lse r;
  r.m = m;
  r.s = a.s * fa + b.s * fb;
  r.u = (a.u + da * a.s) * fa + (b.u + db * b.s) * fb;
  return r;
}

// Add one logit z to a state whose reference st.m is already >= z*log2(e) (up to rounding).
// t = z*log2(e) - m is formed with ONE rounding, so elements near the maximum keep full relative
// accuracy however large the logits are.
__device__ __forceinline__ void lse_add(Lse& st, float z) {
  float t = fmaf(z, kLog2e, -st.m);
  t = (t < -200.f) ? -200.f : t;             // masked (-inf) logits contribute exactly 0; NaN passes through
  float e = ex2(t);
  st.s += e;
  st.u = fmaf(t, e, st.u);
}

__device__ __forceinline__ void lse_raise(Lse& st, float m_new) {
  if (m_new > st.m) {
    float d = st.m - m_new;
    float f = ex2(d);
    st.u = (st.u + d * st.s) * f;
    st.s *= f;
    st.m = m_new;
  }
}

__device__ __forceinline__ Lse wave_reduce(Lse v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    Lse o;
    o.m = __shfl_xor(v.m, off);
    o.s = __shfl_xor(v.s, off);
    o.u = __shfl_xor(v.u, off);
    v = lse_merge(v, o);
  }
  return v;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  return v;
}
__device__ __forceinline__ double wave_max(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmax(v, __shfl_xor(v, off));
  return v;
}

// Wavefront reductions on the data-parallel-primitive path: four rotations inside each row of 16 lanes
// leave every lane with its row's result; row 0's is then added into row 1 and row 2's into row 3
// (row_bcast:15), rows 0+1 into rows 2 and 3 (row_bcast:31), and lane 63 holds the result, grouped as
// (r0 + r1) + (r2 + r3).  Seven instructions, against fifteen with the four row results combined through
// scalar registers, and far shorter dependent chains than six LDS permutes.  All 64 lanes must be active.
template <int CTRL> __device__ __forceinline__ float dpp_rot(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float lane_value(float v, int lane) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}
// (Written as one data-parallel instruction per step where the compiler would not make one: from the builtin
// it makes a move, a canonicalising maximum and the maximum itself, and it has no form for a partial row
// mask.  A data-parallel operand must not be read in the two instruction slots after the instruction that
// wrote it, hence the s_nop.)
#define ADASD_DPP_OP(OP, v, CTRL) asm("s_nop 1\n\t" OP " %0, %0, %0 " CTRL : "+v"(v))
__device__ __forceinline__ float wave_sum_f(float v) {
  v += dpp_rot<0x121>(v);    // row_ror:1
  v += dpp_rot<0x122>(v);    // row_ror:2
  v += dpp_rot<0x124>(v);    // row_ror:4
  v += dpp_rot<0x128>(v);    // row_ror:8
  ADASD_DPP_OP("v_add_f32_dpp", v, "row_bcast:15 row_mask:0xa bank_mask:0xf");
  ADASD_DPP_OP("v_add_f32_dpp", v, "row_bcast:31 row_mask:0xc bank_mask:0xf");
  return lane_value(v, 63);
}
__device__ __forceinline__ float wave_max_f(float v) {
  ADASD_DPP_OP("v_max_f32_dpp", v, "row_ror:1 row_mask:0xf bank_mask:0xf");
  ADASD_DPP_OP("v_max_f32_dpp", v, "row_ror:2 row_mask:0xf bank_mask:0xf");
  ADASD_DPP_OP("v_max_f32_dpp", v, "row_ror:4 row_mask:0xf bank_mask:0xf");
  ADASD_DPP_OP("v_max_f32_dpp", v, "row_ror:8 row_mask:0xf bank_mask:0xf");
  ADASD_DPP_OP("v_max_f32_dpp", v, "row_bcast:15 row_mask:0xa bank_mask:0xf");
  ADASD_DPP_OP("v_max_f32_dpp", v, "row_bcast:31 row_mask:0xc bank_mask:0xf");
  return lane_value(v, 63);
}
#undef ADASD_DPP_OP

__device__ __forceinline__ uint32_t pk_max_f16(uint32_t a, uint32_t b) {
  uint32_t r;
  asm("v_pk_max_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}

template <int DT> __device__ __forceinline__ uint4 neutral_vec() {   // all logits -inf
  return DT == ADASD_BF16 ? make_uint4(0xFF80FF80u, 0xFF80FF80u, 0xFF80FF80u, 0xFF80FF80u)
                          : make_uint4(0xFF800000u, 0xFF800000u, 0xFF800000u, 0xFF800000u);
}

// Largest finite logit held in NV vectors, times log2(e) (kNegHuge if there is none).
// bf16 pairs are compared as packed f16: both formats order their bit patterns the same way, and
// the bf16 patterns of +-inf / NaN read as f16 NaNs, which the packed max ignores.
template <int DT, int NV> __device__ __forceinline__ float vecs_max(const uint4 (&v)[NV]) {
  if (DT == ADASD_BF16) {
    uint32_t m = pk_max_f16(v[0].x, v[0].y);
    m = pk_max_f16(m, v[0].z);
    m = pk_max_f16(m, v[0].w);
#pragma unroll
    for (int j = 1; j < NV; ++j) {
      m = pk_max_f16(m, v[j].x);
      m = pk_max_f16(m, v[j].y);
      m = pk_max_f16(m, v[j].z);
      m = pk_max_f16(m, v[j].w);
    }
    // a half whose f16 exponent field is all ones was never a finite logit of sane size
    uint32_t lo = m << 16, hi = m & 0xffff0000u;
    float flo = ((m & 0x7C00u) == 0x7C00u) ? kNegHuge : __uint_as_float(lo) * kLog2e;
    float fhi = ((m & 0x7C000000u) == 0x7C000000u) ? kNegHuge : __uint_as_float(hi) * kLog2e;
    return fmaxf(flo, fhi);
  } else {
    float m = kNegHuge;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      float a = __uint_as_float(v[j].x), b = __uint_as_float(v[j].y);
      float c = __uint_as_float(v[j].z), d = __uint_as_float(v[j].w);
      m = fmaxf(m, fmaxf(fmaxf(a, b), fmaxf(c, d)));   // NaN-ignoring; +inf surfaces in the sums
    }
    return (m > kNegHuge && m < INFINITY) ? m * kLog2e : kNegHuge;
  }
}

// Phase-1 accumulation of one vector into per-lane sums relative to the reference m.
// (neg_m = -m: a caller whose reference is wave-uniform hands it over in a vector register; as a scalar it
// would be the second scalar operand of the multiply-add next to log2(e), which the instruction cannot
// take, and the compiler copies it into a vector register again and again.)
template <int DT>
__device__ __forceinline__ void lse_accum_neg(const uint4& v, float neg_m, float& s0, float& s1, float& u0, float& u1) {
  constexpr int EPV = Elem<DT>::per_vec;
  float z[EPV];
  unpack<DT>(v, z);
#pragma unroll
  for (int e = 0; e < EPV; e += 2) {
    float t0 = fmaf(z[e], kLog2e, neg_m), t1 = fmaf(z[e + 1], kLog2e, neg_m);
    float e0 = ex2(t0), e1 = ex2(t1);
    s0 += e0;
    s1 += e1;
    u0 = fmaf(fmaxf(t0, -200.f), e0, u0);   // masked logits: (-200) * 0 = 0; a NaN stays one through e
    u1 = fmaf(fmaxf(t1, -200.f), e1, u1);
  }
}
template <int DT>
__device__ __forceinline__ void lse_accum(const uint4& v, float m, float& s0, float& s1, float& u0, float& u1) {
  constexpr int EPV = Elem<DT>::per_vec;
  float z[EPV];
  unpack<DT>(v, z);
#pragma unroll
  for (int e = 0; e < EPV; e += 2) {
    float t0 = fmaf(z[e], kLog2e, -m), t1 = fmaf(z[e + 1], kLog2e, -m);
    float e0 = ex2(t0), e1 = ex2(t1);
    s0 += e0;
    s1 += e1;
    u0 = fmaf(fmaxf(t0, -200.f), e0, u0);   // masked logits: (-200) * 0 = 0; a NaN stays one through e
    u1 = fmaf(fmaxf(t1, -200.f), e1, u1);
  }
}


// Cross-workgroup hand-off without a cache write-back.  An agent-scope fence on gfx950 writes back
// and invalidates the XCD's whole L2, which serialises badly when every workgroup does it.  Instead
// every word that travels between workgroups is written and read with agent-scope ATOMIC accesses, the
// writer waits for its stores to complete (publish_barrier) before it bumps the arrival counter, and the
// reader only issues its loads after the counter's value has come back (control dependency).
//
// Why that is enough, also between workgroups on different XCDs (whose L2 caches are not coherent with
// each other).  The code sequences the memory model prescribes for a release and an acquire at agent
// scope are "write back L2; wait for all memory operations; atomic" and "atomic; invalidate L1/L2".  The
// write-back and the invalidate exist for the ORDINARY stores and loads around the atomic: ordinary data
// may sit dirty in the writer's L2 or stale in the reader's caches.  An agent-scope atomic store itself is
// performed at the memory side of the L2s (it is written through), and an agent-scope atomic load never
// takes a line from a cache that is not coherent at that scope.  Here the payload consists of such
// accesses only, so nothing is left for the cache maintenance to do; what remains of the release is the
// wait for the payload stores to have completed before the counter's read-modify-write is issued
// (s_waitcnt 0 below: a write-through store counts as complete when the memory side has acknowledged it),
// and what remains of the acquire is that the payload loads are issued after the counter's value is known,
// which the branch on that value and the in-order issue of a wavefront give.  The single-read statistics
// kernel does not even need that much: its words carry their own validity (stats_fused.hip).
__device__ __forceinline__ void st_agent(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(int* p, int v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void publish_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_s_waitcnt(0);   // all outstanding memory operations of this wave have completed
}
__device__ __forceinline__ float ld_agent(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int ld_agent(const int* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ double ld_agent(const double* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ---------------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11).
// ---------------------------------------------------------------------------------------------
struct U4 {
  uint32_t w[4];
};
__device__ __forceinline__ U4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                            uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    uint64_t a = (uint64_t)0xD2511F53u * c0;
    uint64_t b = (uint64_t)0xCD9E8D57u * c2;
    // (three-input exclusive or in one instruction: left to itself the compiler makes two of each)
    uint32_t n0 = __builtin_amdgcn_bitop3_b32((uint32_t)(b >> 32), c1, k0, 0x96);
    uint32_t n2 = __builtin_amdgcn_bitop3_b32((uint32_t)(a >> 32), c3, k1, 0x96);
    c1 = (uint32_t)b;
    c3 = (uint32_t)a;
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return U4{{c0, c1, c2, c3}};
}

// ---------------------------------------------------------------------------------------------
// Workspace layout (device memory, carved by the host from one allocation).
// ---------------------------------------------------------------------------------------------
struct RowResult {   // one per logit row
  double lse2;       // log2-sum-exp of the row: m + log2 s   (natural lse = lse2 * ln 2)
  float H;           // entropy, nats
  int32_t bad;       // 1: NaN/+inf logit or no finite logit
};

struct SamplePlan {  // one per sequence, written by the decision kernel
  int32_t row;       // position index r whose row(s) are sampled (k_b for the bonus row)
  int32_t residual;  // 1: sample max(0, p_r - q_r); 0: sample p_row; 2: sample p_row without token `excluded`
  int32_t valid;     // 0: the needed row is non-finite -> token -1
  int32_t excluded;  // token index left out in mode 2, else -1
  double lse2_p, lse2_q;
};

struct PosRecord {   // outcome of one position, left by the long-history decision kernel for the sequence's last workgroup
  int32_t bits;      // 1: position accepted, 2: row pair broken
  uint32_t status;
  float d;           // the distance as written to d_js
  float pad;
};

struct Top2 {        // running best / runner-up of the Gumbel keys (log2 domain)
  float k1; int32_t i1;
  float k2; int32_t i2;
};

}  // namespace adasd
