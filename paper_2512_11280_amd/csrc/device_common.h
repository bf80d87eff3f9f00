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

__device__ __forceinline__ float ex2(float x) { return __builtin_amdgcn_exp2f(x); }  // v_exp_f32
__device__ __forceinline__ float lg2(float x) { return __builtin_amdgcn_logf(x); }   // v_log_f32

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

// Cross-workgroup hand-off without a cache write-back.  An agent-scope fence on gfx950 writes back
// and invalidates the XCD's whole L2, which serialises badly when every workgroup does it.  Instead
// the few words that travel between workgroups are written and read with agent-scope atomic
// accesses (they bypass the non-coherent cache levels), the writer waits for its stores to complete
// (publish_barrier) before it bumps the arrival counter, and the reader only issues its loads after
// the counter's value has come back (control dependency).
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
    uint32_t n0 = (uint32_t)(b >> 32) ^ c1 ^ k0;
    uint32_t n2 = (uint32_t)(a >> 32) ^ c3 ^ k1;
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
  int32_t residual;  // 1: sample max(0, p_r - q_r); 0: sample p_row
  int32_t valid;     // 0: the needed row is non-finite -> token -1
  int32_t pad;
  double lse2_p, lse2_q;
};

struct Top2 {        // running best / runner-up of the Gumbel keys (log2 domain)
  float k1; int32_t i1;
  float k2; int32_t i2;
};

}  // namespace adasd
