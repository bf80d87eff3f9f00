// Diagnostics: a plain streaming read in the launch shape of the statistics kernels (one workgroup per
// 32 KiB piece, every 128-bit load of a thread requested before the first is used).  It gives the rate
// at which this chip delivers the logits to a kernel that does nothing with them: the practical ceiling
// that the statistics kernels' bandwidth figures are read against.
#include "device_common.h"
#include "internal.h"

namespace adasd {

namespace {

constexpr int kStreamVecs = 8;   // 128-bit vectors per thread

__global__ void __launch_bounds__(kBlock)
k_stream_read(const uint4* __restrict__ src, size_t n_vec, uint32_t* __restrict__ sink) {
  const size_t base = (size_t)blockIdx.x * (kStreamVecs * kBlock);
  uint4 v[kStreamVecs];
#pragma unroll
  for (int j = 0; j < kStreamVecs; ++j) {
    const size_t idx = base + threadIdx.x + (size_t)j * kBlock;
    v[j] = idx < n_vec ? src[idx] : make_uint4(0u, 0u, 0u, 0u);
  }
  uint32_t x = 0u;
#pragma unroll
  for (int j = 0; j < kStreamVecs; ++j) x ^= v[j].x ^ v[j].y ^ v[j].z ^ v[j].w;
  // one word per workgroup, so that the loads cannot be dropped; which lane writes depends on the data
  // only through the value written
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x ^= __shfl_xor(x, off);
  __shared__ uint32_t sh[kWaves];
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = x;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t t = 0u;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) t ^= sh[w];
    sink[blockIdx.x] = t;
  }
}

}  // namespace

size_t stream_read_groups(size_t bytes) {
  const size_t per_group = (size_t)kStreamVecs * kBlock * sizeof(uint4);
  return (bytes + per_group - 1) / per_group;
}

hipError_t launch_stream_read(const void* src, size_t bytes, uint32_t* sink, hipStream_t st) {
  const size_t groups = stream_read_groups(bytes);
  if (groups == 0) return hipSuccess;
  launch_kernel(k_stream_read, dim3((unsigned)groups), dim3(kBlock), st, reinterpret_cast<const uint4*>(src),
                bytes / sizeof(uint4), sink);
  return hipGetLastError();
}

}  // namespace adasd
