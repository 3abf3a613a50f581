// Ceiling probes: what the machine delivers on the two resources that bound the CCQ kernels, measured with
// kernels that do nothing else.  ccq_probe_stream_read reads a buffer once with the same 16-byte nontemporal
// loads the decode kernels use for the code stream (no decode, no arithmetic worth naming): the achievable HBM
// rate for a launch of that size.  ccq_probe_mfma_bf16 issues back-to-back 32x32x16 bf16 MFMAs on register
// operands: the achievable matrix-core rate.  Both are part of the measurement, not of the hot path.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "ccq.h"

namespace ccq {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// Thread i requests units i, i + T, ..., i + (U-1) T (T = threads of the grid) before it uses any of them;
// indices past the end are clamped to the last unit, so every request is unconditional and in bounds.
template <int U>
__global__ void __launch_bounds__(512) ccq_probe_read_kernel(const u32x4* src, int64_t units, uint32_t* sink) {
  const int64_t T = (int64_t)gridDim.x * blockDim.x;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  u32x4 v[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int64_t j = i + (int64_t)u * T;
    v[u] = __builtin_nontemporal_load(src + (j < units ? j : units - 1));
  }
  uint32_t acc = 0;
#pragma unroll
  for (int u = 0; u < U; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  // keeps the loads alive without write traffic: one word pattern in 2^32 stores
  if (acc == 0x9E3779B9u) sink[0] = acc;
}

// Each wavefront keeps NA independent accumulator tiles going; operands come from memory once (distinct per
// lane, so that the data switching in the multipliers is that of real operands, which the clock depends on).
template <int NA>
__global__ void __launch_bounds__(256) ccq_probe_mfma_kernel(const bf16x8* operands, int iters, float* sink) {
  const int lane = threadIdx.x & 63;
  bf16x8 a[NA], b[NA];
  f32x16 acc[NA];
#pragma unroll
  for (int i = 0; i < NA; ++i) {
    a[i] = operands[(2 * i) * 64 + lane];
    b[i] = operands[(2 * i + 1) * 64 + lane];
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < NA; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[i], acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NA; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += acc[i][e];
  sink[(int64_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

}  // namespace ccq

using namespace ccq;

extern "C" int ccq_probe_stream_read(const void* src, int64_t bytes, int32_t loads_per_thread, int32_t block_threads, void* sink,
                                     void* hip_stream) {
  if (!src || !sink) return CCQ_ERR_NULL;
  if (bytes < 16 || bytes % 16 != 0) return CCQ_ERR_BAD_PARAM;
  if (block_threads < 64 || block_threads > 512 || block_threads % 64 != 0) return CCQ_ERR_BAD_PARAM;
  if ((reinterpret_cast<uintptr_t>(src) & 15u) || (reinterpret_cast<uintptr_t>(sink) & 3u)) return CCQ_ERR_ALIGN;
  const int64_t units = bytes / 16;
  const int u = loads_per_thread;
  if (u != 1 && u != 2 && u != 4 && u != 8) return CCQ_ERR_BAD_PARAM;
  const int64_t threads = (units + u - 1) / u;
  const int64_t blocks = (threads + block_threads - 1) / block_threads;
  if (blocks > 0x7FFFFFFF) return CCQ_ERR_BAD_PARAM;
  const dim3 grid((unsigned)blocks), block((unsigned)block_threads);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const u32x4* s = static_cast<const u32x4*>(src);
  uint32_t* k = static_cast<uint32_t*>(sink);
  if (u == 1) hipLaunchKernelGGL(ccq_probe_read_kernel<1>, grid, block, 0, st, s, units, k);
  else if (u == 2) hipLaunchKernelGGL(ccq_probe_read_kernel<2>, grid, block, 0, st, s, units, k);
  else if (u == 4) hipLaunchKernelGGL(ccq_probe_read_kernel<4>, grid, block, 0, st, s, units, k);
  else hipLaunchKernelGGL(ccq_probe_read_kernel<8>, grid, block, 0, st, s, units, k);
  return hipGetLastError() == hipSuccess ? CCQ_OK : CCQ_ERR_HIP;
}

extern "C" int ccq_probe_mfma_bf16(const void* operands, int32_t workgroups, int32_t iters, void* sink, void* hip_stream, double* flop_out) {
  if (!operands || !sink) return CCQ_ERR_NULL;
  if (workgroups < 1 || workgroups > (1 << 20) || iters < 1) return CCQ_ERR_BAD_PARAM;
  if ((reinterpret_cast<uintptr_t>(operands) & 15u) || (reinterpret_cast<uintptr_t>(sink) & 3u)) return CCQ_ERR_ALIGN;
  constexpr int NA = 4;
  hipLaunchKernelGGL(ccq_probe_mfma_kernel<NA>, dim3((unsigned)workgroups), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                     static_cast<const bf16x8*>(operands), iters, static_cast<float*>(sink));
  if (flop_out) *flop_out = 2.0 * 32 * 32 * 16 * NA * (double)iters * 4.0 * (double)workgroups;
  return hipGetLastError() == hipSuccess ? CCQ_OK : CCQ_ERR_HIP;
}
