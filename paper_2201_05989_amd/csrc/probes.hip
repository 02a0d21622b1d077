// Machine probes: three small kernels that measure, on the GPU at hand, the rates
// the encoding's passes are compared with - streaming copy (HBM), random 4-byte
// gathers from a table of a given size (L2 or memory-side request rate) and random
// fp32 atomic adds (device-scope atomic rate).  They are not part of the method;
// the caller times them.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hashgrid.h"

namespace hg {

constexpr int kProbeThreads = 256;
constexpr int kProbePerThread = 16;  // independent accesses per thread, all in flight together

// a 32-bit mixer (xorshift-multiply rounds): decorrelates consecutive thread ids
__device__ __forceinline__ uint32_t mix32(uint32_t v) {
  v ^= v >> 16;
  v *= 0x7feb352du;
  v ^= v >> 15;
  v *= 0x846ca68bu;
  v ^= v >> 16;
  return v;
}

using f32x4 = float __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(kProbeThreads) void probe_copy(const f32x4* __restrict__ src, f32x4* __restrict__ dst,
                                                            const uint64_t n_vec) {
  const uint64_t stride = (uint64_t)gridDim.x * kProbeThreads;
  for (uint64_t i = (uint64_t)blockIdx.x * kProbeThreads + threadIdx.x; i < n_vec; i += stride) dst[i] = src[i];
}

__global__ __launch_bounds__(kProbeThreads) void probe_gather(const uint32_t* __restrict__ table, const uint32_t mask,
                                                              const uint32_t seed, uint32_t* __restrict__ sink) {
  const uint32_t tid = blockIdx.x * kProbeThreads + threadIdx.x;
  uint32_t h = mix32(tid * 2654435761u + seed), sum = 0;
#pragma unroll
  for (int j = 0; j < kProbePerThread; ++j) {
    h = mix32(h + (uint32_t)j * 0x9e3779b9u);
    sum += table[h & mask];
  }
  sink[tid] = sum;
}

__global__ __launch_bounds__(kProbeThreads) void probe_atomic_add(float* __restrict__ table, const uint32_t mask,
                                                                  const uint32_t seed) {
  const uint32_t tid = blockIdx.x * kProbeThreads + threadIdx.x;
  uint32_t h = mix32(tid * 2654435761u + seed);
#pragma unroll
  for (int j = 0; j < kProbePerThread; ++j) {
    h = mix32(h + (uint32_t)j * 0x9e3779b9u);
    __hip_atomic_fetch_add(table + (h & mask), 1.0f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

static bool pow2(uint64_t v) { return v && !(v & (v - 1)); }

}  // namespace hg

extern "C" {

hg_status hashgrid_probe_copy(const void* src, void* dst, uint64_t bytes, void* stream) {
  if (bytes == 0) return HG_OK;
  if (!src || !dst || (bytes & 15) || ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15))
    return HG_ERR_INVALID_ARG;
  const uint64_t n_vec = bytes / 16;
  const uint64_t want = (n_vec + hg::kProbeThreads - 1) / hg::kProbeThreads;
  const uint32_t grid = (uint32_t)(want < 16384 ? want : 16384);  // 64 workgroups per CU, grid-stride beyond
  hipLaunchKernelGGL(hg::probe_copy, dim3(grid), dim3(hg::kProbeThreads), 0, static_cast<hipStream_t>(stream),
                     static_cast<const hg::f32x4*>(src), static_cast<hg::f32x4*>(dst), n_vec);
  return hipGetLastError() == hipSuccess ? HG_OK : HG_ERR_DEVICE;
}

hg_status hashgrid_probe_gather(const uint32_t* table, uint64_t table_words, uint64_t n_gathers, uint32_t seed,
                                uint32_t* sink, void* stream) {
  const uint64_t per_wg = (uint64_t)hg::kProbeThreads * hg::kProbePerThread;
  if (n_gathers == 0) return HG_OK;
  if (!table || !sink || !hg::pow2(table_words) || table_words > (1ull << 32) || n_gathers % per_wg ||
      n_gathers / per_wg > 0x7fffffffull)
    return HG_ERR_INVALID_ARG;
  hipLaunchKernelGGL(hg::probe_gather, dim3((uint32_t)(n_gathers / per_wg)), dim3(hg::kProbeThreads), 0,
                     static_cast<hipStream_t>(stream), table, (uint32_t)(table_words - 1), seed, sink);
  return hipGetLastError() == hipSuccess ? HG_OK : HG_ERR_DEVICE;
}

hg_status hashgrid_probe_atomic_add(float* table, uint64_t table_words, uint64_t n_adds, uint32_t seed,
                                    void* stream) {
  const uint64_t per_wg = (uint64_t)hg::kProbeThreads * hg::kProbePerThread;
  if (n_adds == 0) return HG_OK;
  if (!table || !hg::pow2(table_words) || table_words > (1ull << 32) || n_adds % per_wg ||
      n_adds / per_wg > 0x7fffffffull)
    return HG_ERR_INVALID_ARG;
  hipLaunchKernelGGL(hg::probe_atomic_add, dim3((uint32_t)(n_adds / per_wg)), dim3(hg::kProbeThreads), 0,
                     static_cast<hipStream_t>(stream), table, (uint32_t)(table_words - 1), seed);
  return hipGetLastError() == hipSuccess ? HG_OK : HG_ERR_DEVICE;
}

}  // extern "C"
