// Machine probes (libhashgrid_probes, declared in include/hashgrid_probes.h): small kernels
// that measure, on the GPU at hand, the rates the encoding's passes are compared with -
// streaming copy (HBM), random 4-byte gathers from a table of a given size (L2 or memory-side
// request rate), random fp32 atomic adds (device-scope atomic rate) and line fetches in the
// access shape of the forward pass.  They are not part of the method; the caller times them.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hashgrid_probes.h"

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

// The forward pass's access shape on hashed levels: per point and level four lines, two adjacent
// words in each, a barrier per level, a new slice every level.
constexpr int kLineProbeThreads = 1024;
__global__ __launch_bounds__(kLineProbeThreads) void probe_gather_lines(const uint32_t* __restrict__ table,
                                                                        const uint32_t slice_words,
                                                                        const uint32_t n_slices, const uint32_t n_levels,
                                                                        const uint32_t seed, uint32_t* __restrict__ sink) {
  const uint32_t tid = blockIdx.x * kLineProbeThreads + threadIdx.x;
  const uint32_t mask = slice_words - 1u;
  uint32_t h = mix32(tid * 2654435761u + seed), sum = 0;
  for (uint32_t l = 0; l < n_levels; ++l) {
    const uint32_t* t = table + (uint64_t)(l % n_slices) * slice_words;
    uint32_t v[8];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      h = mix32(h + (uint32_t)r * 0x9e3779b9u + l);
      const uint32_t i = h & mask;
      v[2 * r] = t[i];
      v[2 * r + 1] = t[i ^ 1u];
    }
#pragma unroll
    for (int r = 0; r < 8; ++r) sum += v[r];
    __syncthreads();
  }
  sink[tid] = sum;
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

hg_status hashgrid_probe_gather_lines(const uint32_t* table, uint64_t slice_words, uint32_t n_slices,
                                      uint64_t n_points, uint32_t n_levels, uint32_t seed, uint32_t* sink,
                                      void* stream) {
  if (n_points == 0 || n_levels == 0) return HG_OK;
  if (!table || !sink || !hg::pow2(slice_words) || slice_words < 32 || slice_words > (1ull << 31) || n_slices == 0 ||
      n_points % hg::kLineProbeThreads || n_points / hg::kLineProbeThreads > 0x7fffffffull)
    return HG_ERR_INVALID_ARG;
  hipLaunchKernelGGL(hg::probe_gather_lines, dim3((uint32_t)(n_points / hg::kLineProbeThreads)),
                     dim3(hg::kLineProbeThreads), 0, static_cast<hipStream_t>(stream), table, (uint32_t)slice_words,
                     n_slices, n_levels, seed, sink);
  return hipGetLastError() == hipSuccess ? HG_OK : HG_ERR_DEVICE;
}

}  // extern "C"
