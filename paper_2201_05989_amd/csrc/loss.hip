// Training losses (paper Section 4, "Training"): squared error (images, radiance fields) and the
// mean absolute percentage error |p - t| / (|t| + 0.01) (signed distance functions), as the
// gradient with respect to the network's output, which is what the backward pass of the network
// takes, plus the sum of the loss values for monitoring.  A streaming kernel over B * n_out
// scalars: 8 bytes read and 4 written per scalar; at the sizes of a training batch (2^18 scalars)
// it is one launch latency.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "hashgrid.h"

namespace hg {

constexpr int kLossThreads = 256;
constexpr float kMapeOffset = 0.01f;  // Section 4, "Training": the constant in the percentage error's denominator

// value and slope of one scalar's loss; fp32, the sign of p - t is exact (a difference of two floats
// is zero only if they are equal)
template <int KIND>
__device__ __forceinline__ void loss_scalar(float p, float t, float scale, float& slope, float& value) {
  const float diff = p - t;
  if (KIND == HG_LOSS_L2) {
    value = diff * diff;
    slope = scale * (2.0f * diff);
  } else {
    const float inv = 1.0f / (fabsf(t) + kMapeOffset);
    value = fabsf(diff) * inv;
    slope = diff > 0.0f ? scale * inv : (diff < 0.0f ? -(scale * inv) : diff);  // diff itself where it is 0 or NaN
  }
}

template <int KIND, bool VEC>
__global__ __launch_bounds__(kLossThreads) void loss_grad(const uint64_t n, const float* __restrict__ p,
                                                          const float* __restrict__ t, const float scale,
                                                          float* __restrict__ slope, double* __restrict__ loss_sum) {
  double sum = 0.0;
  const uint64_t first = (uint64_t)blockIdx.x * kLossThreads + threadIdx.x, stride = (uint64_t)gridDim.x * kLossThreads;
  const uint64_t n4 = VEC ? n / 4 : 0;
  for (uint64_t q = first; q < n4; q += stride) {
    const float4 pp = reinterpret_cast<const float4*>(p)[q], tt = reinterpret_cast<const float4*>(t)[q];
    float4 s;
    float v0, v1, v2, v3;
    loss_scalar<KIND>(pp.x, tt.x, scale, s.x, v0);
    loss_scalar<KIND>(pp.y, tt.y, scale, s.y, v1);
    loss_scalar<KIND>(pp.z, tt.z, scale, s.z, v2);
    loss_scalar<KIND>(pp.w, tt.w, scale, s.w, v3);
    reinterpret_cast<float4*>(slope)[q] = s;
    sum += ((double)v0 + (double)v1) + ((double)v2 + (double)v3);
  }
  for (uint64_t i = n4 * 4 + first; i < n; i += stride) {  // everything without VEC, else the last n mod 4 scalars
    float s, v;
    loss_scalar<KIND>(p[i], t[i], scale, s, v);
    slope[i] = s;
    sum += (double)v;
  }
  if (!loss_sum) return;  // uniform
  // one addition per workgroup: lanes, then waves
  __shared__ double part[kLossThreads / 64];
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) sum += __shfl_down(sum, o, 64);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x / 64] = sum;
  __syncthreads();
  if (threadIdx.x == 0) {
    double total = 0.0;
#pragma unroll
    for (int w = 0; w < kLossThreads / 64; ++w) total += part[w];
    atomicAdd(loss_sum, total);
  }
}

}  // namespace hg

extern "C" hg_status hashgrid_loss_grad(uint64_t n, const float* prediction, const float* target, uint32_t loss,
                                        float scale, float* dLdout, double* loss_sum, void* stream) {
  if (loss != HG_LOSS_L2 && loss != HG_LOSS_MAPE) return HG_ERR_INVALID_ARG;
  if (!(fabsf(scale) < INFINITY)) return HG_ERR_INVALID_ARG;
  if (n == 0) return HG_OK;
  if (!prediction || !target || !dLdout) return HG_ERR_INVALID_ARG;
  const uintptr_t bits = reinterpret_cast<uintptr_t>(prediction) | reinterpret_cast<uintptr_t>(target) |
                         reinterpret_cast<uintptr_t>(dLdout);
  if ((bits & 3) || (reinterpret_cast<uintptr_t>(loss_sum) & 7)) return HG_ERR_INVALID_ARG;
  const bool vec = (bits & 15) == 0;
  const uint64_t items = vec ? (n + 3) / 4 : n;
  // Few, fat workgroups: each ends with one atomic addition to the same word, and those are served one
  // after the other (256 workgroups that finish together spend 5 us there, more than the kernel's work
  // at the size of a training batch).
  constexpr uint64_t kItemsPerThread = 4;
  const uint64_t want = (items + hg::kLossThreads * kItemsPerThread - 1) / (hg::kLossThreads * kItemsPerThread);
  const uint32_t blocks = (uint32_t)(want > 512 ? 512 : want);
  hipStream_t s = static_cast<hipStream_t>(stream);
  using Kernel = void (*)(uint64_t, const float*, const float*, float, float*, double*);
  static const Kernel kernels[2][2] = {{hg::loss_grad<HG_LOSS_L2, false>, hg::loss_grad<HG_LOSS_L2, true>},
                                       {hg::loss_grad<HG_LOSS_MAPE, false>, hg::loss_grad<HG_LOSS_MAPE, true>}};
  hipLaunchKernelGGL(kernels[loss][vec ? 1 : 0], dim3(blocks), dim3(hg::kLossThreads), 0, s, n, prediction, target,
                     scale, dLdout, loss_sum);
  return hipGetLastError() == hipSuccess ? HG_OK : HG_ERR_DEVICE;
}
