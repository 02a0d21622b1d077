// Optimiser step on the tables (paper Section 4, "Training"): Adam with the
// caller's beta1, beta2, eps (the paper: 0.9, 0.99, 1e-15), the L2 regularisation the
// paper puts on the network's weights and not on table entries (a factor, 0 for the
// tables), entries whose gradient is exactly 0 skipped, full-precision
// master copy plus a half-precision working copy (Section 4, "Performance
// considerations").  A pure streaming kernel: per updated scalar it reads 16
// bytes (gradient, two moments, master value) and writes 14 to 18 (moments,
// master, fp16 copy, and the gradient's zero when asked to clear it); a group
// of four scalars whose gradients are all zero costs 16 bytes of reads and no
// write at all.  The gradient may also be the half-precision one of grad_dtype = fp16 (8 bytes
// per group), multiplied by the reciprocal of the caller's loss scale as it is read.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "hashgrid.h"

namespace hg {

constexpr int kAdamThreads = 256;

struct AdamArgs {
  float lr, beta1, beta2, eps, l2;
  float inv_c1;       // 1 / (1 - beta1^t)
  float inv_sqrt_c2;  // 1 / sqrt(1 - beta2^t)
};

__device__ __forceinline__ void adam_scalar(const AdamArgs& a, float g, float& m, float& v, float& p) {
  m = a.beta1 * m + (1.0f - a.beta1) * g;
  v = a.beta2 * v + (1.0f - a.beta2) * g * g;
  p -= a.lr * (m * a.inv_c1) / (sqrtf(v) * a.inv_sqrt_c2 + a.eps);
}

// Four gradient scalars of either type as floats, times grad_scale for the half-precision ones (what
// undoes the scaling of the loss that keeps half-precision gradients out of the subnormals).
struct alignas(8) Half4 {
  _Float16 h[4];
};
__device__ __forceinline__ float4 load_grad4(const float* g, uint64_t q, float) {
  return reinterpret_cast<const float4*>(g)[q];
}
__device__ __forceinline__ float4 load_grad4(const _Float16* g, uint64_t q, float scale) {
  const Half4 h = reinterpret_cast<const Half4*>(g)[q];
  return make_float4((float)h.h[0] * scale, (float)h.h[1] * scale, (float)h.h[2] * scale, (float)h.h[3] * scale);
}
__device__ __forceinline__ void zero_grad4(float* g, uint64_t q) {
  reinterpret_cast<float4*>(g)[q] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
}
__device__ __forceinline__ void zero_grad4(_Float16* g, uint64_t q) { reinterpret_cast<Half4*>(g)[q] = Half4{}; }

template <bool ZERO_GRAD, typename GT>
__global__ __launch_bounds__(kAdamThreads) void adam_step(const AdamArgs a, const uint64_t n, float* __restrict__ p32,
                                                          _Float16* __restrict__ p16, GT* __restrict__ grad,
                                                          float* __restrict__ m, float* __restrict__ v,
                                                          const float grad_scale) {
  const uint64_t n4 = n / 4;
  for (uint64_t q = (uint64_t)blockIdx.x * kAdamThreads + threadIdx.x; q < n4; q += (uint64_t)gridDim.x * kAdamThreads) {
    float4 g = load_grad4(grad, q, grad_scale);
    // (without the regulariser: nothing to read further and nothing to write where the four gradients are zero)
    if (a.l2 == 0.0f && g.x == 0.0f && g.y == 0.0f && g.z == 0.0f && g.w == 0.0f) continue;
    float4 mm = reinterpret_cast<const float4*>(m)[q];
    float4 vv = reinterpret_cast<const float4*>(v)[q];
    float4 pp = reinterpret_cast<const float4*>(p32)[q];
    if (a.l2 != 0.0f) {  // uniform: the L2 regularisation's term in the gradient
      g.x = fmaf(a.l2, pp.x, g.x);
      g.y = fmaf(a.l2, pp.y, g.y);
      g.z = fmaf(a.l2, pp.z, g.z);
      g.w = fmaf(a.l2, pp.w, g.w);
      if (g.x == 0.0f && g.y == 0.0f && g.z == 0.0f && g.w == 0.0f) {
        if (ZERO_GRAD) zero_grad4(grad, q);
        continue;
      }
    }
    if (g.x != 0.0f) adam_scalar(a, g.x, mm.x, vv.x, pp.x);
    if (g.y != 0.0f) adam_scalar(a, g.y, mm.y, vv.y, pp.y);
    if (g.z != 0.0f) adam_scalar(a, g.z, mm.z, vv.z, pp.z);
    if (g.w != 0.0f) adam_scalar(a, g.w, mm.w, vv.w, pp.w);
    reinterpret_cast<float4*>(m)[q] = mm;
    reinterpret_cast<float4*>(v)[q] = vv;
    reinterpret_cast<float4*>(p32)[q] = pp;
    if (p16) {
      Half4 h;
      h.h[0] = (_Float16)pp.x;
      h.h[1] = (_Float16)pp.y;
      h.h[2] = (_Float16)pp.z;
      h.h[3] = (_Float16)pp.w;
      reinterpret_cast<Half4*>(p16)[q] = h;
    }
    if (ZERO_GRAD) zero_grad4(grad, q);
  }
  // tail of fewer than four scalars
  if (blockIdx.x == 0 && threadIdx.x < n - n4 * 4) {
    const uint64_t i = n4 * 4 + threadIdx.x;
    float g = sizeof(GT) == 2 ? (float)grad[i] * grad_scale : (float)grad[i];
    float mm = m[i], vv = v[i], pp = p32[i];
    g = a.l2 != 0.0f ? fmaf(a.l2, pp, g) : g;
    if (ZERO_GRAD && a.l2 != 0.0f) grad[i] = (GT)0.0f;
    if (g != 0.0f) {
      adam_scalar(a, g, mm, vv, pp);
      m[i] = mm;
      v[i] = vv;
      p32[i] = pp;
      if (p16) p16[i] = (_Float16)pp;
      if (ZERO_GRAD) grad[i] = (GT)0.0f;
    }
  }
}

}  // namespace hg

namespace {

template <typename GT>
hg_status adam_launch(uint64_t n_scalars, float* params_master, void* params_half, GT* grad, float* m, float* v,
                      const hashgrid_adam_config* cfg, uint32_t step, int zero_grad, float grad_scale, void* stream) {
  if (!cfg || step == 0) return HG_ERR_INVALID_ARG;
  if (n_scalars == 0) return HG_OK;
  if (!params_master || !grad || !m || !v) return HG_ERR_INVALID_ARG;
  if (!(cfg->beta1 >= 0.0f && cfg->beta1 < 1.0f && cfg->beta2 >= 0.0f && cfg->beta2 < 1.0f && cfg->eps >= 0.0f &&
        cfg->l2_reg >= 0.0f && cfg->l2_reg < INFINITY))
    return HG_ERR_INVALID_ARG;
  if (!(grad_scale > 0.0f && grad_scale < INFINITY)) return HG_ERR_INVALID_ARG;
  const uintptr_t bits = reinterpret_cast<uintptr_t>(params_master) | reinterpret_cast<uintptr_t>(m) |
                         reinterpret_cast<uintptr_t>(v);
  if ((bits & 15) || (reinterpret_cast<uintptr_t>(params_half) & 7) ||
      (reinterpret_cast<uintptr_t>(grad) & (4 * sizeof(GT) - 1)))
    return HG_ERR_INVALID_ARG;
  hg::AdamArgs a;
  a.lr = cfg->lr;
  a.beta1 = cfg->beta1;
  a.beta2 = cfg->beta2;
  a.eps = cfg->eps;
  a.l2 = cfg->l2_reg;
  a.inv_c1 = (float)(1.0 / (1.0 - pow((double)cfg->beta1, (double)step)));
  a.inv_sqrt_c2 = (float)(1.0 / sqrt(1.0 - pow((double)cfg->beta2, (double)step)));
  const uint64_t groups = (n_scalars / 4 + hg::kAdamThreads - 1) / hg::kAdamThreads;
  const uint32_t blocks = (uint32_t)(groups < 1 ? 1 : (groups > 65536 ? 65536 : groups));
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (zero_grad)
    hipLaunchKernelGGL((hg::adam_step<true, GT>), dim3(blocks), dim3(hg::kAdamThreads), 0, s, a, n_scalars, params_master,
                       static_cast<_Float16*>(params_half), grad, m, v, grad_scale);
  else
    hipLaunchKernelGGL((hg::adam_step<false, GT>), dim3(blocks), dim3(hg::kAdamThreads), 0, s, a, n_scalars, params_master,
                       static_cast<_Float16*>(params_half), grad, m, v, grad_scale);
  return hipGetLastError() == hipSuccess ? HG_OK : HG_ERR_DEVICE;
}

}  // namespace

extern "C" hg_status hashgrid_adam_step(uint64_t n_scalars, float* params_master, void* params_half, float* grad,
                                        float* m, float* v, const hashgrid_adam_config* cfg, uint32_t step,
                                        int zero_grad, void* stream) {
  return adam_launch<float>(n_scalars, params_master, params_half, grad, m, v, cfg, step, zero_grad, 1.0f, stream);
}

extern "C" hg_status hashgrid_adam_step_half_grad(uint64_t n_scalars, float* params_master, void* params_half,
                                                  void* grad_half, float* m, float* v,
                                                  const hashgrid_adam_config* cfg, uint32_t step, int zero_grad,
                                                  float grad_scale, void* stream) {
  return adam_launch<_Float16>(n_scalars, params_master, params_half, static_cast<_Float16*>(grad_half), m, v, cfg,
                               step, zero_grad, grad_scale, stream);
}
