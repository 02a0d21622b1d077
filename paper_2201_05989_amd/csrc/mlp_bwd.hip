// Backward pass of the paper's small network (Section 4, "Architecture": two hidden layers of 64
// neurons, ReLU, linear output layer) on the matrix cores: from the encoded features y and the
// upstream gradient dL/dout to dL/dy (which hashgrid_encode_bwd[_ws] then takes to the tables) and
// the gradients of the three weight matrices, in one kernel.  Hidden activations are recomputed
// from y (they never existed in memory: the forward kernel keeps them in LDS), so nothing but y
// has to be kept from the forward pass.
//
// Work unit: one wave and 32 points.  Everything a wave needs of its 32 points lives in its own
// LDS rows [point][neuron] (padded as in the forward kernel); a gradient matrix overwrites the
// activation whose ReLU mask it has just used.  Products, all v_mfma_f32_32x32x8_f16 (fp16
// operands, fp32 accumulation), D[i][j] = sum_k A[i][k] B[k][j] with, per lane l:
//   A: row i = l % 32, k = 4 (l / 32) .. + 3;  B: column j = l % 32, the same k;
//   D: column j = l % 32, rows i = 8 (r / 4) + 4 (l / 32) + r % 4, r = 0 .. 15.
//   forward and data gradients contract over neurons: both operands are 8-byte reads of four
//     consecutive neurons of one LDS row (weights [out][in], or transposed copies [in][out]);
//   weight gradients contract over the 32 points: both operands are columns of the point rows
//     (four 2-byte reads, a row apart); their sums stay in registers while the wave walks its
//     blocks of points, are then added up across the workgroup's waves in LDS and leave with one
//     atomic add per scalar and workgroup.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hashgrid.h"

namespace hg {

constexpr int kHid = 64;      // neurons of a hidden layer
constexpr int kPad = 4;       // halves of padding per LDS row
constexpr int kHidStride = kHid + kPad;
constexpr int kPts = 32;      // points of a wave's block

using half4 = _Float16 __attribute__((ext_vector_type(4)));
using float16v = float __attribute__((ext_vector_type(16)));

__device__ __forceinline__ float16v zero16() {
  float16v z;
#pragma unroll
  for (int i = 0; i < 16; ++i) z[i] = 0.0f;
  return z;
}

// acc[i][j] += sum_k a[i][k] * b[j][k]: rows i of `a`, rows j of `b`, 8 * ksteps consecutive k each
__device__ __forceinline__ float16v mm_rows(const _Float16* __restrict__ a, int a_stride, const _Float16* __restrict__ b,
                                            int b_stride, int ksteps, float16v acc) {
  const int lane = threadIdx.x & 63, r = lane & 31, k0 = 4 * (lane >> 5);
  const _Float16* pa = a + r * a_stride + k0;
  const _Float16* pb = b + r * b_stride + k0;
  for (int ks = 0; ks < ksteps; ++ks)
    acc = __builtin_amdgcn_mfma_f32_32x32x8f16(*reinterpret_cast<const half4*>(pa + 8 * ks),
                                               *reinterpret_cast<const half4*>(pb + 8 * ks), acc, 0, 0, 0);
  return acc;
}

// acc[i][j] += sum_p x[p][i0 + i] * z[p][j0 + j] over the 32 rows p of `x` and `z`
__device__ __forceinline__ float16v mm_cols(const _Float16* __restrict__ x, int x_stride, int i0,
                                            const _Float16* __restrict__ z, int z_stride, int j0, float16v acc) {
  const int lane = threadIdx.x & 63, r = lane & 31, k0 = 4 * (lane >> 5);
#pragma unroll
  for (int ks = 0; ks < kPts / 8; ++ks) {
    half4 a, b;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      a[t] = x[(8 * ks + k0 + t) * x_stride + i0 + r];
      b[t] = z[(8 * ks + k0 + t) * z_stride + j0 + r];
    }
    acc = __builtin_amdgcn_mfma_f32_32x32x8f16(a, b, acc, 0, 0, 0);
  }
  return acc;
}

// A lane's 16 results of one block are point p = lane % 32, neurons n0 + 8 q + 4 (lane / 32) + t.
// relu, round to half, store into rows[p][n]
__device__ __forceinline__ void store_relu(_Float16* __restrict__ rows, int stride, int n0, const float16v& acc) {
  const int lane = threadIdx.x & 63;
  _Float16* row = rows + (lane & 31) * stride + n0 + 4 * (lane >> 5);
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    half4 h;
#pragma unroll
    for (int t = 0; t < 4; ++t) h[t] = (_Float16)fmaxf(acc[4 * q + t], 0.0f);
    *reinterpret_cast<half4*>(row + 8 * q) = h;
  }
}
// the gradient of a ReLU layer, in place of its activations: rows[p][n] = half(acc) where rows[p][n] > 0, else 0
__device__ __forceinline__ void store_masked(_Float16* __restrict__ rows, int stride, int n0, const float16v& acc) {
  const int lane = threadIdx.x & 63;
  _Float16* row = rows + (lane & 31) * stride + n0 + 4 * (lane >> 5);
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const half4 act = *reinterpret_cast<const half4*>(row + 8 * q);
    half4 g;
#pragma unroll
    for (int t = 0; t < 4; ++t) g[t] = act[t] > (_Float16)0.0f ? (_Float16)acc[4 * q + t] : (_Float16)0.0f;
    *reinterpret_cast<half4*>(row + 8 * q) = g;
  }
}

struct MlpBwdShape {
  int n_in, n_out;
  int kin_pad;   // n_in rounded up to 32: columns of the y rows (zero beyond n_in), rows of the transposed W1
  int out_pad;   // n_out rounded up to 8: columns of the dL/dout rows
  int y_stride, g_stride, w1_stride, w3t_stride;
  // offsets in halves from the start of LDS
  int o_w1, o_w2, o_w2t, o_w1t, o_w3t, o_waves, wave_halves;
  __host__ __device__ static MlpBwdShape make(int n_in, int n_out) {
    MlpBwdShape s;
    s.n_in = n_in;
    s.n_out = n_out;
    s.kin_pad = (n_in + 31) / 32 * 32;
    s.out_pad = (n_out + 7) / 8 * 8;
    s.y_stride = s.kin_pad + kPad;
    s.g_stride = 32 + kPad;  // a full block of 32 columns (the weight-gradient product reads them all), zero beyond n_out
    s.w1_stride = n_in + kPad;
    s.w3t_stride = s.out_pad + kPad;
    s.o_w1 = 0;
    s.o_w2 = s.o_w1 + kHid * s.w1_stride;
    s.o_w2t = s.o_w2 + kHid * kHidStride;
    s.o_w1t = s.o_w2t + kHid * kHidStride;
    s.o_w3t = s.o_w1t + s.kin_pad * kHidStride;
    s.o_waves = s.o_w3t + kHid * s.w3t_stride;
    s.wave_halves = kPts * (s.y_stride + 2 * kHidStride + s.g_stride);
    s.o_waves = (s.o_waves + 7) / 8 * 8;  // 16-byte alignment of the point rows
    return s;
  }
  __host__ __device__ size_t lds_bytes(int waves) const {
    const size_t work = (size_t)(o_waves + waves * wave_halves) * 2;
    const size_t red = (size_t)o_waves * 2 + (size_t)(kHid * kin_pad + kHid * kHid + 32 * kHid) * 4;  // the final sums
    return work > red ? work : red;
  }
};

// KB: 32-column blocks of y (1 for up to 32 encoded features, else 2)
template <int KB>
__global__ __launch_bounds__(512) void mlp_bwd_kernel(const uint32_t B, const MlpBwdShape sh,
                                                      const _Float16* __restrict__ y, const _Float16* __restrict__ W1,
                                                      const _Float16* __restrict__ W2, const _Float16* __restrict__ W3,
                                                      const float* __restrict__ dout, _Float16* __restrict__ dy,
                                                      float* __restrict__ dW1, float* __restrict__ dW2,
                                                      float* __restrict__ dW3) {
  extern __shared__ _Float16 lds[];
  const int n_in = sh.n_in, n_out = sh.n_out;
  const int threads = (int)blockDim.x, waves = threads / 64, wave = (int)threadIdx.x / 64, lane = (int)threadIdx.x & 63;
  _Float16* w1 = lds + sh.o_w1;    // [64][n_in]        W1[n][k]
  _Float16* w2 = lds + sh.o_w2;    // [64][64]          W2[m][n]
  _Float16* w2t = lds + sh.o_w2t;  // [64][64]          W2[m][n] at [n][m]
  _Float16* w1t = lds + sh.o_w1t;  // [kin_pad][64]     W1[n][k] at [k][n], zero rows beyond n_in
  _Float16* w3t = lds + sh.o_w3t;  // [64][out_pad]     W3[o][n] at [n][o], zero columns beyond n_out
  for (int i = threadIdx.x; i < kHid * n_in; i += threads) {
    const int n = i / n_in, k = i % n_in;
    const _Float16 v = W1[i];
    w1[n * sh.w1_stride + k] = v;
    w1t[k * kHidStride + n] = v;
  }
  for (int i = threadIdx.x; i < (sh.kin_pad - n_in) * kHid; i += threads)
    w1t[(n_in + i / kHid) * kHidStride + i % kHid] = (_Float16)0.0f;
  for (int i = threadIdx.x; i < kHid * kHid; i += threads) {
    const int m = i / kHid, n = i % kHid;
    const _Float16 v = W2[i];
    w2[m * kHidStride + n] = v;
    w2t[n * kHidStride + m] = v;
  }
  for (int i = threadIdx.x; i < kHid * sh.out_pad; i += threads) {
    const int n = i / sh.out_pad, o = i % sh.out_pad;
    w3t[n * sh.w3t_stride + o] = o < n_out ? W3[o * kHid + n] : (_Float16)0.0f;
  }
  _Float16* mine = lds + sh.o_waves + wave * sh.wave_halves;
  _Float16* Y = mine;                         // [32][kin_pad]  encoded features, zero beyond n_in
  _Float16* H1 = Y + kPts * sh.y_stride;      // [32][64]       h1, later dL/d(pre-activation 1)
  _Float16* H2 = H1 + kPts * kHidStride;      // [32][64]       h2, later dL/d(pre-activation 2)
  _Float16* G3 = H2 + kPts * kHidStride;      // [32][32]       dL/dout, zero beyond n_out
  for (int i = lane; i < kPts * sh.y_stride; i += 64) Y[i] = (_Float16)0.0f;  // (the padding columns stay zero)
  for (int i = lane; i < kPts * sh.g_stride; i += 64) G3[i] = (_Float16)0.0f;
  __syncthreads();

  float16v aW2[4], aW1[2 * KB], aW3[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) aW2[i] = zero16();
#pragma unroll
  for (int i = 0; i < 2 * KB; ++i) aW1[i] = zero16();
#pragma unroll
  for (int i = 0; i < 2; ++i) aW3[i] = zero16();

  const uint32_t n_blocks = (B + kPts - 1) / kPts;
  const int pieces = n_in / 8;  // 16-byte pieces of a row of y
  for (uint32_t blk = blockIdx.x * waves + wave; blk < n_blocks; blk += gridDim.x * waves) {
    const uint64_t p0 = (uint64_t)blk * kPts;
    // y rows and dL/dout rows of the block into LDS (points beyond the batch: zeros, which add nothing)
    for (int i = lane; i < kPts * pieces; i += 64) {
      const int p = i / pieces, q = i % pieces;
      uint4 v = {0u, 0u, 0u, 0u};
      if (p0 + p < B) v = *reinterpret_cast<const uint4*>(y + (p0 + p) * n_in + 8 * q);
      *reinterpret_cast<uint2*>(Y + p * sh.y_stride + 8 * q) = uint2{v.x, v.y};  // rows are 8-byte aligned
      *reinterpret_cast<uint2*>(Y + p * sh.y_stride + 8 * q + 4) = uint2{v.z, v.w};
    }
    for (int i = lane; i < kPts * n_out; i += 64) {
      const int p = i / n_out, o = i % n_out;
      G3[p * sh.g_stride + o] = p0 + p < B ? (_Float16)dout[(p0 + p) * n_out + o] : (_Float16)0.0f;
    }
    // forward: h1 = relu(W1 y), h2 = relu(W2 h1)
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
      store_relu(H1, kHidStride, 32 * nb, mm_rows(w1 + 32 * nb * sh.w1_stride, sh.w1_stride, Y, sh.y_stride, n_in / 8, zero16()));
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
      store_relu(H2, kHidStride, 32 * nb, mm_rows(w2 + 32 * nb * kHidStride, kHidStride, H1, kHidStride, kHid / 8, zero16()));
    // output layer: dW3[o][n] += sum_p dout[p][o] h2[p][n];  dL/dh2 = W3^T dout, through the ReLU, in place of h2
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) aW3[nb] = mm_cols(G3, sh.g_stride, 0, H2, kHidStride, 32 * nb, aW3[nb]);
    {
      float16v d[2];
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
        d[nb] = mm_rows(w3t + 32 * nb * sh.w3t_stride, sh.w3t_stride, G3, sh.g_stride, sh.out_pad / 8, zero16());
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) store_masked(H2, kHidStride, 32 * nb, d[nb]);
    }
    // second layer: dW2[m][n] += sum_p g2[p][m] h1[p][n];  dL/dh1 = W2^T g2, through the ReLU, in place of h1
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
        aW2[2 * mb + nb] = mm_cols(H2, kHidStride, 32 * mb, H1, kHidStride, 32 * nb, aW2[2 * mb + nb]);
    {
      float16v d[2];
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
        d[nb] = mm_rows(w2t + 32 * nb * kHidStride, kHidStride, H2, kHidStride, kHid / 8, zero16());
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) store_masked(H1, kHidStride, 32 * nb, d[nb]);
    }
    // first layer: dW1[n][k] += sum_p g1[p][n] y[p][k];  dL/dy = W1^T g1
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
        aW1[KB * nb + kb] = mm_cols(H1, kHidStride, 32 * nb, Y, sh.y_stride, 32 * kb, aW1[KB * nb + kb]);
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
      const float16v d = mm_rows(w1t + 32 * kb * kHidStride, kHidStride, H1, kHidStride, kHid / 8, zero16());
      const uint64_t p = p0 + (lane & 31);
      if (p < B) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int k = 32 * kb + 8 * q + 4 * (lane >> 5);
          if (k < n_in) {  // n_in is a multiple of 8: four at once
            half4 h;
#pragma unroll
            for (int t = 0; t < 4; ++t) h[t] = (_Float16)d[4 * q + t];
            *reinterpret_cast<half4*>(dy + p * n_in + k) = h;
          }
        }
      }
    }
  }

  // the weight gradients of the workgroup: one wave after the other adds its sums into LDS, then
  // one atomic add per scalar
  __syncthreads();  // every wave is done with its point rows
  float* red = reinterpret_cast<float*>(lds + sh.o_waves);
  float* r1 = red;                        // [64][kin_pad]
  float* r2 = r1 + kHid * sh.kin_pad;     // [64][64]
  float* r3 = r2 + kHid * kHid;           // [32][64]
  const int n_red = kHid * sh.kin_pad + kHid * kHid + 32 * kHid;
  for (int i = threadIdx.x; i < n_red; i += threads) red[i] = 0.0f;
  __syncthreads();
  const int col = lane & 31, row4 = 4 * (lane >> 5);
  for (int w = 0; w < waves; ++w) {
    if (wave == w) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = 8 * (r / 4) + row4 + r % 4;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
#pragma unroll
          for (int nb = 0; nb < 2; ++nb) r2[(32 * mb + row) * kHid + 32 * nb + col] += aW2[2 * mb + nb][r];
#pragma unroll
          for (int kb = 0; kb < KB; ++kb) r1[(32 * mb + row) * sh.kin_pad + 32 * kb + col] += aW1[KB * mb + kb][r];
        }
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) r3[row * kHid + 32 * nb + col] += aW3[nb][r];
      }
    }
    __syncthreads();
  }
  for (int i = threadIdx.x; i < kHid * n_in; i += threads) {
    const float v = r1[(i / n_in) * sh.kin_pad + i % n_in];
    if (v != 0.0f) __hip_atomic_fetch_add(dW1 + i, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  for (int i = threadIdx.x; i < kHid * kHid; i += threads)
    if (r2[i] != 0.0f) __hip_atomic_fetch_add(dW2 + i, r2[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  for (int i = threadIdx.x; i < n_out * kHid; i += threads)
    if (r3[i] != 0.0f) __hip_atomic_fetch_add(dW3 + i, r3[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace hg

extern "C" hg_status hashgrid_mlp_bwd(uint32_t B, uint32_t n_in, uint32_t n_out, const void* y, const void* W1,
                                      const void* W2, const void* W3, const float* dLdout, void* dLdy, float* dW1,
                                      float* dW2, float* dW3, void* stream) {
  if (B == 0) return HG_OK;
  if (B > HG_MAX_BATCH) return HG_ERR_UNSUPPORTED;
  if (!y || !W1 || !W2 || !W3 || !dLdout || !dLdy || !dW1 || !dW2 || !dW3 || n_out == 0 || n_in == 0)
    return HG_ERR_INVALID_ARG;
  if (n_in % 8 != 0 || n_in > 64 || n_out > 32) return HG_ERR_UNSUPPORTED;
  auto bad = [](const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; };
  if (bad(y, 16) || bad(dLdy, 8) || bad(W1, 2) || bad(W2, 2) || bad(W3, 2) || bad(dLdout, 4) || bad(dW1, 4) ||
      bad(dW2, 4) || bad(dW3, 4))
    return HG_ERR_INVALID_ARG;
  const hg::MlpBwdShape sh = hg::MlpBwdShape::make((int)n_in, (int)n_out);
  constexpr size_t kLdsLimit = 160 * 1024;
  int waves = 8;
  while (waves > 1 && sh.lds_bytes(waves) > kLdsLimit) waves /= 2;
  if (sh.lds_bytes(waves) > kLdsLimit) return HG_ERR_UNSUPPORTED;
  static const hipError_t lds_ok = [] {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(hg::mlp_bwd_kernel<1>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit);
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(hg::mlp_bwd_kernel<2>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit);
    return e;
  }();
  if (lds_ok != hipSuccess) return HG_ERR_DEVICE;
  static const uint32_t cus = [] {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
      n = 256;
    return (uint32_t)n;
  }();
  const uint32_t n_blocks = (B + hg::kPts - 1) / hg::kPts;
  const uint32_t want = (n_blocks + waves - 1) / waves;
  const dim3 grid(want < cus ? want : cus), block(64 * waves);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (sh.kin_pad == 32)
    hipLaunchKernelGGL((hg::mlp_bwd_kernel<1>), grid, block, sh.lds_bytes(waves), s, B, sh, static_cast<const _Float16*>(y),
                       static_cast<const _Float16*>(W1), static_cast<const _Float16*>(W2),
                       static_cast<const _Float16*>(W3), dLdout, static_cast<_Float16*>(dLdy), dW1, dW2, dW3);
  else
    hipLaunchKernelGGL((hg::mlp_bwd_kernel<2>), grid, block, sh.lds_bytes(waves), s, B, sh, static_cast<const _Float16*>(y),
                       static_cast<const _Float16*>(W1), static_cast<const _Float16*>(W2),
                       static_cast<const _Float16*>(W3), dLdout, static_cast<_Float16*>(dLdy), dW1, dW2, dW3);
  return hipGetLastError() == hipSuccess ? HG_OK : HG_ERR_DEVICE;
}
