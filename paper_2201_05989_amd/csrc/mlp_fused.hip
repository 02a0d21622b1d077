// The encoding followed by the small network of the paper (Section 4, "Architecture": two hidden
// layers of 64 neurons, ReLU, linear output layer), in one kernel: the encoded features go from
// the gathers into LDS and through three matrix products on the matrix cores without ever
// reaching memory.  The network is tiny next to the gathers (7168 multiply-adds per point against
// 128 random table reads), so the kernel keeps the shape of the forward kernel - one thread per
// point, 1024-thread workgroups, one barrier per level so that the workgroups walk the level
// slices together - and appends the network per wave: each wave owns the 64 rows of activations
// of its own points.
//
// Matrix products: D[neuron][point] = sum_k W[neuron][k] * act[point][k] with
// v_mfma_f32_32x32x8_f16 (fp16 operands, fp32 accumulation).  Per lane l of a wave:
//   A operand (32 neurons x 8 inputs): neuron l % 32, inputs 4 * (l / 32) .. + 3;
//   B operand (8 inputs x 32 points):  point l % 32, inputs 4 * (l / 32) .. + 3;
//   D (32 neurons x 32 points), 16 values: point l % 32, neurons 8 * (r / 4) + 4 * (l / 32) + r % 4.
// Both operands are therefore 8-byte reads of four consecutive inputs of one row, and a lane's
// results are four runs of four consecutive neurons of one point: activations are kept in LDS as
// [point][neuron] rows, weights as [neuron][input] rows, each row padded by four halves so that
// the 32 rows a read touches fall into different banks.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hashgrid.h"
#include "hashgrid_common.hpp"
#include "hashgrid_internal.hpp"

namespace hg {

constexpr int kMlpBlock = 1024;   // threads = points of a workgroup, at most (fewer for small batches)
constexpr int kHidden = 64;       // neurons of a hidden layer
constexpr int kRowPad = 4;        // halves of padding per LDS row
constexpr int kActStride = kHidden + kRowPad;
constexpr int kMaxOut = 32;       // output neurons (one 32-row block of the matrix instruction)

using half4 = _Float16 __attribute__((ext_vector_type(4)));
using float16v = float __attribute__((ext_vector_type(16)));

// One 32 x 32 block of W[32 rows from w_row0][K] * act[32 points from p_row0][K]^T.
template <int K>
__device__ __forceinline__ float16v block_product(const _Float16* __restrict__ w, int w_stride, int w_row0,
                                                  const _Float16* __restrict__ act, int p_row0) {
  const int lane = threadIdx.x & 63, r = lane & 31, k0 = 4 * (lane >> 5);
  const _Float16* wa = w + (w_row0 + r) * w_stride + k0;
  const _Float16* pb = act + (p_row0 + r) * kActStride + k0;
  float16v acc;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.0f;
#pragma unroll
  for (int ks = 0; ks < K / 8; ++ks) {
    const half4 a = *reinterpret_cast<const half4*>(wa + ks * 8);
    const half4 b = *reinterpret_cast<const half4*>(pb + ks * 8);
    acc = __builtin_amdgcn_mfma_f32_32x32x8f16(a, b, acc, 0, 0, 0);
  }
  return acc;
}

// relu, round to half, store a lane's 16 results of one block: point p_row0 + lane % 32, neurons
// n_row0 + 8 q + 4 (lane / 32) + t
__device__ __forceinline__ void store_hidden(_Float16* __restrict__ act, int p_row0, int n_row0, const float16v& acc) {
  const int lane = threadIdx.x & 63;
  _Float16* row = act + (p_row0 + (lane & 31)) * kActStride + n_row0 + 4 * (lane >> 5);
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    half4 h;
#pragma unroll
    for (int t = 0; t < 4; ++t) h[t] = (_Float16)fmaxf(acc[4 * q + t], 0.0f);
    *reinterpret_cast<half4*>(row + 8 * q) = h;
  }
}

// The network on the 64 points of the calling wave, whose rows of inputs (n_in halves each) are in
// `act`; weights in LDS as laid out by load_weights.  A layer's four blocks are computed before its
// results overwrite the activations they were computed from.  point0: global index of the
// workgroup's first point.
__device__ __forceinline__ void network_of_wave(_Float16* __restrict__ act, const _Float16* __restrict__ w1,
                                                const int w1_stride, const _Float16* __restrict__ w2,
                                                const _Float16* __restrict__ w3, const int n_in, const uint32_t n_out,
                                                const uint32_t B, const uint64_t point0, float* __restrict__ out) {
  const int p0 = (int)(threadIdx.x & ~63u);
  float16v h[4];
#pragma unroll
  for (int blk = 0; blk < 4; ++blk) {
    const int pr = p0 + 32 * (blk & 1), nr = 32 * (blk >> 1);
    h[blk] = n_in == 64   ? block_product<64>(w1, w1_stride, nr, act, pr)
             : n_in == 32 ? block_product<32>(w1, w1_stride, nr, act, pr)
             : n_in == 16 ? block_product<16>(w1, w1_stride, nr, act, pr)
             : n_in == 8  ? block_product<8>(w1, w1_stride, nr, act, pr)
             : n_in == 24 ? block_product<24>(w1, w1_stride, nr, act, pr)
             : n_in == 40 ? block_product<40>(w1, w1_stride, nr, act, pr)
             : n_in == 48 ? block_product<48>(w1, w1_stride, nr, act, pr)
                          : block_product<56>(w1, w1_stride, nr, act, pr);
  }
#pragma unroll
  for (int blk = 0; blk < 4; ++blk) store_hidden(act, p0 + 32 * (blk & 1), 32 * (blk >> 1), h[blk]);
#pragma unroll
  for (int blk = 0; blk < 4; ++blk)
    h[blk] = block_product<kHidden>(w2, kActStride, 32 * (blk >> 1), act, p0 + 32 * (blk & 1));
#pragma unroll
  for (int blk = 0; blk < 4; ++blk) store_hidden(act, p0 + 32 * (blk & 1), 32 * (blk >> 1), h[blk]);
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    const float16v o = block_product<kHidden>(w3, kActStride, 0, act, p0 + 32 * half);
    const uint64_t point = point0 + p0 + 32 * half + (lane & 31);
    if (point < B) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const uint32_t neuron = 8 * (r / 4) + 4 * (lane >> 5) + (r % 4);
        if (neuron < n_out) out[point * n_out + neuron] = o[r];
      }
    }
  }
}

// weights -> LDS in 8-byte pieces (rows are multiples of four halves, host-checked alignment): w1
// [kHidden][n_in + pad], w2 [kHidden][kActStride], w3 [kMaxOut][kActStride] with rows from n_out on zero
__device__ __forceinline__ void load_weights(_Float16* __restrict__ w1, _Float16* __restrict__ w2,
                                             _Float16* __restrict__ w3, const _Float16* __restrict__ W1,
                                             const _Float16* __restrict__ W2, const _Float16* __restrict__ W3,
                                             const int n_in, const uint32_t n_out) {
  const int block = (int)blockDim.x, w1_stride = n_in + kRowPad;
  const int q1 = n_in / 4;  // pieces per row of W1
  for (int i = threadIdx.x; i < kHidden * q1; i += block)
    *reinterpret_cast<half4*>(w1 + (i / q1) * w1_stride + 4 * (i % q1)) = reinterpret_cast<const half4*>(W1)[i];
  constexpr int q2 = kHidden / 4;
  for (int i = threadIdx.x; i < kHidden * q2; i += block)
    *reinterpret_cast<half4*>(w2 + (i / q2) * kActStride + 4 * (i % q2)) = reinterpret_cast<const half4*>(W2)[i];
  for (int i = threadIdx.x; i < kMaxOut * q2; i += block) {
    half4 v = {(_Float16)0.0f, (_Float16)0.0f, (_Float16)0.0f, (_Float16)0.0f};
    if ((uint32_t)(i / q2) < n_out) v = reinterpret_cast<const half4*>(W3)[i];
    *reinterpret_cast<half4*>(w3 + (i / q2) * kActStride + 4 * (i % q2)) = v;
  }
}

// The network alone, on features that are in memory (hashgrid_mlp_fwd): every thread brings the row of
// its point into LDS, then each wave runs the network on its 64 points.
constexpr int kMlpOnlyBlock = 256;
__global__ __launch_bounds__(kMlpOnlyBlock) void mlp_fwd_from_features(const uint32_t B, const int n_in,
                                                                       const _Float16* __restrict__ y,
                                                                       const _Float16* __restrict__ W1,
                                                                       const _Float16* __restrict__ W2,
                                                                       const _Float16* __restrict__ W3,
                                                                       const uint32_t n_out, float* __restrict__ out) {
  extern __shared__ _Float16 lds[];
  const int w1_stride = n_in + kRowPad;
  _Float16* act = lds;                                // [kMlpOnlyBlock][kActStride]
  _Float16* w1 = act + kMlpOnlyBlock * kActStride;    // as in encode_mlp_fwd
  _Float16* w2 = w1 + kHidden * w1_stride;
  _Float16* w3 = w2 + kHidden * kActStride;
  load_weights(w1, w2, w3, W1, W2, W3, n_in, n_out);
  const uint64_t point0 = (uint64_t)blockIdx.x * kMlpOnlyBlock;
  const uint64_t b0 = point0 + threadIdx.x;
  const uint64_t b = b0 < B ? b0 : B - 1;  // idle lanes of the last workgroup shadow the last point
  _Float16* my_row = act + threadIdx.x * kActStride;
  for (int k = 0; k < n_in; k += 4)  // rows of y are 16-byte aligned, rows in LDS 8-byte
    *reinterpret_cast<half4*>(my_row + k) = *reinterpret_cast<const half4*>(y + b * n_in + k);
  __syncthreads();
  network_of_wave(act, w1, w1_stride, w2, w3, n_in, n_out, B, point0, out);
}

template <int D, int F>
__global__ __launch_bounds__(kMlpBlock) void encode_mlp_fwd(const LevelTable lv, const bool smooth, const uint32_t B,
                                                            const float* __restrict__ x,
                                                            const _Float16* __restrict__ theta,
                                                            const _Float16* __restrict__ W1,
                                                            const _Float16* __restrict__ W2,
                                                            const _Float16* __restrict__ W3, const uint32_t n_out,
                                                            float* __restrict__ out, _Float16* __restrict__ y_out) {
  extern __shared__ _Float16 lds[];
  const int n_in = (int)lv.L * F;  // a multiple of 8, at most 64 (checked on the host)
  const int w1_stride = n_in + kRowPad;
  const int block = (int)blockDim.x;
  _Float16* act = lds;                                // [block][kActStride]
  _Float16* w1 = act + block * kActStride;            // [kHidden][n_in + pad]
  _Float16* w2 = w1 + kHidden * w1_stride;            // [kHidden][kActStride]
  _Float16* w3 = w2 + kHidden * kActStride;           // [kMaxOut][kActStride], rows from n_out on are zero

  load_weights(w1, w2, w3, W1, W2, W3, n_in, n_out);

  // the encoding, as in the forward kernel: one thread per point, level by level
  const uint32_t b0 = blockIdx.x * block + threadIdx.x;
  const uint32_t b = b0 < B ? b0 : B - 1;  // idle lanes of the last workgroup shadow the last point
  float xp[D];
#pragma unroll
  for (int i = 0; i < D; ++i) xp[i] = x[(uint64_t)b * D + i];
  _Float16* my_row = act + threadIdx.x * kActStride;
  // two levels in flight, as in the forward kernel: the gathers of level l + 1 are issued before level l
  // is blended (two register sets that alternate)
  Vec<_Float16, F> e[2][1 << D];
  float wr[2][1 << (D - 1)], w0[2], u0[2];
  auto gather_level = [&](const uint32_t l, const int set) {
    uint32_t idx[1 << D];
    level_corners<D, true>(lv, l, smooth, xp, idx, wr[set], w0[set], u0[set]);
    const Vec<_Float16, F>* tab = reinterpret_cast<const Vec<_Float16, F>*>(theta) + lv.offset[l];
#pragma unroll
    for (uint32_t m = 0; m < (1u << D); ++m) e[set][m] = tab[idx[m]];
  };
  auto blend_level = [&](const uint32_t l, const int set) {
    float acc[F];
#pragma unroll
    for (int f = 0; f < F; ++f) acc[f] = 0.0f;
#pragma unroll
    for (uint32_t m = 0; m < (1u << D); ++m) {
      const float wt = wr[set][m >> 1] * ((m & 1u) ? w0[set] : u0[set]);
#pragma unroll
      for (int f = 0; f < F; ++f) acc[f] = fmaf(wt, (float)e[set][m].v[f], acc[f]);
    }
#pragma unroll
    for (int f = 0; f < F; ++f) my_row[l * F + f] = (_Float16)acc[f];  // rows are 8-byte, not 16-byte, aligned
    asm volatile("" ::: "memory");  // keep the gathers of one level together
    __syncthreads();                // (also: the weights are in place before the first product)
  };
  gather_level(0, 0);
  for (uint32_t l = 0; l < lv.L; l += 2) {
    if (l + 1 < lv.L) gather_level(l + 1, 1);
    blend_level(l, 0);
    if (l + 1 < lv.L) {  // uniform
      if (l + 2 < lv.L) gather_level(l + 2, 0);
      blend_level(l + 1, 1);
    }
  }

  // training: the encoded features, as the network sees them (rounded to half), are kept for the
  // backward pass of the network; each thread copies its own row
  if (y_out != nullptr && b0 < B) {
    for (int k = 0; k < n_in; k += 4)
      *reinterpret_cast<half4*>(y_out + (uint64_t)b0 * n_in + k) = *reinterpret_cast<const half4*>(my_row + k);
  }

  network_of_wave(act, w1, w1_stride, w2, w3, n_in, n_out, B, (uint64_t)blockIdx.x * block, out);
}

template <int D, int F>
static hg_status launch_mlp(const hashgrid* h, uint32_t B, const float* x, const void* params, const void* W1,
                            const void* W2, const void* W3, uint32_t n_out, float* out, void* y_out, hipStream_t s) {
  const int n_in = (int)h->lv.L * F;
  const uint32_t block = point_major_block(B);
  const size_t lds = ((size_t)block * kActStride + (size_t)kHidden * (n_in + kRowPad) +
                      (size_t)(kHidden + kMaxOut) * kActStride) * sizeof(_Float16);
  static const hipError_t lds_ok = hipFuncSetAttribute(reinterpret_cast<const void*>(encode_mlp_fwd<D, F>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  if (lds_ok != hipSuccess) return HG_ERR_DEVICE;
  hipLaunchKernelGGL((encode_mlp_fwd<D, F>), dim3((B + block - 1) / block), dim3(block), lds, s, h->lv,
                     h->cfg.interp == HG_INTERP_SMOOTHSTEP, B, x, static_cast<const _Float16*>(params),
                     static_cast<const _Float16*>(W1), static_cast<const _Float16*>(W2),
                     static_cast<const _Float16*>(W3), n_out, out, static_cast<_Float16*>(y_out));
  return hipGetLastError() == hipSuccess ? HG_OK : HG_ERR_DEVICE;
}

}  // namespace hg

static hg_status encode_mlp_fwd_any(const hashgrid_t* hg, uint32_t B, const float* x, const void* params, const void* W1,
                                    const void* W2, const void* W3, uint32_t n_out, float* out, void* y_out,
                                    void* stream) {
  if (!hg) return HG_ERR_INVALID_ARG;
  if (B == 0) return HG_OK;
  if (B > HG_MAX_BATCH) return HG_ERR_UNSUPPORTED;
  if (!x || !params || !W1 || !W2 || !W3 || !out || n_out == 0) return HG_ERR_INVALID_ARG;
  const hashgrid_config& c = hg->cfg;
  const uint32_t n_in = c.L * c.F;
  if (c.param_dtype != HG_F16 || !hg->lv.T_is_pow2 || c.d < 2 || n_in % 8 != 0 || n_in > (uint32_t)hg::kHidden ||
      n_out > (uint32_t)hg::kMaxOut)
    return HG_ERR_UNSUPPORTED;
  auto bad = [](const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; };
  if (bad(x, 4) || bad(params, c.F * 2) || bad(W1, 8) || bad(W2, 8) || bad(W3, 8) || bad(out, 4) || bad(y_out, 16))
    return HG_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
#define HG_MLP(D, F) hg::launch_mlp<D, F>(hg, B, x, params, W1, W2, W3, n_out, out, y_out, s)
  switch (c.d * 16 + c.F) {
    case 2 * 16 + 1: return HG_MLP(2, 1);
    case 2 * 16 + 2: return HG_MLP(2, 2);
    case 2 * 16 + 4: return HG_MLP(2, 4);
    case 2 * 16 + 8: return HG_MLP(2, 8);
    case 3 * 16 + 1: return HG_MLP(3, 1);
    case 3 * 16 + 2: return HG_MLP(3, 2);
    case 3 * 16 + 4: return HG_MLP(3, 4);
    case 3 * 16 + 8: return HG_MLP(3, 8);
    default: return HG_ERR_UNSUPPORTED;
  }
#undef HG_MLP
}

extern "C" hg_status hashgrid_encode_mlp_fwd(const hashgrid_t* hg, uint32_t B, const float* x, const void* params,
                                             const void* W1, const void* W2, const void* W3, uint32_t n_out,
                                             float* out, void* stream) {
  return encode_mlp_fwd_any(hg, B, x, params, W1, W2, W3, n_out, out, nullptr, stream);
}

extern "C" hg_status hashgrid_encode_mlp_fwd_train(const hashgrid_t* hg, uint32_t B, const float* x, const void* params,
                                                   const void* W1, const void* W2, const void* W3, uint32_t n_out,
                                                   float* out, void* y, void* stream) {
  if (B != 0 && !y) return HG_ERR_INVALID_ARG;
  return encode_mlp_fwd_any(hg, B, x, params, W1, W2, W3, n_out, out, y, stream);
}

extern "C" hg_status hashgrid_mlp_fwd(uint32_t B, uint32_t n_in, uint32_t n_out, const void* y, const void* W1,
                                      const void* W2, const void* W3, float* out, void* stream) {
  if (B == 0) return HG_OK;
  if (B > HG_MAX_BATCH) return HG_ERR_UNSUPPORTED;
  if (!y || !W1 || !W2 || !W3 || !out || n_in == 0 || n_out == 0) return HG_ERR_INVALID_ARG;
  if (n_in % 8 != 0 || n_in > (uint32_t)hg::kHidden || n_out > (uint32_t)hg::kMaxOut) return HG_ERR_UNSUPPORTED;
  auto bad = [](const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; };
  if (bad(y, 16) || bad(W1, 8) || bad(W2, 8) || bad(W3, 8) || bad(out, 4)) return HG_ERR_INVALID_ARG;
  const size_t lds = ((size_t)hg::kMlpOnlyBlock * hg::kActStride + (size_t)hg::kHidden * (n_in + hg::kRowPad) +
                      (size_t)(hg::kHidden + hg::kMaxOut) * hg::kActStride) * sizeof(_Float16);  // 53 KB at most
  hipLaunchKernelGGL(hg::mlp_fwd_from_features, dim3((B + hg::kMlpOnlyBlock - 1) / hg::kMlpOnlyBlock),
                     dim3(hg::kMlpOnlyBlock), lds, static_cast<hipStream_t>(stream), B, (int)n_in,
                     static_cast<const _Float16*>(y), static_cast<const _Float16*>(W1),
                     static_cast<const _Float16*>(W2), static_cast<const _Float16*>(W3), n_out, out);
  return hipGetLastError() == hipSuccess ? HG_OK : HG_ERR_DEVICE;
}
