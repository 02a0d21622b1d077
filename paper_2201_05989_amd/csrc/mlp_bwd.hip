// Backward pass of the paper's small network (Section 4, "Architecture": two hidden layers of 64
// neurons, ReLU, linear output layer) on the matrix cores: from the encoded features y and the
// upstream gradient dL/dout to dL/dy (which hashgrid_encode_bwd[_ws] then takes to the tables) and
// the gradients of the three weight matrices, in one kernel.  Hidden activations are recomputed
// from y (they never existed in memory: the forward kernel keeps them in LDS), so nothing but y
// has to be kept from the forward pass.
//
// Work unit: one wave and 32 points.  Activations and gradients of a block never leave the wave's
// registers; LDS holds the weights only.  Every product is v_mfma_f32_32x32x8_f16 (fp16 operands,
// fp32 accumulation), D[i][j] = sum_k A[i][k] B[k][j] with, per lane l (c = l % 32, h = l / 32):
//   A: row i = c, k = 4 h .. 4 h + 3;   B: column j = c, the same k;
//   D: column j = c, rows i = 8 q + 4 h + t in register 4 q + t (q, t = 0 .. 3).
// A lane's part of D, rounded to half, is therefore already its part of the B (or A) operand of a
// product that contracts over D's rows, eight rows per instruction: register group q is step q.
// Two layouts of a matrix z[point][neuron] of a block follow:
//   "P": lane = point c, registers = neurons 32 T + 8 q + 4 h + t of tile T.  It is the B operand of
//        W z (A = rows of the weights from LDS), whose result is again in layout P: the chain
//        y -> h1 -> h2 and dL/dout -> g2 -> g1 -> dL/dy runs P to P.
//   "N": lane = neuron 32 T + c, registers = points 8 q + 4 h + t.  The same product with the operands
//        exchanged, z as A and the same weight fragment as B, gives the transposed result: layout N.
//        Layout N is what the weight gradients contract over (the points): dW[m][n] = sum_p g[p][m]
//        z[p][n] takes g in layout N as A and z in layout N as B.
// So every layer issues two instructions per weight fragment read from LDS, one for each layout of
// its result, and the weight gradients need no memory operand at all.  y in layout N is y in layout P
// times the identity, exchanged (exact).  Weight-gradient sums stay in registers while the wave
// walks its blocks of points, are then added up across the workgroup's waves in LDS and leave with
// one atomic add per scalar and workgroup.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

#include "hashgrid.h"

namespace hg {

constexpr int kHid = 64;      // neurons of a hidden layer
constexpr int kPad = 4;       // halves of padding per LDS row: the 8-byte reads of 32 lanes a row apart cover all banks
constexpr int kHidStride = kHid + kPad;
constexpr int kPts = 32;      // points of a wave's block
constexpr int kWaves = 4;     // waves of a workgroup: one per SIMD, which leaves a wave all 512 registers

using half4 = _Float16 __attribute__((ext_vector_type(4)));
using float16v = float __attribute__((ext_vector_type(16)));

__device__ __forceinline__ float16v zero16() {
  float16v z;
#pragma unroll
  for (int i = 0; i < 16; ++i) z[i] = 0.0f;
  return z;
}
__device__ __forceinline__ float16v mfma(const half4 a, const half4 b, const float16v c) {
  return __builtin_amdgcn_mfma_f32_32x32x8f16(a, b, c, 0, 0, 0);
}
using short4v = short __attribute__((ext_vector_type(4)));
using float4v = float __attribute__((ext_vector_type(4)));
// register group q of a result, rounded to half (nearest even)
__device__ __forceinline__ half4 to_half(const float16v& acc, const int q) {
  const float4v v = {acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
  return __builtin_convertvector(v, half4);
}
// ReLU on halves: as 16-bit integers the negative halves (and -0) are the negative numbers
__device__ __forceinline__ half4 relu(const half4 v) {
  return __builtin_bit_cast(half4, __builtin_elementwise_max(__builtin_bit_cast(short4v, v), (short4v)0));
}
// g where the activation act (not negative: it went through relu) is positive, else 0: all ones
// where the bits of act are not zero, two packed instructions for two halves (written out: the
// compiler would turn the C expression into a compare and a select per half)
__device__ __forceinline__ half4 where_positive(const half4 g, const half4 act) {
  uint2 a = __builtin_bit_cast(uint2, act);
  const uint2 gb = __builtin_bit_cast(uint2, g);
  // (op_sel_hi: the upper half of the instruction takes the shift count from the constant's lower 16 bits too)
  asm("v_pk_sub_i16 %0, 0, %0\n\tv_pk_ashrrev_i16 %0, 15, %0 op_sel_hi:[0,1]" : "+v"(a.x));
  asm("v_pk_sub_i16 %0, 0, %0\n\tv_pk_ashrrev_i16 %0, 15, %0 op_sel_hi:[0,1]" : "+v"(a.y));
  return __builtin_bit_cast(half4, uint2{gb.x & a.x, gb.y & a.y});
}

struct MlpBwdShape {
  int n_in, n_out;
  int kin_pad;   // n_in rounded up to 32: columns of the staged W1 (zero beyond n_in), rows of its transposed copy
  int out_pad;   // n_out rounded up to 8: columns of the transposed W3
  int w1_stride, w3t_stride;
  // offsets in halves from the start of LDS
  int o_w1, o_w2, o_w2t, o_w1t, o_w3t, o_end;
  __host__ __device__ static MlpBwdShape make(int n_in, int n_out) {
    MlpBwdShape s;
    s.n_in = n_in;
    s.n_out = n_out;
    s.kin_pad = (n_in + 31) / 32 * 32;
    s.out_pad = (n_out + 7) / 8 * 8;
    s.w1_stride = s.kin_pad + kPad;
    s.w3t_stride = s.out_pad + kPad;
    s.o_w1 = 0;
    s.o_w2 = s.o_w1 + kHid * s.w1_stride;
    s.o_w2t = s.o_w2 + kHid * kHidStride;
    s.o_w1t = s.o_w2t + kHid * kHidStride;
    s.o_w3t = s.o_w1t + s.kin_pad * kHidStride;
    s.o_end = (s.o_w3t + kHid * s.w3t_stride + 7) / 8 * 8;
    return s;
  }
  // the weights; afterwards the same memory takes the waves' weight-gradient sums, at most 96 registers of
  // 64 lanes per wave at a time
  __host__ __device__ size_t lds_bytes(int waves) const {
    const size_t weights = (size_t)o_end * 2, sums = (size_t)waves * 96 * 64 * 4;
    return weights > sums ? weights : sums;
  }
};

// KB: 32-column blocks of y (1 for up to 32 encoded features, else 2); OS: groups of eight outputs
template <int KB, int OS>
__global__ __launch_bounds__(64 * kWaves) void mlp_bwd_kernel(const uint32_t B, const MlpBwdShape sh,
                                                      const _Float16* __restrict__ y, const _Float16* __restrict__ W1,
                                                      const _Float16* __restrict__ W2, const _Float16* __restrict__ W3,
                                                      const float* __restrict__ dout, _Float16* __restrict__ dy,
                                                      float* __restrict__ dW1, float* __restrict__ dW2,
                                                      float* __restrict__ dW3) {
  extern __shared__ _Float16 lds[];
  const int n_in = sh.n_in, n_out = sh.n_out;
  const int threads = (int)blockDim.x, waves = threads / 64, wave = (int)threadIdx.x / 64, lane = (int)threadIdx.x & 63;
  _Float16* w1 = lds + sh.o_w1;    // [64][kin_pad]     W1[n][k], zero columns beyond n_in
  _Float16* w2 = lds + sh.o_w2;    // [64][64]          W2[m][n]
  _Float16* w2t = lds + sh.o_w2t;  // [64][64]          W2[m][n] at [n][m]
  _Float16* w1t = lds + sh.o_w1t;  // [kin_pad][64]     W1[n][k] at [k][n], zero rows beyond n_in
  _Float16* w3t = lds + sh.o_w3t;  // [64][out_pad]     W3[o][n] at [n][o], zero columns beyond n_out
  // staging in pieces of four halves where the arrays allow 8-byte loads (every row length here is a multiple of 8 halves)
  const bool wide = ((reinterpret_cast<uintptr_t>(W1) | reinterpret_cast<uintptr_t>(W2) | reinterpret_cast<uintptr_t>(W3)) & 7) == 0;
  auto piece = [&](const _Float16* src, const bool inside) {
    half4 v = {(_Float16)0.0f, (_Float16)0.0f, (_Float16)0.0f, (_Float16)0.0f};
    if (inside) {
      if (wide) {  // uniform
        v = *reinterpret_cast<const half4*>(src);
      } else {
#pragma unroll
        for (int t = 0; t < 4; ++t) v[t] = src[t];
      }
    }
    return v;
  };
  constexpr int kThreads = 64 * kWaves;
#pragma unroll
  for (int j = 0; j < kHid * kHid / 4 / kThreads; ++j) {  // W2: 1024 pieces
    const int i = (int)threadIdx.x + j * kThreads, m = i / (kHid / 4), n = 4 * (i % (kHid / 4));
    const half4 v = piece(W2 + 4 * i, true);
    *reinterpret_cast<half4*>(w2 + m * kHidStride + n) = v;
#pragma unroll
    for (int t = 0; t < 4; ++t) w2t[(n + t) * kHidStride + m] = v[t];
  }
  for (int i = threadIdx.x; i < kHid * sh.kin_pad / 4; i += kThreads) {  // W1, zero columns beyond n_in
    const int n = i / (sh.kin_pad / 4), k = 4 * (i % (sh.kin_pad / 4));
    const half4 v = piece(W1 + n * n_in + k, k < n_in);
    *reinterpret_cast<half4*>(w1 + n * sh.w1_stride + k) = v;
#pragma unroll
    for (int t = 0; t < 4; ++t) w1t[(k + t) * kHidStride + n] = v[t];
  }
  for (int i = threadIdx.x; i < sh.out_pad * (kHid / 4); i += kThreads) {  // W3, zero columns beyond n_out
    const int o = i / (kHid / 4), n = 4 * (i % (kHid / 4));
    const half4 v = piece(W3 + o * kHid + n, o < n_out);
#pragma unroll
    for (int t = 0; t < 4; ++t) w3t[(n + t) * sh.w3t_stride + o] = v[t];
  }
  __syncthreads();

  const int c = lane & 31, h = lane >> 5;
  // this lane's 8-byte fragment of row 32 T + c of a weight array, columns 8 ks + 4 h .. + 3
  auto frag = [&](const _Float16* w, const int stride, const int T, const int ks) {
    return *reinterpret_cast<const half4*>(w + (32 * T + c) * stride + 8 * ks + 4 * h);
  };

  float16v aW2[4], aW1[2 * KB], aW3[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) aW2[i] = zero16();
#pragma unroll
  for (int i = 0; i < 2 * KB; ++i) aW1[i] = zero16();
#pragma unroll
  for (int i = 0; i < 2; ++i) aW3[i] = zero16();

  // the identity's fragments for the exchange of y (step ks: rows 8 ks + 4 h + t, column c)
  half4 one[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)
#pragma unroll
    for (int t = 0; t < 4; ++t) one[ks][t] = (8 * ks + 4 * h + t == c) ? (_Float16)1.0f : (_Float16)0.0f;

  // y and dL/dout of a block in layout P, as they come from memory (lane = point, four encoded features
  // or outputs per step; points beyond the batch and columns beyond n_in / n_out: zeros, which add nothing)
  uint2 y_next[4 * KB];
  float4v d_next[OS];
  // (no branches: a point beyond the batch reads the last point's row, a column beyond the row its
  // last columns, and the value is replaced by zero)
  auto request = [&](const uint64_t p0) {
    const uint64_t p = p0 + c;
    const bool inside = p < B;
    const uint64_t pr = inside ? p : (uint64_t)B - 1;
#pragma unroll
    for (int ks = 0; ks < 4 * KB; ++ks) {
      const int k = 8 * ks + 4 * h;
      const uint2 v = *reinterpret_cast<const uint2*>(y + pr * n_in + (k < n_in ? k : n_in - 4));
      const bool keep = inside && k < n_in;
      y_next[ks] = uint2{keep ? v.x : 0u, keep ? v.y : 0u};
    }
#pragma unroll
    for (int ks = 0; ks < OS; ++ks)
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int o = 8 * ks + 4 * h + t;
        const float v = dout[pr * n_out + (o < n_out ? o : n_out - 1)];
        d_next[ks][t] = (inside && o < n_out) ? v : 0.0f;
      }
  };

  // One block of 32 points.  FULL: all 32 are inside the batch (no bounds checks, one basic block
  // for the scheduler); the last, ragged block takes the checked variant, where points beyond the
  // batch enter as zeros, which add nothing, and are not stored.
  auto block = [&](const uint64_t p0, const uint64_t p0_next, auto full) {
    constexpr bool FULL = decltype(full)::value;
    const uint64_t p = p0 + c;
    const bool mine = FULL || p < B;
    // this block's y and dL/dout (layout P) were requested one block ahead; request the next block's
    half4 yP[4 * KB], g3P[OS];
#pragma unroll
    for (int ks = 0; ks < 4 * KB; ++ks) yP[ks] = __builtin_bit_cast(half4, y_next[ks]);
#pragma unroll
    for (int ks = 0; ks < OS; ++ks)
#pragma unroll
      for (int t = 0; t < 4; ++t) g3P[ks][t] = (_Float16)d_next[ks][t];  // rounded to half
    request(p0_next);
    // dL/dout in layout N (lane = output, registers = points) = (layout P) x identity, exchanged
    half4 g3N[4];
    {
      float16v aN = zero16();
#pragma unroll
      for (int ks = 0; ks < OS; ++ks) aN = mfma(g3P[ks], one[ks], aN);
#pragma unroll
      for (int q = 0; q < 4; ++q) g3N[q] = to_half(aN, q);  // exact: a copy of one half
    }

    // forward: h1 = relu(W1 y), h2 = relu(W2 h1), both in both layouts
    half4 h1P[8], h1N[8], h2P[8], h2N[8];
#pragma unroll
    for (int T = 0; T < 2; ++T) {
      float16v aP = zero16(), aN = zero16();
#pragma unroll
      for (int ks = 0; ks < 4 * KB; ++ks) {
        const half4 w = frag(w1, sh.w1_stride, T, ks);
        aP = mfma(w, yP[ks], aP);
        aN = mfma(yP[ks], w, aN);
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        h1P[4 * T + q] = relu(to_half(aP, q));
        h1N[4 * T + q] = relu(to_half(aN, q));
      }
    }
#pragma unroll
    for (int T = 0; T < 2; ++T) {
      float16v aP = zero16(), aN = zero16();
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const half4 w = frag(w2, kHidStride, T, ks);
        aP = mfma(w, h1P[ks], aP);
        aN = mfma(h1P[ks], w, aN);
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        h2P[4 * T + q] = relu(to_half(aP, q));  // (only its signs are used)
        h2N[4 * T + q] = relu(to_half(aN, q));
      }
    }
    // output layer: dW3[o][n] += sum_p dout[p][o] h2[p][n];  g2 = (W3^T dout) through the ReLU of layer 2
#pragma unroll
    for (int T = 0; T < 2; ++T)
#pragma unroll
      for (int q = 0; q < 4; ++q) aW3[T] = mfma(g3N[q], h2N[4 * T + q], aW3[T]);
    half4 g2P[8], g2N[8];
#pragma unroll
    for (int T = 0; T < 2; ++T) {
      float16v aP = zero16(), aN = zero16();
#pragma unroll
      for (int ks = 0; ks < OS; ++ks) {
        const half4 w = frag(w3t, sh.w3t_stride, T, ks);
        aP = mfma(w, g3P[ks], aP);
        aN = mfma(g3P[ks], w, aN);
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        g2P[4 * T + q] = where_positive(to_half(aP, q), h2P[4 * T + q]);
        g2N[4 * T + q] = where_positive(to_half(aN, q), h2N[4 * T + q]);
      }
    }
    // second layer: dW2[m][n] += sum_p g2[p][m] h1[p][n];  g1 = (W2^T g2) through the ReLU of layer 1
#pragma unroll
    for (int Tm = 0; Tm < 2; ++Tm)
#pragma unroll
      for (int Tn = 0; Tn < 2; ++Tn)
#pragma unroll
        for (int q = 0; q < 4; ++q) aW2[2 * Tm + Tn] = mfma(g2N[4 * Tm + q], h1N[4 * Tn + q], aW2[2 * Tm + Tn]);
    half4 g1P[8], g1N[8];
#pragma unroll
    for (int T = 0; T < 2; ++T) {
      float16v aP = zero16(), aN = zero16();
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const half4 w = frag(w2t, kHidStride, T, ks);
        aP = mfma(w, g2P[ks], aP);
        aN = mfma(g2P[ks], w, aN);
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        g1P[4 * T + q] = where_positive(to_half(aP, q), h1P[4 * T + q]);
        g1N[4 * T + q] = where_positive(to_half(aN, q), h1N[4 * T + q]);
      }
    }
    // first layer: dW1[n][k] += sum_p g1[p][n] y[p][k], with y in layout N = (y in layout P) x identity, exchanged
#pragma unroll
    for (int Tk = 0; Tk < KB; ++Tk) {
      float16v aN = zero16();
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) aN = mfma(yP[4 * Tk + ks], one[ks], aN);
      half4 yN[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) yN[q] = to_half(aN, q);  // exact: a copy of one half
#pragma unroll
      for (int Tn = 0; Tn < 2; ++Tn)
#pragma unroll
        for (int q = 0; q < 4; ++q) aW1[KB * Tn + Tk] = mfma(g1N[4 * Tn + q], yN[q], aW1[KB * Tn + Tk]);
    }
    // dL/dy = W1^T g1, layout P: four features per register group, straight to memory
#pragma unroll
    for (int Tk = 0; Tk < KB; ++Tk) {
      float16v d = zero16();
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) d = mfma(frag(w1t, kHidStride, Tk, ks), g1P[ks], d);
      if (mine) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int k = 32 * Tk + 8 * q + 4 * h;
          if (k < n_in) *reinterpret_cast<half4*>(dy + p * n_in + k) = to_half(d, q);  // n_in is a multiple of 8: four at once
        }
      }
    }
  };

  const uint32_t n_blocks = (B + kPts - 1) / kPts;
  const uint32_t stride = gridDim.x * waves;
  uint32_t blk = blockIdx.x * waves + wave;
  request((uint64_t)blk * kPts);  // (a block beyond the batch: all zeros)
  for (; blk < n_blocks; blk += stride) {
    // (keeps the compiler from holding the weight fragments, which do not change from block to block, in registers)
    asm volatile("" ::: "memory");
    const uint64_t p0 = (uint64_t)blk * kPts, p0_next = ((uint64_t)blk + stride) * kPts;
    if (p0 + kPts <= B) block(p0, p0_next, std::true_type{});
    else block(p0, p0_next, std::false_type{});
  }

  // The weight gradients of the workgroup.  Every wave writes its sums to LDS as they lie in its
  // registers ([wave][register][lane]; the weights are no longer needed), then every thread adds up
  // the waves' values of its share of (register, lane) pairs and sends one atomic add per scalar:
  // the 32 lanes of a half-wave hold 32 consecutive columns of a row.  Two rounds, so that the
  // area stays below 96 KiB: the second layer's 64 registers, then the first and the output layer's.
  float* red = reinterpret_cast<float*>(lds);
  const int row4 = 4 * h;
  auto reduce = [&](auto&& store_all, const int n_regs, auto&& target_of) {
    __syncthreads();  // the area is free: every wave is done with the weights (first round) or the round before
    store_all(red + wave * n_regs * 64 + lane);  // register r to [r * 64]
    __syncthreads();
    for (int r = wave; r < n_regs; r += waves) {
      float v = 0.0f;
      for (int w = 0; w < waves; ++w) v += red[(w * n_regs + r) * 64 + lane];
      float* t = target_of(r);
      if (t != nullptr && v != 0.0f) __hip_atomic_fetch_add(t, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  };
  // register r of accumulator tile r / 16: row 8 ((r % 16) / 4) + 4 h + r % 4, column c of the tile
  auto row_of = [&](const int r) { return 8 * ((r % 16) / 4) + row4 + r % 4; };
  reduce(
      [&](float* mine) {
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
          for (int q = 0; q < 16; ++q) mine[(16 * a + q) * 64] = aW2[a][q];
      },
      64, [&](const int r) { return dW2 + (32 * (r / 32) + row_of(r)) * kHid + 32 * ((r / 16) % 2) + c; });
  reduce(
      [&](float* mine) {
#pragma unroll
        for (int a = 0; a < 2 * KB; ++a)
#pragma unroll
          for (int q = 0; q < 16; ++q) mine[(16 * a + q) * 64] = aW1[a][q];
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
          for (int q = 0; q < 16; ++q) mine[(32 * KB + 16 * a + q) * 64] = aW3[a][q];
      },
      32 * KB + 32,
      [&](const int r) -> float* {
        if (r < 32 * KB) {  // aW1[KB * Tn + Tk]: rows n of tile Tn, columns k of tile Tk
          const int a = r / 16, k = 32 * (a % KB) + c;
          return k < n_in ? dW1 + (32 * (a / KB) + row_of(r)) * n_in + k : nullptr;
        }
        const int a = (r - 32 * KB) / 16, o = row_of(r);  // aW3[Tn]: rows o, columns n of tile Tn
        return o < n_out ? dW3 + o * kHid + 32 * a + c : nullptr;
      });
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
  const int waves = hg::kWaves;
  if (sh.lds_bytes(waves) > kLdsLimit) return HG_ERR_UNSUPPORTED;
  using Kernel = void (*)(uint32_t, hg::MlpBwdShape, const _Float16*, const _Float16*, const _Float16*, const _Float16*,
                          const float*, _Float16*, float*, float*, float*);
  static const Kernel kernels[2][4] = {
      {hg::mlp_bwd_kernel<1, 1>, hg::mlp_bwd_kernel<1, 2>, hg::mlp_bwd_kernel<1, 3>, hg::mlp_bwd_kernel<1, 4>},
      {hg::mlp_bwd_kernel<2, 1>, hg::mlp_bwd_kernel<2, 2>, hg::mlp_bwd_kernel<2, 3>, hg::mlp_bwd_kernel<2, 4>}};
  static const hipError_t lds_ok = [] {
    hipError_t e = hipSuccess;
    for (int i = 0; i < 2 && e == hipSuccess; ++i)
      for (int j = 0; j < 4 && e == hipSuccess; ++j)
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernels[i][j]), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)kLdsLimit);
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
  hipLaunchKernelGGL(kernels[sh.kin_pad / 32 - 1][sh.out_pad / 8 - 1], grid, block, sh.lds_bytes(waves), s, B, sh,
                     static_cast<const _Float16*>(y), static_cast<const _Float16*>(W1), static_cast<const _Float16*>(W2),
                     static_cast<const _Float16*>(W3), dLdout, static_cast<_Float16*>(dLdy), dW1, dW2, dW3);
  return hipGetLastError() == hipSuccess ? HG_OK : HG_ERR_DEVICE;
}
