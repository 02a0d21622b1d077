// Backward pass of the paper's small network (Section 4, "Architecture": two hidden layers of 64
// neurons, ReLU, linear output layer) on the matrix cores: from the encoded features y and the
// upstream gradient dL/dout to dL/dy (which hashgrid_encode_bwd[_ws] then takes to the tables) and
// the gradients of the three weight matrices, in one kernel.  Hidden activations are recomputed
// from y (they never existed in memory: the forward kernel keeps them in LDS), so nothing but y
// has to be kept from the forward pass.
//
// Work unit: one wave and 32 points.  Activations and gradients of a block never leave the wave's
// registers; LDS holds the weights only.  Every product is v_mfma_f32_32x32x16_f16 (fp16 operands,
// fp32 accumulation), D[i][j] = sum_k A[i][k] B[k][j] over 16 values of k, with, per lane l
// (c = l % 32, h = l / 32):
//   A: row i = c, eight values of k in registers;   B: column j = c, eight values of k;
//   D: column j = c, rows i = 8 q + 4 h + t in register 4 q + t (q, t = 0 .. 3).
// Which eight k a lane holds is the instruction's business only in that A and B must agree, so k is
// numbered here the way D comes out: slot s = 0 .. 7 of lane half h in step j stands for
// k = 16 j + 8 (s / 4) + 4 h + s % 4.  Then a lane's part of D, rounded to half, register groups
// 2 j and 2 j + 1, is already its part of the B (or A) operand of step j of a product that contracts
// over D's rows, and the matching fragment of a weight row is two 8-byte pieces 16 bytes apart.
// Two layouts of a matrix z[point][neuron] of a block follow:
//   "P": lane = point c, registers = neurons 32 T + 8 q + 4 h + t of tile T.  It is the B operand of
//        W z (A = rows of the weights from LDS), whose result is again in layout P: the chain
//        y -> h1 -> h2 and dL/dout -> g2 -> g1 -> dL/dy runs P to P.
//   "N": lane = neuron 32 T + c, registers = points 8 q + 4 h + t: what the weight gradients contract
//        over (the points): dW[m][n] = sum_p g[p][m] z[p][n] takes g in layout N as A and z in layout N
//        as B.  Layout N of a tile is its layout P times the identity with the operands exchanged (z as
//        A, the identity's fragment as B): the transposed result, every sum a single term, so exact.
// So a layer costs its products, one rounding of its result, and two more instructions per tile for
// the second layout; the weight gradients need no memory operand at all.  Weight-gradient sums stay
// in registers while the wave walks its blocks of points, are then added up across the workgroup's
// waves in LDS and leave with one atomic add per scalar and workgroup.
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
constexpr int kSub = 2;       // blocks of 32 points a wave has in flight

using half4 = _Float16 __attribute__((ext_vector_type(4)));
using half8 = _Float16 __attribute__((ext_vector_type(8)));
using short8v = short __attribute__((ext_vector_type(8)));
using float8v = float __attribute__((ext_vector_type(8)));
using float16v = float __attribute__((ext_vector_type(16)));

__device__ __forceinline__ float16v zero16() {
  float16v z;
#pragma unroll
  for (int i = 0; i < 16; ++i) z[i] = 0.0f;
  return z;
}
__device__ __forceinline__ float16v mfma(const half8 a, const half8 b, const float16v c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}
// register groups 2 j and 2 j + 1 of a result, rounded to half (nearest even): step j of an operand
__device__ __forceinline__ half8 to_half(const float16v& acc, const int j) {
  float8v v;
#pragma unroll
  for (int s = 0; s < 8; ++s) v[s] = acc[8 * j + s];
  return __builtin_convertvector(v, half8);
}
// ReLU on halves: as 16-bit integers the negative halves (and -0) are the negative numbers
__device__ __forceinline__ half8 relu(const half8 v) {
  return __builtin_bit_cast(half8, __builtin_elementwise_max(__builtin_bit_cast(short8v, v), (short8v)0));
}
// g where the activation act (not negative: it went through relu) is positive, else 0: all ones
// where the bits of act are not zero, two packed instructions for two halves (written out: the
// compiler would turn the C expression into a compare and a select per half)
__device__ __forceinline__ half8 where_positive(const half8 g, const half8 act) {
  uint4 a = __builtin_bit_cast(uint4, act);
  const uint4 gb = __builtin_bit_cast(uint4, g);
  // (op_sel_hi: the upper half of the instruction takes the shift count from the constant's lower 16 bits too)
  asm("v_pk_sub_i16 %0, 0, %0\n\tv_pk_ashrrev_i16 %0, 15, %0 op_sel_hi:[0,1]" : "+v"(a.x));
  asm("v_pk_sub_i16 %0, 0, %0\n\tv_pk_ashrrev_i16 %0, 15, %0 op_sel_hi:[0,1]" : "+v"(a.y));
  asm("v_pk_sub_i16 %0, 0, %0\n\tv_pk_ashrrev_i16 %0, 15, %0 op_sel_hi:[0,1]" : "+v"(a.z));
  asm("v_pk_sub_i16 %0, 0, %0\n\tv_pk_ashrrev_i16 %0, 15, %0 op_sel_hi:[0,1]" : "+v"(a.w));
  return __builtin_bit_cast(half8, uint4{gb.x & a.x, gb.y & a.y, gb.z & a.z, gb.w & a.w});
}

struct MlpBwdShape {
  int n_in, n_out;
  int kin_pad;   // n_in rounded up to 32: columns of the staged W1 (zero beyond n_in), rows of its transposed copy
  int out_pad;   // n_out rounded up to 16: columns of the transposed W3
  int w1_stride, w3t_stride;
  // offsets in halves from the start of LDS
  int o_w1, o_w2, o_w2t, o_w1t, o_w3t, o_end;
  __host__ __device__ static MlpBwdShape make(int n_in, int n_out) {
    MlpBwdShape s;
    s.n_in = n_in;
    s.n_out = n_out;
    s.kin_pad = (n_in + 31) / 32 * 32;
    s.out_pad = (n_out + 15) / 16 * 16;
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

// Where a weight-gradient sum goes.  A workgroup's sums are numbered by (register g, lane) as they lie
// in a wave's accumulators: g = 0 .. 63 the four 32 x 32 tiles of dW2 ([2 Tm + Tn]), then 32 KB
// registers of dW1 ([KB Tn + Tk]: rows n of tile Tn, columns k of tile Tk), then 32 of dW3 ([Tn]: rows
// o, columns n of tile Tn); register r of a tile holds row 8 (r / 4) + 4 (lane / 32) + r % 4 at
// column lane % 32.  nullptr for the padding (k >= n_in, o >= n_out).
__device__ __forceinline__ float* sum_target(const int g, const int lane, const int kb, const int n_in, const int n_out,
                                             float* dW1, float* dW2, float* dW3) {
  const int c = lane & 31, r = g % 16, row = 8 * (r / 4) + 4 * (lane >> 5) + r % 4;
  if (g < 64) return dW2 + (32 * (g / 32) + row) * kHid + 32 * ((g / 16) % 2) + c;
  if (g < 64 + 32 * kb) {
    const int a = (g - 64) / 16, k = 32 * (a % kb) + c;
    return k < n_in ? dW1 + (32 * (a / kb) + row) * n_in + k : nullptr;
  }
  const int a = (g - 64 - 32 * kb) / 16;
  return row < n_out ? dW3 + row * kHid + 32 * a + c : nullptr;
}
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
  const int c = lane & 31, h = lane >> 5;
  constexpr uint32_t kRound = kSub * kPts;  // points of a wave's round
  const uint32_t n_rounds = (B + kRound - 1) / kRound;
  const uint32_t stride = gridDim.x * waves;
  uint32_t rnd = blockIdx.x * waves + wave;
  // y and dL/dout of a block in layout P, as they come from memory (lane = point, two pieces of four
  // encoded features or outputs per step; points beyond the batch and columns beyond n_in / n_out:
  // zeros, which add nothing).  No branches: a point beyond the batch reads the last point's row, a
  // column beyond the row its last columns, and the value is replaced by zero.
  // A wave works on kSub blocks of 32 points at a time: their chains of products do not depend on
  // each other, so the matrix cores run one block's products while the vector unit rounds the other's.
  uint2 y_next[kSub][4 * KB];
  float d_next[kSub][OS][4];
  auto request = [&](const uint64_t p0) {
#pragma unroll
    for (int u = 0; u < kSub; ++u) {
      const uint64_t p = p0 + kPts * u + c;
      const bool inside = p < B;
      const uint64_t pr = inside ? p : (uint64_t)B - 1;
#pragma unroll
      for (int ks = 0; ks < 4 * KB; ++ks) {
        const int k = 8 * ks + 4 * h;
        const uint2 v = *reinterpret_cast<const uint2*>(y + pr * n_in + (k < n_in ? k : n_in - 4));
        const bool keep = inside && k < n_in;
        y_next[u][ks] = uint2{keep ? v.x : 0u, keep ? v.y : 0u};
      }
#pragma unroll
      for (int ks = 0; ks < OS; ++ks)
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int o = 8 * ks + 4 * h + t;
          const float v = dout[pr * n_out + (o < n_out ? o : n_out - 1)];
          d_next[u][ks][t] = (inside && o < n_out) ? v : 0.0f;
        }
    }
  };

  request((uint64_t)rnd * kRound);  // the first round's, under the staging of the weights (beyond the batch: all zeros)

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

  constexpr int OJ = (OS + 1) / 2;  // steps of 16 outputs
  // this lane's fragment of row 32 T + c of a weight array for step j: columns 16 j + 4 h .. + 3 and 16 j + 8 + 4 h .. + 3
  auto frag = [&](const _Float16* w, const int stride, const int T, const int j) {
    const _Float16* at = w + (32 * T + c) * stride + 16 * j + 4 * h;
    const half4 lo = *reinterpret_cast<const half4*>(at), hi = *reinterpret_cast<const half4*>(at + 8);
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  };

  float16v aW2[4], aW1[2 * KB], aW3[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) aW2[i] = zero16();
#pragma unroll
  for (int i = 0; i < 2 * KB; ++i) aW1[i] = zero16();
#pragma unroll
  for (int i = 0; i < 2; ++i) aW3[i] = zero16();

  // the identity's fragments for the exchange of y and dL/dout (step j, slot s: row 16 j + 8 (s / 4) + 4 h + s % 4, column c)
  half8 one[2];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int s8 = 0; s8 < 8; ++s8) one[j][s8] = (16 * j + 8 * (s8 / 4) + 4 * h + s8 % 4 == c) ? (_Float16)1.0f : (_Float16)0.0f;

  // kSub blocks of 32 points from p0 on.  FULL: all of them are inside the batch; otherwise dL/dy of the
  // points beyond it is not stored.
  auto blocks = [&](const uint64_t p0, const uint64_t p0_next, auto full) {
    constexpr bool FULL = decltype(full)::value;
    // these blocks' y and dL/dout (layout P) were requested one round ahead; request the next ones
    half8 yP[kSub][2 * KB], g3P[kSub][OJ];
#pragma unroll
    for (int u = 0; u < kSub; ++u) {
#pragma unroll
      for (int j = 0; j < 2 * KB; ++j)
        yP[u][j] = __builtin_bit_cast(
            half8, uint4{y_next[u][2 * j].x, y_next[u][2 * j].y, y_next[u][2 * j + 1].x, y_next[u][2 * j + 1].y});
#pragma unroll
      for (int j = 0; j < OJ; ++j)
#pragma unroll
        for (int s8 = 0; s8 < 8; ++s8)  // rounded to half
          g3P[u][j][s8] = (2 * j + s8 / 4 < OS) ? (_Float16)d_next[u][(2 * j + s8 / 4) % OS][s8 % 4] : (_Float16)0.0f;
    }
    request(p0_next);
    // layout N of one 32-column tile of a matrix in layout P (steps z[0], z[1] of the tile): z x identity
    // with the operands exchanged; every sum has one term, so the copy is exact
    auto exchange = [&](const half8* z, const int steps, half8* out) {
      float16v aN = zero16();
#pragma unroll
      for (int j = 0; j < 2; ++j)
        if (j < steps) aN = mfma(z[j], one[j], aN);
#pragma unroll
      for (int j = 0; j < 2; ++j) out[j] = to_half(aN, j);
    };
    // dL/dout in layout N (lane = output, registers = points)
    half8 g3N[kSub][2];
#pragma unroll
    for (int u = 0; u < kSub; ++u) exchange(g3P[u], OJ, g3N[u]);

    // forward: h1 = relu(W1 y), h2 = relu(W2 h1) ([2 T + j]: tile T, step j)
    half8 h1P[kSub][4], h1N[kSub][4], h2P[kSub][4], h2N[kSub][4];
#pragma unroll
    for (int T = 0; T < 2; ++T) {
      float16v aP[kSub];
#pragma unroll
      for (int u = 0; u < kSub; ++u) aP[u] = zero16();
#pragma unroll
      for (int j = 0; j < 2 * KB; ++j) {
        const half8 w = frag(w1, sh.w1_stride, T, j);
#pragma unroll
        for (int u = 0; u < kSub; ++u) aP[u] = mfma(w, yP[u][j], aP[u]);
      }
#pragma unroll
      for (int u = 0; u < kSub; ++u) {
#pragma unroll
        for (int j = 0; j < 2; ++j) h1P[u][2 * T + j] = relu(to_half(aP[u], j));
        exchange(&h1P[u][2 * T], 2, &h1N[u][2 * T]);
      }
    }
#pragma unroll
    for (int T = 0; T < 2; ++T) {
      float16v aP[kSub];
#pragma unroll
      for (int u = 0; u < kSub; ++u) aP[u] = zero16();
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const half8 w = frag(w2, kHidStride, T, j);
#pragma unroll
        for (int u = 0; u < kSub; ++u) aP[u] = mfma(w, h1P[u][j], aP[u]);
      }
#pragma unroll
      for (int u = 0; u < kSub; ++u) {
#pragma unroll
        for (int j = 0; j < 2; ++j) h2P[u][2 * T + j] = relu(to_half(aP[u], j));
        exchange(&h2P[u][2 * T], 2, &h2N[u][2 * T]);
      }
    }
    // output layer: dW3[o][n] += sum_p dout[p][o] h2[p][n];  g2 = (W3^T dout) through the ReLU of layer 2
#pragma unroll
    for (int u = 0; u < kSub; ++u)
#pragma unroll
      for (int T = 0; T < 2; ++T)
#pragma unroll
        for (int j = 0; j < 2; ++j) aW3[T] = mfma(g3N[u][j], h2N[u][2 * T + j], aW3[T]);
    half8 g2P[kSub][4], g2N[kSub][4];
#pragma unroll
    for (int T = 0; T < 2; ++T) {
      float16v aP[kSub];
#pragma unroll
      for (int u = 0; u < kSub; ++u) aP[u] = zero16();
#pragma unroll
      for (int j = 0; j < OJ; ++j) {
        const half8 w = frag(w3t, sh.w3t_stride, T, j);
#pragma unroll
        for (int u = 0; u < kSub; ++u) aP[u] = mfma(w, g3P[u][j], aP[u]);
      }
#pragma unroll
      for (int u = 0; u < kSub; ++u) {
#pragma unroll
        for (int j = 0; j < 2; ++j) g2P[u][2 * T + j] = where_positive(to_half(aP[u], j), h2P[u][2 * T + j]);
        exchange(&g2P[u][2 * T], 2, &g2N[u][2 * T]);
      }
    }
    // second layer: dW2[m][n] += sum_p g2[p][m] h1[p][n];  g1 = (W2^T g2) through the ReLU of layer 1
#pragma unroll
    for (int u = 0; u < kSub; ++u)
#pragma unroll
      for (int Tm = 0; Tm < 2; ++Tm)
#pragma unroll
        for (int Tn = 0; Tn < 2; ++Tn)
#pragma unroll
          for (int j = 0; j < 2; ++j)
            aW2[2 * Tm + Tn] = mfma(g2N[u][2 * Tm + j], h1N[u][2 * Tn + j], aW2[2 * Tm + Tn]);
    half8 g1P[kSub][4], g1N[kSub][4];
#pragma unroll
    for (int T = 0; T < 2; ++T) {
      float16v aP[kSub];
#pragma unroll
      for (int u = 0; u < kSub; ++u) aP[u] = zero16();
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const half8 w = frag(w2t, kHidStride, T, j);
#pragma unroll
        for (int u = 0; u < kSub; ++u) aP[u] = mfma(w, g2P[u][j], aP[u]);
      }
#pragma unroll
      for (int u = 0; u < kSub; ++u) {
#pragma unroll
        for (int j = 0; j < 2; ++j) g1P[u][2 * T + j] = where_positive(to_half(aP[u], j), h1P[u][2 * T + j]);
        exchange(&g1P[u][2 * T], 2, &g1N[u][2 * T]);
      }
    }
    // first layer: dW1[n][k] += sum_p g1[p][n] y[p][k]
#pragma unroll
    for (int u = 0; u < kSub; ++u)
#pragma unroll
      for (int Tk = 0; Tk < KB; ++Tk) {
        half8 yN[2];
        exchange(&yP[u][2 * Tk], 2, yN);
#pragma unroll
        for (int Tn = 0; Tn < 2; ++Tn)
#pragma unroll
          for (int j = 0; j < 2; ++j) aW1[KB * Tn + Tk] = mfma(g1N[u][2 * Tn + j], yN[j], aW1[KB * Tn + Tk]);
      }
    // dL/dy = W1^T g1, layout P: four features per register group, straight to memory
#pragma unroll
    for (int Tk = 0; Tk < KB; ++Tk) {
      float16v d[kSub];
#pragma unroll
      for (int u = 0; u < kSub; ++u) d[u] = zero16();
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const half8 w = frag(w1t, kHidStride, Tk, j);
#pragma unroll
        for (int u = 0; u < kSub; ++u) d[u] = mfma(w, g1P[u][j], d[u]);
      }
#pragma unroll
      for (int u = 0; u < kSub; ++u) {
        const uint64_t p = p0 + kPts * u + c;
        if (FULL || p < B) {
#pragma unroll
          for (int j = 0; j < 2; ++j) {
            const half8 v = to_half(d[u], j);
#pragma unroll
            for (int e = 0; e < 2; ++e) {
              const int k = 32 * Tk + 16 * j + 8 * e + 4 * h;
              if (k < n_in)  // n_in is a multiple of 8: four at once
                *reinterpret_cast<half4*>(dy + p * n_in + k) = e == 0 ? __builtin_shufflevector(v, v, 0, 1, 2, 3)
                                                                     : __builtin_shufflevector(v, v, 4, 5, 6, 7);
            }
          }
        }
      }
    }
  };

  for (; rnd < n_rounds; rnd += stride) {
    // (keeps the compiler from holding the weight fragments, which do not change from round to round, in registers)
    asm volatile("" ::: "memory");
    const uint64_t p0 = (uint64_t)rnd * kRound, p0_next = ((uint64_t)rnd + stride) * kRound;
    if (p0 + kRound <= B) blocks(p0, p0_next, std::true_type{});
    else blocks(p0, p0_next, std::false_type{});
  }

  // The weight gradients of the workgroup.  Every wave writes its sums to LDS as they lie in its
  // registers ([wave][register][lane]; the weights are no longer needed), then every thread adds up
  // the waves' values of its share of (register, lane) pairs and sends one atomic add per scalar:
  // the 32 lanes of a half-wave hold 32 consecutive columns of a row.  Two rounds, so that the
  // area stays below 96 KiB: the second layer's 64 registers, then the first and the output layer's.
  // (Writing the workgroups' sums to a scratch buffer for a second kernel to add up was measured and is
  // slower than these atomics: 49 against 40 us at 2^18 points.)
  float* red = reinterpret_cast<float*>(lds);
  const int rot = (int)((blockIdx.x * 13u) % 64u);
  auto reduce = [&](auto&& store_all, const int g0, const int n_regs) {
    __syncthreads();  // the area is free: every wave is done with the weights (first round) or the round before
    store_all(red + wave * n_regs * 64 + lane);  // register r to [r * 64]
    __syncthreads();
    // (workgroups start at different registers, so that at any time they add to different lines of the gradient)
    for (int i = wave; i < n_regs; i += waves) {
      const int r = (i + rot) % n_regs;
      float v = 0.0f;
      for (int w = 0; w < waves; ++w) v += red[(w * n_regs + r) * 64 + lane];
      float* t = sum_target(g0 + r, lane, KB, n_in, n_out, dW1, dW2, dW3);
      if (t != nullptr && v != 0.0f) __hip_atomic_fetch_add(t, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  };
  reduce(
      [&](float* mine) {
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
          for (int q = 0; q < 16; ++q) mine[(16 * a + q) * 64] = aW2[a][q];
      },
      0, 64);
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
      64, 32 * KB + 32);
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
  // one workgroup per compute unit of the current device, at most
  int dev = 0, n_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu <= 0)
    n_cu = 256;
  const uint32_t cus = (uint32_t)n_cu;
  const uint32_t n_rounds = (B + hg::kSub * hg::kPts - 1) / (hg::kSub * hg::kPts);
  const uint32_t want = (n_rounds + waves - 1) / waves;
  const dim3 grid(want < cus ? want : cus), block(64 * waves);
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(kernels[sh.kin_pad / 32 - 1][(n_out + 7) / 8 - 1], grid, block, sh.lds_bytes(waves), s, B, sh,
                     static_cast<const _Float16*>(y), static_cast<const _Float16*>(W1), static_cast<const _Float16*>(W2),
                     static_cast<const _Float16*>(W3), dLdout, static_cast<_Float16*>(dLdy), dW1, dW2, dW3);
  return hipGetLastError() == hipSuccess ? HG_OK : HG_ERR_DEVICE;
}
