// The record of the sorted backward pass (what bin_scatter writes and bin_accumulate reads) and the
// fixed-point product of the accumulate pass.  Header-only and also compiled for the host, where
// tests check the format and its rounding without a GPU.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hg {

// A weight in [0,1] as a small float: `MBITS` mantissa bits under a 6-bit exponent, 0 for weights
// below 2^(LOW-127) (LOW is the fp32 exponent field that exponent code 1 stands for; such weights,
// 2^-62 and less, are far below what the fixed-point sums resolve).  The interpolation weights
// multiply dL/dy, so what the gradient needs of them is relative precision: half a unit of the
// mantissa, 2^-(MBITS+1), whatever the size of the weight.
template <int MBITS, int LOW>
__host__ __device__ __forceinline__ uint32_t pack_weight(float w) {
  const uint32_t b = __builtin_bit_cast(uint32_t, w) + (1u << (22 - MBITS));  // round to MBITS mantissa bits
  const uint32_t e8 = b >> 23;
  return e8 < (uint32_t)LOW ? 0u : ((e8 - (LOW - 1)) << MBITS) | ((b >> (23 - MBITS)) & ((1u << MBITS) - 1u));
}
template <int MBITS, int LOW>
__host__ __device__ __forceinline__ float unpack_weight(uint32_t c) {
  // exponent code and mantissa sit in the float's own order: one shift and one add rebuild it
  const uint32_t bits = (c << (23 - MBITS)) + ((uint32_t)(LOW - 1) << 23);
  return c >> MBITS ? __builtin_bit_cast(float, bits) : 0.0f;
}
constexpr uint32_t kFirstVoxel = 15u;  // value of the record's k field for a pair in the first voxel along dimension 0

// One record = one pair of corners that differ along dimension 0, both inside one chunk.
// Two header words, then the level's F values of dL/dy as they came (fp16 pairs share a word):
//   bits 0-11   la, chunk-local index of the lower corner;
//   bits 12-15  k: on a hashed level the upper corner is lb = la ^ (2^(k+1) - 1), k = number of
//               trailing one bits of the lower corner's coordinate along dimension 0 (pi_1 = 1
//               in Eq. 4, so stepping that coordinate XORs the index with this mask, cut to the
//               table size when the table is smaller than a chunk); on a 1:1 level lb = la + 1.
//               k = 15 (kFirstVoxel) says that this coordinate is 0 (so k is 0) and that the
//               next field is in its second form;
//   bits 16-38  the fractional position wf0 along dimension 0.  Whenever the scaled coordinate is 1
//               or more, its fraction is a multiple of 2^-23 and the field holds it exactly, in
//               units of 2^-23: both weights of the pair, wf0 and 1 - wf0, are exact.  In the first
//               voxel (scaled coordinate below 1, k = 15) the fraction can be any float: the field
//               then holds the smaller of wf0 and 1 - wf0 as a small float (16 mantissa bits) and,
//               in its top bit, which of the two that is; the other weight is 1 minus it
//               (for the smoothstep variant: of S(wf0) and S(1 - wf0) = 1 - S(wf0));
//   bits 39-63  wrow, product of the weights of the other dimensions, as a small float (19
//               mantissa bits; 0 and 1 exact).
// 12 bytes at F = 2 with fp16 dL/dy.  A corner's summand weight * dL/dy therefore moves by at most
// 2^-20 of itself through wrow, and by 2^-17 more for a pair in the first voxel: relative
// precision, inside the 1e-5 the gradient is held to.
// The two passes over the records are bound by memory bandwidth: their size is what sets the time.
template <typename IT, int F>
struct Record {
  static constexpr uint32_t kPayloadWords = (F * sizeof(IT) + 3) / 4;
  static constexpr uint32_t kWords = 2 + kPayloadWords;
  struct Stored {
    uint32_t w[kWords];
  };
  // `smooth`: the smoothstep variant (Appendix A of the paper).  Only the first-voxel form needs to
  // know: it stores the pair's final weights S(wf0), S(1 - wf0), because S would double the relative
  // error of a rounded small fraction; everywhere else the fraction is exact and S is applied by the reader.
  static __host__ __device__ __forceinline__ Stored make(uint32_t la, uint32_t k, float wf0, float wrow, const IT (&g)[F],
                                                         bool smooth = false) {
    uint32_t q0;
    if (k == kFirstVoxel) {
      const float one_minus = 1.0f - wf0;
      const float up = smooth ? wf0 * wf0 * (3.0f - 2.0f * wf0) : wf0;
      const float lo = smooth ? one_minus * one_minus * (3.0f - 2.0f * one_minus) : one_minus;
      const bool upper_small = up <= lo;                // which of the pair's two weights the field holds
      q0 = (upper_small ? 0u : 1u << 22) | pack_weight<16, 64>(upper_small ? up : lo);
    } else {
      q0 = (uint32_t)rintf(wf0 * 0x1p23f);
      q0 = q0 < 0x7fffffu ? q0 : 0x7fffffu;
    }
    const uint32_t qr = pack_weight<19, 65>(wrow);
    const uint64_t p = (uint64_t)(la | (k << 12)) | ((uint64_t)q0 << 16) | ((uint64_t)qr << 39);
    Stored r;
    r.w[0] = (uint32_t)p;
    r.w[1] = (uint32_t)(p >> 32);
    IT pay[kPayloadWords * 4 / sizeof(IT)];
#pragma unroll
    for (uint32_t f = 0; f < kPayloadWords * 4 / sizeof(IT); ++f) pay[f] = f < (uint32_t)F ? g[f] : (IT)0;
    __builtin_memcpy(&r.w[2], pay, kPayloadWords * 4);
    return r;
  }
  static __host__ __device__ __forceinline__ Stored load(const uint32_t* base, uint32_t i) {
    const uint32_t* p = base + (uint64_t)i * kWords;
    Stored r;
#pragma unroll
    for (uint32_t q = 0; q < kWords; ++q) r.w[q] = __builtin_nontemporal_load(p + q);
    return r;
  }
  // la, lb, the pair's two weights along dimension 0 (w_lo for the lower corner, w_up for the upper
  // one: 1 - wf0 and wf0, to which the reader applies the smoothstep where the variant asks for it,
  // unless `first` says that the record is in its first-voxel form, which holds the final weights)
  // and the F totals of the pair, wrow * dL/dy_f, as doubles times `scale`: a 20-bit by at most
  // 24-bit product, exact in a double.
  // `xmask`: on a hashed level, the chunk's entry count minus one (a table smaller than a chunk
  // wraps the XOR); `cmask`: the chunk capacity minus one
  static __host__ __device__ __forceinline__ void unpack_scaled(const Stored& r, bool dense, uint32_t cmask, uint32_t xmask,
                                                       double scale, uint32_t& la, uint32_t& lb, float& w_lo,
                                                       float& w_up, bool& first, double (&G)[F]) {
    const uint64_t p = (uint64_t)r.w[0] | ((uint64_t)r.w[1] << 32);
    la = r.w[0] & 0xfffu & cmask;
    uint32_t k = (r.w[0] >> 12) & 0xfu;
    const uint32_t q0 = (uint32_t)(p >> 16) & 0x7fffffu;
    first = k == kFirstVoxel;
    if (__builtin_expect(first, 0)) {  // rare: one voxel in N_l along dimension 0
      k = 0;
      const float small = unpack_weight<16, 64>(q0 & 0x3fffffu), big = 1.0f - small;
      const bool upper_small = (q0 >> 22) == 0u;
      w_up = upper_small ? small : big;
      w_lo = upper_small ? big : small;
    } else {
      w_up = (float)q0 * 0x1p-23f;
      w_lo = 1.0f - w_up;  // exact
    }
    lb = dense ? (la + 1u) & cmask : la ^ (((2u << k) - 1u) & xmask);
    const double wrow = (double)unpack_weight<19, 65>((uint32_t)(p >> 39)) * scale;
    IT pay[kPayloadWords * 4 / sizeof(IT)];
    __builtin_memcpy(pay, &r.w[2], kPayloadWords * 4);
#pragma unroll
    for (int f = 0; f < F; ++f) G[f] = wrow * (double)(float)pay[f];
  }
};

// round(w * G) to a 64-bit integer (ties to even), for |w * G| < 2^51: adding
// 1.5 * 2^52 leaves the integer, in two's complement, in the low bits of the
// double.  One rounding, of the exact product.
constexpr int kFixedBits = 51;
__host__ __device__ __forceinline__ unsigned long long fixed_product(float w, double G) {
  const double d = __builtin_fma((double)w, G, 0x1.8p52);
  return (unsigned long long)(__builtin_bit_cast(long long, d) - __builtin_bit_cast(long long, 0x1.8p52));
}

}  // namespace hg
