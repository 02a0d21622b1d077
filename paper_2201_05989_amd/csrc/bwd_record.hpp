// The record of the sorted backward pass (what bin_scatter writes and bin_accumulate reads) and the
// fixed-point product of the accumulate pass.  Header-only and also compiled for the host, where
// tests check the format and its rounding without a GPU.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hg {

// One record = one pair of corners that differ along dimension 0, both inside one chunk.
// Two header words, then the level's F values of dL/dy as they came (fp16 pairs share a word):
//   bits 0-11   la, chunk-local index of the lower corner;
//   bits 12-15  k: on a hashed level the upper corner is lb = la ^ (2^(k+1) - 1), k = number of
//               trailing one bits of the lower corner's coordinate along dimension 0 (pi_1 = 1
//               in Eq. 4, so stepping that coordinate XORs the index with this mask, cut to the
//               table size when the table is smaller than a chunk); on a 1:1 level lb = la + 1;
//   bits 16-38  wf0, fractional position along dimension 0, in units of 2^-23 (exact whenever
//               the scaled coordinate is 1 or more, because then its fraction is a multiple of
//               2^-23; otherwise rounded, off by 2^-24 at most);
//   bits 39-63  wrow, product of the weights of the other dimensions, in units of 2^-24 (0 and
//               1 exact, off by 2^-25 at most).
// 12 bytes at F = 2 with fp16 dL/dy.  Both weights lie in [0,1] and the weights of a pair, and
// of the rows of a point, sum to 1, so the rounding moves a gradient entry by at most about
// 2^-23 times the sum of |dL/dy| over the corners that touch it.  The two passes over the
// records are bound by memory bandwidth: their size is what sets the time.
template <typename IT, int F>
struct Record {
  static constexpr uint32_t kPayloadWords = (F * sizeof(IT) + 3) / 4;
  static constexpr uint32_t kWords = 2 + kPayloadWords;
  struct Stored {
    uint32_t w[kWords];
  };
  static __host__ __device__ __forceinline__ Stored make(uint32_t la, uint32_t k, float wf0, float wrow, const IT (&g)[F]) {
    uint32_t q0 = (uint32_t)rintf(wf0 * 0x1p23f);
    q0 = q0 < 0x7fffffu ? q0 : 0x7fffffu;
    uint32_t qr = (uint32_t)rintf(wrow * 0x1p24f);
    qr = qr < 0x1000000u ? qr : 0x1000000u;
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
  // la, lb, wf0 and the F totals of the pair, wrow * dL/dy_f, as doubles times `scale`: a 25-bit
  // by at most 24-bit product, exact in a double
  // `xmask`: on a hashed level, the chunk's entry count minus one (a table smaller than a chunk
  // wraps the XOR); `cmask`: the chunk capacity minus one
  static __host__ __device__ __forceinline__ void unpack_scaled(const Stored& r, bool dense, uint32_t cmask, uint32_t xmask,
                                                       double scale, uint32_t& la, uint32_t& lb, float& wf0,
                                                       double (&G)[F]) {
    const uint64_t p = (uint64_t)r.w[0] | ((uint64_t)r.w[1] << 32);
    la = r.w[0] & 0xfffu & cmask;
    const uint32_t k = (r.w[0] >> 12) & 0xfu;
    lb = dense ? (la + 1u) & cmask : la ^ (((2u << k) - 1u) & xmask);
    wf0 = (float)((uint32_t)(p >> 16) & 0x7fffffu) * 0x1p-23f;
    const double wrow = (double)(uint32_t)(p >> 39) * (scale * 0x1p-24);
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
