// Shared device-side pieces of the gfx950 hash-encoding kernels: the level table
// passed by value to every kernel, the fp32 scale/floor step and the corner
// index maps (paper Section 3, Eq. 2-4).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hashgrid.h"

namespace hg {

// Level table of Eq. 2-3, built once on the host and handed to kernels as a
// by-value argument (it lives in the kernarg segment, read through the scalar
// cache; the library owns no device memory).
struct LevelTable {
  uint64_t offset[HG_MAX_LEVELS];  // first entry of the level in the flat table
  uint32_t N[HG_MAX_LEVELS];       // resolution N_l
  uint32_t verts[HG_MAX_LEVELS];   // grid vertices per axis on a 1:1 level (N_l+1; N_l+2 when shifted)
  uint32_t size[HG_MAX_LEVELS];    // entries of the level
  uint32_t dense_mask;             // bit l set: level l is 1:1 indexed
  uint32_t L;
  uint32_t T;
  uint32_t T_is_pow2;
};

// Eq. 4: pi_1 = 1, pi_2 = 2654435761, pi_3 = 805459861.
__host__ __device__ __forceinline__ constexpr uint32_t prime(int i) {
  return i == 0 ? 1u : (i == 1 ? 2654435761u : 805459861u);
}

// Section 3: scale one coordinate by N_l (one rounded fp32 multiply), take the
// lower voxel corner and the fractional position.  `shift` is the half-voxel
// offset of Appendix A (0 or 0.5).  The corner is clamped to [0, cmax] so that a
// coordinate outside [0,1) (a violated precondition) can never index outside a
// 1:1 level; for valid input the clamp is the identity.
__host__ __device__ __forceinline__ void split(float x, float Nf, float shift, float cmaxf, uint32_t& c0, float& w) {
  float p = x * Nf;
  p = p + shift;  // the file is compiled with fp contraction off: two roundings
  float fl = floorf(p);
  w = p - fl;     // exact
  c0 = (uint32_t)fminf(fmaxf(fl, 0.0f), cmaxf);
}

// Per-dimension contribution of a corner coordinate to the entry index: on a 1:1
// level v_i * verts^i (summed), on a hashed level v_i * pi_i (XORed).
template <int D>
struct CornerTerms {
  uint32_t t[D][2];
};

template <int D>
__device__ __forceinline__ CornerTerms<D> corner_terms(const uint32_t (&c0)[D], bool dense, uint32_t verts) {
  CornerTerms<D> r;
  uint32_t stride = 1;
#pragma unroll
  for (int i = 0; i < D; ++i) {
    uint32_t mul = dense ? stride : prime(i);
    r.t[i][0] = c0[i] * mul;
    r.t[i][1] = r.t[i][0] + mul;  // (c0+1)*mul in wrap-around arithmetic
    stride *= verts;
  }
  return r;
}

template <int D>
__device__ __forceinline__ uint32_t corner_index(const CornerTerms<D>& ct, uint32_t m, bool dense, uint32_t T,
                                                 bool pow2) {
  if (dense) {
    uint32_t idx = 0;
#pragma unroll
    for (int i = 0; i < D; ++i) idx += ct.t[i][(m >> i) & 1u];
    return idx;
  }
  uint32_t h = 0;
#pragma unroll
  for (int i = 0; i < D; ++i) h ^= ct.t[i][(m >> i) & 1u];
  return pow2 ? (h & (T - 1u)) : (h % T);
}

// Device-scope atomic add of one scalar of the table gradient.  Half-precision gradients (the
// paper accumulates them in half precision, Section 4 / Fig. 5) use the packed two-half atomic, the
// partner half receiving +0: the buffer must therefore start on a 4-byte boundary and its allocation
// must extend to one.
using half2_t = _Float16 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void grad_atomic_add(float* base, uint64_t i, float v) {
  __hip_atomic_fetch_add(base + i, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void grad_atomic_add(_Float16* base, uint64_t i, float v) {
  const uintptr_t a = reinterpret_cast<uintptr_t>(base + i);
  half2_t pk;
  pk.x = (a & 2u) ? (_Float16)0.0f : (_Float16)v;
  pk.y = (a & 2u) ? (_Float16)v : (_Float16)0.0f;
  __builtin_amdgcn_global_atomic_fadd_v2f16(reinterpret_cast<half2_t*>(a & ~(uintptr_t)3), pk);
}
// ... of two neighbouring scalars that start on a 4-byte boundary (one request instead of two)
__device__ __forceinline__ void grad_atomic_add2(float*, uint64_t, float, float) {}  // (never called: fp32 gradients add scalars)
__device__ __forceinline__ void grad_atomic_add2(_Float16* base, uint64_t i, float v0, float v1) {
  half2_t pk;
  pk.x = (_Float16)v0;
  pk.y = (_Float16)v1;
  __builtin_amdgcn_global_atomic_fadd_v2f16(reinterpret_cast<half2_t*>(base + i), pk);
}

// Appendix A: S(w) = w^2 (3 - 2w), S'(w) = 6 w (1 - w).
__host__ __device__ __forceinline__ float smoothstep(float w) { return w * w * (3.0f - 2.0f * w); }
__device__ __forceinline__ float dsmoothstep(float w) { return 6.0f * w * (1.0f - w); }

// F scalars of one table entry / one output fragment, loaded and stored as one
// vector access (two for the 32-byte ones: the entry points ask for 16-byte
// alignment at most, so the type must not promise more).
template <typename T, int F>
struct alignas(sizeof(T) * F > 16 ? 16 : sizeof(T) * F) Vec {
  T v[F];
};

// Entry indices of the 2^D corners for a level known (uniformly) to be 1:1 or
// hashed, T a power of two on the hashed side: no per-lane selects between the
// two index maps and no integer division.
template <int D, bool DENSE>
__device__ __forceinline__ void corner_indices_uniform(const uint32_t (&c0)[D], uint32_t verts, uint32_t mask,
                                                       uint32_t (&idx)[1 << D]) {
  uint32_t t[D][2];
  uint32_t stride = 1;
#pragma unroll
  for (int i = 0; i < D; ++i) {
    const uint32_t mul = DENSE ? stride : prime(i);
    t[i][0] = c0[i] * mul;
    t[i][1] = t[i][0] + mul;
    stride *= verts;
  }
#pragma unroll
  for (uint32_t m = 0; m < (1u << D); ++m) {
    uint32_t v = t[0][m & 1u];
#pragma unroll
    for (int i = 1; i < D; ++i) v = DENSE ? v + t[i][(m >> i) & 1u] : v ^ t[i][(m >> i) & 1u];
    idx[m] = DENSE ? v : v & mask;
  }
}

// Per level and point: the 2^D entry indices and the weights of the corners, split into the
// product over dimensions 1.. (wr) and the two weights of dimension 0 (w0 upper, u0 lower).
// c0: the voxel's lower corner (integer coordinates).
template <int D, bool POW2>
__device__ __forceinline__ void level_corners(const LevelTable& lv, uint32_t l, bool smooth, const float (&xp)[D],
                                              uint32_t (&idx)[1 << D], float (&wr)[1 << (D - 1)], float& w0,
                                              float& u0, uint32_t (&c0)[D]) {
  const float Nf = (float)lv.N[l];
  const float shift = smooth ? 0.5f : 0.0f;
  const float cmaxf = smooth ? Nf : Nf - 1.0f;
  float w[D], u[D];
#pragma unroll
  for (int i = 0; i < D; ++i) {
    float wf;
    split(xp[i], Nf, shift, cmaxf, c0[i], wf);
    w[i] = smooth ? smoothstep(wf) : wf;
    u[i] = smooth ? smoothstep(1.0f - wf) : 1.0f - wf;
  }
  if ((lv.dense_mask >> l) & 1u) {  // uniform
    corner_indices_uniform<D, true>(c0, lv.verts[l], 0u, idx);
  } else if (POW2) {
    corner_indices_uniform<D, false>(c0, 0u, lv.T - 1u, idx);
  } else {
    const CornerTerms<D> ct = corner_terms<D>(c0, false, 0u);
#pragma unroll
    for (uint32_t m = 0; m < (1u << D); ++m) idx[m] = corner_index<D>(ct, m, false, lv.T, false);
  }
#pragma unroll
  for (uint32_t r = 0; r < (1u << (D - 1)); ++r) {
    float p = 1.0f;
#pragma unroll
    for (int i = 1; i < D; ++i) p *= ((r >> (i - 1)) & 1u) ? w[i] : u[i];
    wr[r] = p;
  }
  w0 = w[0];
  u0 = u[0];
}

template <int D, bool POW2>
__device__ __forceinline__ void level_corners(const LevelTable& lv, uint32_t l, bool smooth, const float (&xp)[D],
                                              uint32_t (&idx)[1 << D], float (&wr)[1 << (D - 1)], float& w0,
                                              float& u0) {
  uint32_t c0[D];
  level_corners<D, POW2>(lv, l, smooth, xp, idx, wr, w0, u0, c0);
}

}  // namespace hg
