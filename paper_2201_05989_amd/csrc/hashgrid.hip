// C ABI of the multiresolution hash encoding (declared in include/hashgrid.h)
// and the general gfx950 kernels that serve every supported configuration.
//
// Kernel shape: the paper evaluates the tables level by level so that only a few
// level slices are live in cache at once (Section 4, "Performance
// considerations"); the general kernels here keep that order: one thread per
// (point, level), the level being the slow grid dimension.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <new>
#include <type_traits>

#include "hashgrid.h"
#include "hashgrid_common.hpp"
#include "hashgrid_internal.hpp"
#include "bwd_bins.hpp"

namespace hg {

constexpr int kBlock = 256;

// ------------------------------------------------------------------ kernels

// Per (point, level): the 2^d entry indices and interpolation weights
// (Section 3), optionally the derivative of each weight along each axis.
template <int D>
struct Corners {
  uint32_t idx[1 << D];
  float wt[1 << D];
};

template <int D, bool WITH_DERIV>
__device__ __forceinline__ void corners_of(const LevelTable& lv, uint32_t l, bool smooth, const float* xp,
                                           Corners<D>& out, float (*dwt)[1 << D]) {
  const uint32_t N = lv.N[l];
  const bool dense = (lv.dense_mask >> l) & 1u;
  const float Nf = (float)N;
  const float shift = smooth ? 0.5f : 0.0f;
  const float cmaxf = smooth ? Nf : Nf - 1.0f;
  uint32_t c0[D];
  float w[D], u[D], dw[D];  // weight of the upper corner, of the lower corner, d(upper)/dx
#pragma unroll
  for (int i = 0; i < D; ++i) {
    float wf;
    split(xp[i], Nf, shift, cmaxf, c0[i], wf);
    // 1 - S(w) = S(1 - w): evaluating the lower weight this way keeps its relative
    // accuracy when S(w) is close to 1
    w[i] = smooth ? smoothstep(wf) : wf;
    u[i] = smooth ? smoothstep(1.0f - wf) : 1.0f - wf;
    if (WITH_DERIV) dw[i] = smooth ? dsmoothstep(wf) * Nf : Nf;
  }
  const CornerTerms<D> ct = corner_terms<D>(c0, dense, lv.verts[l]);
#pragma unroll
  for (uint32_t m = 0; m < (1u << D); ++m) {
    out.idx[m] = corner_index<D>(ct, m, dense, lv.T, lv.T_is_pow2 != 0);
    float wt = 1.0f;
#pragma unroll
    for (int i = 0; i < D; ++i) wt *= ((m >> i) & 1u) ? w[i] : u[i];
    out.wt[m] = wt;
    if (WITH_DERIV) {
#pragma unroll
      for (int j = 0; j < D; ++j) {
        float g = ((m >> j) & 1u) ? dw[j] : -dw[j];
#pragma unroll
        for (int i = 0; i < D; ++i)
          if (i != j) g *= ((m >> i) & 1u) ? w[i] : u[i];
        dwt[j][m] = g;
      }
    }
  }
}

template <int D>
__device__ __forceinline__ void load_point(const float* __restrict__ x, uint32_t b, float (&xp)[D]) {
#pragma unroll
  for (int i = 0; i < D; ++i) xp[i] = x[(uint64_t)b * D + i];
}

// Forward, Section 3 / Fig. 3 steps 1-4.
template <int D, int F, typename PT, typename IT>
__global__ __launch_bounds__(kBlock) void fwd_general(const LevelTable lv, const bool smooth, const uint32_t B,
                                                      const float* __restrict__ x, const PT* __restrict__ theta,
                                                      IT* __restrict__ y) {
  const uint32_t l = blockIdx.y;
  const uint32_t b = blockIdx.x * kBlock + threadIdx.x;
  if (b >= B) return;
  float xp[D];
  load_point<D>(x, b, xp);
  Corners<D> cn;
  corners_of<D, false>(lv, l, smooth, xp, cn, nullptr);
  const Vec<PT, F>* tab = reinterpret_cast<const Vec<PT, F>*>(theta) + lv.offset[l];
  float acc[F];
#pragma unroll
  for (int f = 0; f < F; ++f) acc[f] = 0.0f;
#pragma unroll
  for (uint32_t m = 0; m < (1u << D); ++m) {
    const Vec<PT, F> e = tab[cn.idx[m]];
#pragma unroll
    for (int f = 0; f < F; ++f) acc[f] = fmaf(cn.wt[m], (float)e.v[f], acc[f]);
  }
  Vec<IT, F> out;
#pragma unroll
  for (int f = 0; f < F; ++f) out.v[f] = (IT)acc[f];
  reinterpret_cast<Vec<IT, F>*>(y)[(uint64_t)b * lv.L + l] = out;
}

// Forward, point-major: one thread owns a point and walks the levels in
// order, so x is read once and the output row leaves the thread as 16-byte
// pieces.  (The level-major kernel above writes 2*sizeof(io) bytes per thread
// with a stride of a whole row; each such fragment costs a whole 32-byte sector
// of write traffic.)  The paper's level-by-level order (Section 4), which keeps
// one level's slice hot in cache, is kept in time rather than in the grid: all
// resident workgroups start at level 0 together, and the barrier per level
// keeps the 16 waves of a workgroup on the same slice, which holds the L2 hit
// rate at that of the level-major grid.
constexpr int kPmBlock = 1024;
// Threads (= points) per workgroup of the point-major kernels.  One workgroup's time does not
// depend on how many others run - the kernels are bound by what one CU's texture path and L1
// deliver - so 2^14 points in sixteen full workgroups take as long as 2^18 in 256, and 300 K points
// in 293 as long as 2^19.  The batch is therefore spread evenly: k = number of rounds the batch
// needs at full size, then B / (k * CUs) points per workgroup, rounded up to whole waves.  (The
// counting variant always runs full workgroups: they cover whole tiles of the backward pass.)
static uint32_t cu_count() {
  static const uint32_t cus = [] {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
      n = 256;
    return (uint32_t)n;
  }();
  return cus;
}
uint32_t point_major_block(uint32_t B) {
  const uint32_t cus = cu_count();
  const uint64_t per_round = (uint64_t)kPmBlock * cus;
  const uint64_t rounds = (B + per_round - 1) / per_round;
  const uint64_t per_wg = (B + rounds * cus - 1) / (rounds * cus);
  const uint32_t block = (uint32_t)((per_wg + 63) / 64 * 64);
  return block < 64 ? 64 : (block > (uint32_t)kPmBlock ? (uint32_t)kPmBlock : block);
}
constexpr size_t kMaxCountingLds = 128 * 1024;  // histograms of a counting forward workgroup (one workgroup per CU)

// Levels whose outputs fill one store: 16 bytes, or one level when a level's F outputs are wider.
template <int F, typename IT>
struct OutPiece {
  static constexpr int kLevelBytes = F * (int)sizeof(IT);
  static constexpr int kBytes = kLevelBytes > 16 ? kLevelBytes : 16;
  static constexpr int kLevels = kBytes / kLevelBytes;
  static constexpr bool kPair = kBytes == 16;  // two pieces make a 32-byte sector
};

// With COUNT the kernel also fills, for the binned backward pass over the same points, the
// table that pass would otherwise count in a kernel of its own: counts[tile][bin] = pairs of
// corners of the tile's kBinThreads points that fall into the bin (bwd_binned.hip).  The
// gathers leave the vector ALU and the LDS idle, so the counting rides along.
struct CountArgs {
  BinPlan bp;
  uint32_t* counts;  // [n_tiles][n_bins]
  uint32_t n_bins, n_tiles;
};
struct NoCount {};

// SB: points per thread.  A workgroup then walks SB blocks of blockDim.x points level by level,
// so that a level's slice, once in the XCD's L2, serves SB times the points before the next
// level replaces it (for batches of several rounds of workgroups per CU).
template <int D, int F, typename PT, typename IT, bool POW2, bool COUNT, int SB = 1>
__global__ __launch_bounds__(kPmBlock) void fwd_point_major(const LevelTable lv, const bool smooth, const uint32_t B,
                                                            const float* __restrict__ x,
                                                            const PT* __restrict__ theta, IT* __restrict__ y,
                                                            const typename std::conditional<COUNT, CountArgs, NoCount>::type ca) {
  using Piece = OutPiece<F, IT>;
  constexpr int G = Piece::kLevels;
  constexpr uint32_t kTiles = SB * kPmBlock / kBinThreads;  // tiles of the backward pass per workgroup
  static_assert(kPmBlock % kBinThreads == 0, "a forward workgroup covers whole tiles");
  extern __shared__ uint32_t hist[];  // COUNT: [kTiles][n_bins]
  if constexpr (COUNT) {
    for (uint32_t i = threadIdx.x; i < kTiles * ca.n_bins; i += kPmBlock) hist[i] = 0;
    __syncthreads();
  }
  bool valid[SB];
  float xp[SB][D];
  Vec<IT, F * G>* yrow[SB];
#pragma unroll
  for (int q = 0; q < SB; ++q) {
    const uint64_t b0 = ((uint64_t)blockIdx.x * SB + q) * blockDim.x + threadIdx.x;  // blockDim.x = kPmBlock with COUNT
    valid[q] = b0 < B;
    const uint32_t b = valid[q] ? (uint32_t)b0 : B - 1;  // idle lanes shadow the last point
    load_point<D>(x, b, xp[q]);
    yrow[q] = reinterpret_cast<Vec<IT, F * G>*>(y + (uint64_t)b * lv.L * F);
  }
  // 16-byte pieces are stored two at a time so that a 32-byte sector of the row is written
  // once, not twice
  Vec<IT, F * G> held[SB];
  // One point per thread, no counting: the gathers of level l+1 are issued before level l is blended, so
  // the texture path has work while the waves compute indices and wait at the barrier (two register
  // sets that alternate; the parity of a level inside a piece must be known at compile time).  With
  // the counting on the side the plain order is the faster one: there the counting fills those gaps.
  constexpr bool PIPE = SB == 1 && G % 2 == 0 && !COUNT;
  constexpr int kSets = PIPE ? 2 : 1;
  Vec<PT, F> e[kSets][SB][1 << D];
  float wr[kSets][SB][1 << (D - 1)], w0[kSets][SB], u0[kSets][SB];
  auto gather_level = [&](const uint32_t l, const int set) {
    const Vec<PT, F>* tab = reinterpret_cast<const Vec<PT, F>*>(theta) + lv.offset[l];
#pragma unroll
    for (int q = 0; q < SB; ++q) {
      uint32_t idx[1 << D], c0[D];
      level_corners<D, POW2>(lv, l, smooth, xp[q], idx, wr[set][q], w0[set][q], u0[set][q], c0);
#pragma unroll
      for (uint32_t m = 0; m < (1u << D); ++m) e[set][q][m] = tab[idx[m]];
      if constexpr (COUNT) {
        // The bin of each pair of corners along dimension 0, as rows_of (bwd_bins.hpp) defines it, from
        // what the gathers have just computed: a hashed level's bin is the chunk of the lower corner's
        // entry, a 1:1 level's the group of grid rows of the pair.  (COUNT implies a power-of-two T.)
        if (valid[q]) {
          const uint32_t cl = ca.bp.chunk_log2, gb0 = ca.bp.bin_base[l];
          uint32_t* h = hist + (q * (kPmBlock / kBinThreads) + threadIdx.x / kBinThreads) * ca.n_bins;
          if ((lv.dense_mask >> l) & 1u) {  // uniform
            const uint32_t sh = ca.bp.row_shift[l], verts = lv.verts[l];
#pragma unroll
            for (uint32_t r = 0; r < (1u << (D - 1)); ++r) {
              uint32_t row = c0[1] + (r & 1u);
              if (D == 3) row += (c0[D - 1] + (r >> 1)) * verts;
              count_one(h, gb0 + (row >> sh));
            }
          } else if ((c0[0] & ((1u << cl) - 1u)) != (1u << cl) - 1u) {  // else the pairs straddle two chunks: no record
#pragma unroll
            for (uint32_t r = 0; r < (1u << (D - 1)); ++r)
              count_one(h, gb0 + (idx[2 * r] >> cl));
          }
        }
      }
    }
  };
  if constexpr (PIPE) gather_level(0, 0);
  for (uint32_t l0 = 0; l0 < lv.L; l0 += G) {
    Vec<IT, F * G> out[SB];
#pragma unroll
    for (int j = 0; j < G; ++j) {
      const uint32_t l = l0 + j;
      const int set = PIPE ? (j & 1) : 0;  // lv.L is a multiple of G (checked at launch), G even: l and j have the same parity
      if constexpr (PIPE) {
        if (l + 1 < lv.L) gather_level(l + 1, set ^ 1);
      } else {
        gather_level(l, 0);
      }
#pragma unroll
      for (int q = 0; q < SB; ++q) {
        float acc[F];
#pragma unroll
        for (int f = 0; f < F; ++f) acc[f] = 0.0f;
#pragma unroll
        for (uint32_t m = 0; m < (1u << D); ++m) {
          const float wt = wr[set][q][m >> 1] * ((m & 1u) ? w0[set][q] : u0[set][q]);
#pragma unroll
          for (int f = 0; f < F; ++f) acc[f] = fmaf(wt, (float)e[set][q][m].v[f], acc[f]);
        }
#pragma unroll
        // (the compiler folds this conversion into the last multiply-add in some instantiations and
        // not in others - one rounding instead of two - so two variants of the kernel may differ in
        // the last bit of an fp16 output that is an exact tie)
        for (int f = 0; f < F; ++f) out[q].v[F * j + f] = (IT)acc[f];
      }
      asm volatile("" ::: "memory");  // keep the gathers of one level together
      // Pacing only: the barrier keeps the waves of the workgroup on the same level's slice; no data
      // passes between them here.  Measured: the counting variant is faster with the bare barrier
      // (no fence: its LDS atomics need not have landed), the plain one with the fenced one.
      if constexpr (COUNT) __builtin_amdgcn_s_barrier();
      else __syncthreads();
    }
    const uint32_t piece = l0 / G;
#pragma unroll
    for (int q = 0; q < SB; ++q) {
      if (Piece::kPair && (piece & 1u) == 0 && l0 + G < lv.L) {
        held[q] = out[q];  // even piece with a partner: keep it until the partner is ready
      } else if (valid[q]) {
        if (Piece::kPair && (piece & 1u)) yrow[q][piece - 1] = held[q];
        yrow[q][piece] = out[q];
      }
    }
  }
  if constexpr (COUNT) {
    __syncthreads();  // every wave's LDS atomics have landed: the histograms are complete
#pragma unroll
    for (uint32_t t = 0; t < kTiles; ++t) {
      const uint32_t tile = blockIdx.x * kTiles + t;
      if (tile >= ca.n_tiles) break;
      for (uint32_t i = threadIdx.x; i < ca.n_bins; i += kPmBlock)
        ca.counts[(uint64_t)tile * ca.n_bins + i] = hist[t * ca.n_bins + i];
    }
  }
}

// Gradient with respect to the position, point-major, same structure as the forward kernel
// (one barrier per level, dL/dy read as 16-byte pieces).  Per level the 2^D gathered entries
// are first contracted with dL/dy (s_m = sum_f g_f theta_m,f); the derivative of the d-linear
// blend of the s_m then follows dimension by dimension: along a dimension with weights (u, w)
// and slope dw, a pair (lower a, upper b) becomes value u a + w b and derivative dw (b - a).
template <int D, int F, typename PT, typename IT, bool POW2, int SB = 1>  // SB: points per thread, as in fwd_point_major
__global__ __launch_bounds__(kPmBlock) void bwd_input_point_major(const LevelTable lv, const bool smooth,
                                                                  const uint32_t B, const float* __restrict__ x,
                                                                  const PT* __restrict__ theta,
                                                                  const IT* __restrict__ dy, float* __restrict__ dx) {
  using Piece = OutPiece<F, IT>;
  constexpr int G = Piece::kLevels;
  bool valid[SB];
  uint32_t b[SB];
  float xp[SB][D], gx[SB][D];
  const Vec<IT, F * G>* grow[SB];
#pragma unroll
  for (int q = 0; q < SB; ++q) {
    const uint64_t b0 = ((uint64_t)blockIdx.x * SB + q) * blockDim.x + threadIdx.x;
    valid[q] = b0 < B;
    b[q] = valid[q] ? (uint32_t)b0 : B - 1;
    load_point<D>(x, b[q], xp[q]);
    grow[q] = reinterpret_cast<const Vec<IT, F * G>*>(dy + (uint64_t)b[q] * lv.L * F);
#pragma unroll
    for (int j = 0; j < D; ++j) gx[q][j] = 0.0f;
  }
  const float shift = smooth ? 0.5f : 0.0f;
  for (uint32_t l0 = 0; l0 < lv.L; l0 += G) {
    Vec<IT, F * G> g[SB];
#pragma unroll
    for (int q = 0; q < SB; ++q) g[q] = grow[q][l0 / G];
#pragma unroll
    for (int j = 0; j < G; ++j) {
      const uint32_t l = l0 + j;
      const float Nf = (float)lv.N[l];
      const float cmaxf = smooth ? Nf : Nf - 1.0f;
      const Vec<PT, F>* tab = reinterpret_cast<const Vec<PT, F>*>(theta) + lv.offset[l];
      Vec<PT, F> e[SB][1 << D];
      float w[SB][D], u[SB][D], dw[SB][D];
#pragma unroll
      for (int q = 0; q < SB; ++q) {
        uint32_t c0[D], idx[1 << D];
#pragma unroll
        for (int i = 0; i < D; ++i) {
          float wf;
          split(xp[q][i], Nf, shift, cmaxf, c0[i], wf);
          w[q][i] = smooth ? smoothstep(wf) : wf;
          u[q][i] = smooth ? smoothstep(1.0f - wf) : 1.0f - wf;
          dw[q][i] = smooth ? dsmoothstep(wf) * Nf : Nf;
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
        for (uint32_t m = 0; m < (1u << D); ++m) e[q][m] = tab[idx[m]];
      }
#pragma unroll
      for (int q = 0; q < SB; ++q) {
        // val[m]: blend over the dimensions folded so far; der[i][m]: its derivative along dimension i
        float val[1 << D], der[D][1 << D];
#pragma unroll
        for (uint32_t m = 0; m < (1u << D); ++m) {
          float sm = 0.0f;
#pragma unroll
          for (int f = 0; f < F; ++f) sm = fmaf((float)g[q].v[F * j + f], (float)e[q][m].v[f], sm);
          val[m] = sm;
        }
#pragma unroll
        for (int i = 0; i < D; ++i) {        // fold dimension i: corners m (bit i clear) and m | 1<<i
#pragma unroll
          for (uint32_t m = 0; m < (1u << D); ++m) {
            if (m & ((2u << i) - 1u)) continue;  // representatives: bits 0..i clear
            const uint32_t hi = m | (1u << i);
#pragma unroll
            for (int k = 0; k < i; ++k) der[k][m] = u[q][i] * der[k][m] + w[q][i] * der[k][hi];
            der[i][m] = dw[q][i] * (val[hi] - val[m]);
            val[m] = u[q][i] * val[m] + w[q][i] * val[hi];
          }
        }
#pragma unroll
        for (int i = 0; i < D; ++i) gx[q][i] += der[i][0];
      }
      asm volatile("" ::: "memory");
      __syncthreads();
    }
  }
#pragma unroll
  for (int q = 0; q < SB; ++q) {
    if (valid[q]) {
#pragma unroll
      for (int i = 0; i < D; ++i) dx[(uint64_t)b[q] * D + i] = gx[q][i];
    }
  }
}

// Backward to the tables, Fig. 3 caption: scatter-add of weight * dL/dy.
//
// The L2 atomic units of this chip retire about one atomic *request* per clock
// per XCD, where a request is whatever part of one wave instruction falls into
// one aligned 64-byte block; how many lanes it carries does not matter.  So the
// lanes are arranged to make requests fat: 2F consecutive lanes share one
// (point, level); lane (xbit, f) owns feature f of the lower or upper corner
// along dimension 0.  Those two corners are neighbours in memory (1:1 levels:
// index + 1; hashed levels: pi_1 = 1 keeps them in one small aligned block), so
// the 2F lanes of a group address 2F adjacent floats and mostly travel as one
// request instead of 2F.
template <int D, int F, typename IT>
__global__ __launch_bounds__(kBlock) void bwd_general(const LevelTable lv, const bool smooth, const uint32_t B,
                                                      const float* __restrict__ x, const IT* __restrict__ dy,
                                                      float* __restrict__ grad) {
  constexpr uint32_t G = 2 * F;  // lanes per (point, level)
  const uint32_t l = blockIdx.y;
  const uint32_t sub = threadIdx.x % G;
  const uint32_t xbit = sub / F, f = sub % F;
  const uint64_t b64 = (uint64_t)blockIdx.x * (kBlock / G) + threadIdx.x / G;
  if (b64 >= B) return;
  const uint32_t b = (uint32_t)b64;
  float xp[D];
  load_point<D>(x, b, xp);
  Corners<D> cn;
  corners_of<D, false>(lv, l, smooth, xp, cn, nullptr);
  const float g = (float)dy[((uint64_t)b * lv.L + l) * F + f];
  float* gl = grad + lv.offset[l] * F + f;
#pragma unroll
  for (uint32_t r = 0; r < (1u << (D - 1)); ++r) {  // corners along the other dimensions
    const uint32_t m0 = r << 1;
    const uint32_t idx = xbit ? cn.idx[m0 | 1u] : cn.idx[m0];
    const float wt = xbit ? cn.wt[m0 | 1u] : cn.wt[m0];
    __hip_atomic_fetch_add(gl + (uint64_t)idx * F, wt * g, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

// The same with half-precision gradients, accumulated with the packed two-half atomic as the paper
// does (Section 4; Fig. 5: efficient for pairs of features, not for single ones): a lane owns two
// neighbouring features of one corner, so F lanes share a (point, level) (2 lanes at F = 1, where
// each atomic carries one feature and a zero for the neighbouring entry).
template <int D, int F, typename IT>
__global__ __launch_bounds__(kBlock) void bwd_general_half(const LevelTable lv, const bool smooth, const uint32_t B,
                                                           const float* __restrict__ x, const IT* __restrict__ dy,
                                                           _Float16* __restrict__ grad) {
  constexpr uint32_t P = F >= 2 ? F / 2 : 1;  // feature pairs per entry
  constexpr uint32_t G = 2 * P;               // lanes per (point, level)
  const uint32_t l = blockIdx.y;
  const uint32_t sub = threadIdx.x % G;
  const uint32_t xbit = sub / P, fp = sub % P;
  const uint64_t b64 = (uint64_t)blockIdx.x * (kBlock / G) + threadIdx.x / G;
  if (b64 >= B) return;
  const uint32_t b = (uint32_t)b64;
  float xp[D];
  load_point<D>(x, b, xp);
  Corners<D> cn;
  corners_of<D, false>(lv, l, smooth, xp, cn, nullptr);
  const IT* gp = dy + ((uint64_t)b * lv.L + l) * F + 2 * fp;
  const float g0 = (float)gp[0], g1 = F >= 2 ? (float)gp[F >= 2 ? 1 : 0] : 0.0f;
  _Float16* gl = grad + lv.offset[l] * F;
#pragma unroll
  for (uint32_t r = 0; r < (1u << (D - 1)); ++r) {
    const uint32_t m0 = r << 1;
    const uint32_t idx = xbit ? cn.idx[m0 | 1u] : cn.idx[m0];
    const float wt = xbit ? cn.wt[m0 | 1u] : cn.wt[m0];
    if (F >= 2) grad_atomic_add2(gl, (uint64_t)idx * F + 2 * fp, wt * g0, wt * g1);  // (offset + idx) * F is even
    else grad_atomic_add(gl, (uint64_t)idx, wt * g0);
  }
}

// Gradient with respect to the position: one thread per point, all levels.
template <int D, int F, typename PT, typename IT>
__global__ __launch_bounds__(kBlock) void bwd_input_general(const LevelTable lv, const bool smooth, const uint32_t B,
                                                            const float* __restrict__ x,
                                                            const PT* __restrict__ theta,
                                                            const IT* __restrict__ dy, float* __restrict__ dx) {
  const uint32_t b = blockIdx.x * kBlock + threadIdx.x;
  if (b >= B) return;
  float xp[D];
  load_point<D>(x, b, xp);
  float gx[D];
#pragma unroll
  for (int j = 0; j < D; ++j) gx[j] = 0.0f;
  for (uint32_t l = 0; l < lv.L; ++l) {
    Corners<D> cn;
    float dwt[D][1 << D];
    corners_of<D, true>(lv, l, smooth, xp, cn, dwt);
    const Vec<PT, F>* tab = reinterpret_cast<const Vec<PT, F>*>(theta) + lv.offset[l];
    const Vec<IT, F> g = reinterpret_cast<const Vec<IT, F>*>(dy)[(uint64_t)b * lv.L + l];
#pragma unroll
    for (uint32_t m = 0; m < (1u << D); ++m) {
      const Vec<PT, F> e = tab[cn.idx[m]];
      float s = 0.0f;
#pragma unroll
      for (int f = 0; f < F; ++f) s = fmaf((float)g.v[f], (float)e.v[f], s);
#pragma unroll
      for (int j = 0; j < D; ++j) gx[j] = fmaf(dwt[j][m], s, gx[j]);
    }
  }
#pragma unroll
  for (int j = 0; j < D; ++j) dx[(uint64_t)b * D + j] = gx[j];
}

// The fp32 decisions of one level, for bit-exact comparison.
// Precondition check for callers: how many of the B * d coordinates are not in [0,1) (NaN and
// infinities included).  One atomic per wave that found any.
__global__ __launch_bounds__(kBlock) void count_outside_unit(const uint64_t n, const float* __restrict__ x,
                                                             uint32_t* __restrict__ count) {
  uint32_t bad = 0;
  for (uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (uint64_t)gridDim.x * kBlock) {
    const float v = x[i];
    bad += !(v >= 0.0f && v < 1.0f);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) bad += __shfl_xor(bad, o);
  if ((threadIdx.x & 63) == 0 && bad) atomicAdd(count, bad);
}

template <int D>
__global__ __launch_bounds__(kBlock) void indices_general(const LevelTable lv, const bool smooth, const uint32_t B,
                                                          const float* __restrict__ x, const uint32_t l,
                                                          uint32_t* __restrict__ idx, float* __restrict__ w) {
  const uint32_t b = blockIdx.x * kBlock + threadIdx.x;
  if (b >= B) return;
  float xp[D];
  load_point<D>(x, b, xp);
  Corners<D> cn;
  corners_of<D, false>(lv, l, smooth, xp, cn, nullptr);
  if (idx) {
#pragma unroll
    for (uint32_t m = 0; m < (1u << D); ++m) idx[(uint64_t)b * (1u << D) + m] = cn.idx[m];
  }
  if (w) {
    const float Nf = (float)lv.N[l];
#pragma unroll
    for (int i = 0; i < D; ++i) {
      uint32_t c0;
      float wf;
      split(xp[i], Nf, smooth ? 0.5f : 0.0f, smooth ? Nf : Nf - 1.0f, c0, wf);
      w[(uint64_t)b * D + i] = wf;
    }
  }
}

// ------------------------------------------------------------------ host side

// Eq. 2-3 in extended precision.  A level whose real-valued resolution is an
// integer (b^l landing on one, e.g. b = 2, and always level L-1 = N_max) keeps
// that integer: the progression is defined over [N_min, N_max] (Section 3).
static hg_status build_levels(const hashgrid_config& c, LevelTable& lv, uint64_t& total) {
  const long double log2_b =
      c.L > 1 ? (log2l((long double)c.N_max) - log2l((long double)c.N_min)) / (long double)(c.L - 1) : 0.0L;
  lv = LevelTable{};
  lv.L = c.L;
  lv.T = c.T;
  lv.T_is_pow2 = (c.T & (c.T - 1u)) == 0u;
  uint64_t off = 0;
  for (uint32_t l = 0; l < c.L; ++l) {
    const long double s = (long double)c.N_min * exp2l((long double)l * log2_b);
    const uint64_t N = (uint64_t)floorl(s + 1e-6L);
    if (N + 2u > 0xFFFFFFFFull) return HG_ERR_UNSUPPORTED;
    const uint64_t per_axis = N + 1u + (c.interp == HG_INTERP_SMOOTHSTEP ? 1u : 0u);
    uint64_t verts = 1;
    bool dense = true;
    for (uint32_t i = 0; i < c.d; ++i) {
      verts *= per_axis;
      if (verts > (uint64_t)c.T) { dense = false; break; }
    }
    lv.N[l] = (uint32_t)N;
    lv.verts[l] = (uint32_t)per_axis;
    lv.size[l] = dense ? (uint32_t)verts : c.T;
    lv.offset[l] = off;
    if (dense) lv.dense_mask |= 1u << l;
    off += lv.size[l];
  }
  total = off;
  return HG_OK;
}

static inline bool misaligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }
static inline size_t dtype_size(uint32_t t) { return t == HG_F16 ? 2 : 4; }
// alignment the entry points ask of an array of F-scalar entries: one entry, 16 bytes at most
static inline size_t entry_align(uint32_t F, uint32_t t) { return F * dtype_size(t) > 16 ? 16 : F * dtype_size(t); }

static hg_status launched() { return hipGetLastError() == hipSuccess ? HG_OK : HG_ERR_DEVICE; }

// Two points per thread once the batch needs two or more rounds of full workgroups per CU
static bool fwd_two_points_per_thread(uint32_t B) { return (uint64_t)B >= 2ull * kPmBlock * cu_count(); }

template <int D, int F, typename PT, typename IT>
static hg_status launch_fwd(const hashgrid* h, uint32_t B, const float* x, const void* params, void* y,
                            hipStream_t s) {
  {
    constexpr uint32_t G = OutPiece<F, IT>::kLevels;
    if (h->lv.L % G == 0 && !misaligned(y, 16) && !misaligned(params, F * sizeof(PT) > 16 ? 16 : F * sizeof(PT))) {
      const uint32_t block = point_major_block(B);
      const dim3 grid((B + block - 1) / block);
      const bool smooth = h->cfg.interp == HG_INTERP_SMOOTHSTEP;
      if (h->lv.T_is_pow2 && fwd_two_points_per_thread(B))
        hipLaunchKernelGGL((fwd_point_major<D, F, PT, IT, true, false, 2>), dim3((B + 2 * kPmBlock - 1) / (2 * kPmBlock)),
                           dim3(kPmBlock), 0, s, h->lv, smooth, B, x, static_cast<const PT*>(params),
                           static_cast<IT*>(y), NoCount{});
      else if (h->lv.T_is_pow2)
        hipLaunchKernelGGL((fwd_point_major<D, F, PT, IT, true, false>), grid, dim3(block), 0, s, h->lv, smooth, B,
                           x, static_cast<const PT*>(params), static_cast<IT*>(y), NoCount{});
      else
        hipLaunchKernelGGL((fwd_point_major<D, F, PT, IT, false, false>), grid, dim3(block), 0, s, h->lv, smooth,
                           B, x, static_cast<const PT*>(params), static_cast<IT*>(y), NoCount{});
      return launched();
    }
  }
  dim3 grid((B + kBlock - 1) / kBlock, h->lv.L);
  hipLaunchKernelGGL((fwd_general<D, F, PT, IT>), grid, dim3(kBlock), 0, s, h->lv,
                     h->cfg.interp == HG_INTERP_SMOOTHSTEP, B, x, static_cast<const PT*>(params),
                     static_cast<IT*>(y));
  return launched();
}

template <int D, int F, typename PT, typename IT>
static hg_status launch_bwd_input(const hashgrid* h, uint32_t B, const float* x, const void* params,
                                  const void* dy, float* dx, hipStream_t s) {
  {
    constexpr uint32_t G = OutPiece<F, IT>::kLevels;
    if (h->lv.L % G == 0 && !misaligned(dy, 16) && !misaligned(params, F * sizeof(PT) > 16 ? 16 : F * sizeof(PT))) {
      const uint32_t block = point_major_block(B);
      const dim3 pm_grid((B + block - 1) / block);
      const bool smooth = h->cfg.interp == HG_INTERP_SMOOTHSTEP;
      if (h->lv.T_is_pow2 && fwd_two_points_per_thread(B))
        hipLaunchKernelGGL((bwd_input_point_major<D, F, PT, IT, true, 2>),
                           dim3((B + 2 * kPmBlock - 1) / (2 * kPmBlock)), dim3(kPmBlock), 0, s, h->lv, smooth, B, x,
                           static_cast<const PT*>(params), static_cast<const IT*>(dy), dx);
      else if (h->lv.T_is_pow2)
        hipLaunchKernelGGL((bwd_input_point_major<D, F, PT, IT, true>), pm_grid, dim3(block), 0, s, h->lv, smooth,
                           B, x, static_cast<const PT*>(params), static_cast<const IT*>(dy), dx);
      else
        hipLaunchKernelGGL((bwd_input_point_major<D, F, PT, IT, false>), pm_grid, dim3(block), 0, s, h->lv, smooth,
                           B, x, static_cast<const PT*>(params), static_cast<const IT*>(dy), dx);
      return launched();
    }
  }
  dim3 grid((B + kBlock - 1) / kBlock);
  hipLaunchKernelGGL((bwd_input_general<D, F, PT, IT>), grid, dim3(kBlock), 0, s, h->lv,
                     h->cfg.interp == HG_INTERP_SMOOTHSTEP, B, x, static_cast<const PT*>(params),
                     static_cast<const IT*>(dy), dx);
  return launched();
}

template <int D, int F, typename IT>
static hg_status launch_bwd(const hashgrid* h, uint32_t B, const float* x, const void* dy, void* grad,
                            hipStream_t s) {
  const bool smooth = h->cfg.interp == HG_INTERP_SMOOTHSTEP;
  if (h->cfg.grad_dtype == HG_F16) {
    constexpr uint32_t per_block = kBlock / (F >= 2 ? F : 2);
    dim3 grid((uint32_t)(((uint64_t)B + per_block - 1) / per_block), h->lv.L);
    hipLaunchKernelGGL((bwd_general_half<D, F, IT>), grid, dim3(kBlock), 0, s, h->lv, smooth, B, x,
                       static_cast<const IT*>(dy), static_cast<_Float16*>(grad));
    return launched();
  }
  constexpr uint32_t per_block = kBlock / (2 * F);
  dim3 grid((uint32_t)(((uint64_t)B + per_block - 1) / per_block), h->lv.L);
  hipLaunchKernelGGL((bwd_general<D, F, IT>), grid, dim3(kBlock), 0, s, h->lv, smooth, B, x,
                     static_cast<const IT*>(dy), static_cast<float*>(grad));
  return launched();
}

// Forward pass that also fills counts[n_tiles][n_bins] for the binned backward pass (d = 2 or 3,
// power-of-two T: what that pass serves).  HG_ERR_UNSUPPORTED where the point-major kernel
// cannot run (misaligned y or tables, a row of y that is not a whole number of 16-byte pieces)
// or the histograms do not fit.
template <int D, int F, typename PT, typename IT>
static hg_status launch_fwd_counting_t(const hashgrid* h, uint32_t B, const float* x, const void* params, void* y,
                                       uint32_t* counts, uint32_t n_bins, uint32_t n_tiles, hipStream_t s) {
  constexpr uint32_t G = OutPiece<F, IT>::kLevels;
  const bool two = fwd_two_points_per_thread(B) && (size_t)(2 * kPmBlock / kBinThreads) * n_bins * 4 <= 64 * 1024;
  const size_t lds = (size_t)((two ? 2 : 1) * kPmBlock / kBinThreads) * n_bins * 4;
  if (h->lv.L % G != 0 || misaligned(y, 16) || misaligned(params, F * sizeof(PT) > 16 ? 16 : F * sizeof(PT)) ||
      !h->lv.T_is_pow2 || h->bp.corner_records || lds > kMaxCountingLds ||
      h->bp.tile_mult != 1)  // (its tiles are 512 points; it counts pairs of corners)
    return HG_ERR_UNSUPPORTED;
  if (lds > 64 * 1024) {  // more dynamic LDS than the default limit: opt in once per kernel
    static const hipError_t lds_ok =
        hipFuncSetAttribute(reinterpret_cast<const void*>(fwd_point_major<D, F, PT, IT, true, true>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMaxCountingLds);
    if (lds_ok != hipSuccess) return HG_ERR_DEVICE;
  }
  CountArgs ca;
  ca.bp = h->bp;
  ca.counts = counts;
  ca.n_bins = n_bins;
  ca.n_tiles = n_tiles;
  if (two)
    hipLaunchKernelGGL((fwd_point_major<D, F, PT, IT, true, true, 2>), dim3((B + 2 * kPmBlock - 1) / (2 * kPmBlock)),
                       dim3(kPmBlock), lds, s, h->lv, h->cfg.interp == HG_INTERP_SMOOTHSTEP, B, x,
                       static_cast<const PT*>(params), static_cast<IT*>(y), ca);
  else
    hipLaunchKernelGGL((fwd_point_major<D, F, PT, IT, true, true>), dim3((B + kPmBlock - 1) / kPmBlock), dim3(kPmBlock),
                       lds, s, h->lv, h->cfg.interp == HG_INTERP_SMOOTHSTEP, B, x, static_cast<const PT*>(params),
                       static_cast<IT*>(y), ca);
  return launched();
}

hg_status launch_fwd_counting(const hashgrid* h, uint32_t B, const float* x, const void* params, void* y,
                              uint32_t* counts, uint32_t n_bins, uint32_t n_tiles, hipStream_t s) {
  const hashgrid_config& c = h->cfg;
  const bool p16 = c.param_dtype == HG_F16, i16 = c.io_dtype == HG_F16;
#define HG_FWDC(D, F)                                                                                              \
  (p16 ? (i16 ? launch_fwd_counting_t<D, F, _Float16, _Float16>(h, B, x, params, y, counts, n_bins, n_tiles, s)    \
              : launch_fwd_counting_t<D, F, _Float16, float>(h, B, x, params, y, counts, n_bins, n_tiles, s))      \
       : (i16 ? launch_fwd_counting_t<D, F, float, _Float16>(h, B, x, params, y, counts, n_bins, n_tiles, s)       \
              : launch_fwd_counting_t<D, F, float, float>(h, B, x, params, y, counts, n_bins, n_tiles, s)))
  switch (c.d * 16 + c.F) {
    case 2 * 16 + 1: return HG_FWDC(2, 1);
    case 2 * 16 + 2: return HG_FWDC(2, 2);
    case 2 * 16 + 4: return HG_FWDC(2, 4);
    case 2 * 16 + 8: return HG_FWDC(2, 8);
    case 3 * 16 + 1: return HG_FWDC(3, 1);
    case 3 * 16 + 2: return HG_FWDC(3, 2);
    case 3 * 16 + 4: return HG_FWDC(3, 4);
    case 3 * 16 + 8: return HG_FWDC(3, 8);
    default: return HG_ERR_UNSUPPORTED;
  }
#undef HG_FWDC
}

// Expands `CALL(D, F)` for the runtime (d, F) pair.
#define HG_DISPATCH_DF(d, F, CALL)                       \
  switch ((d) * 16 + (F)) {                              \
    case 1 * 16 + 1: return CALL(1, 1);                  \
    case 1 * 16 + 2: return CALL(1, 2);                  \
    case 1 * 16 + 4: return CALL(1, 4);                  \
    case 1 * 16 + 8: return CALL(1, 8);                  \
    case 2 * 16 + 1: return CALL(2, 1);                  \
    case 2 * 16 + 2: return CALL(2, 2);                  \
    case 2 * 16 + 4: return CALL(2, 4);                  \
    case 2 * 16 + 8: return CALL(2, 8);                  \
    case 3 * 16 + 1: return CALL(3, 1);                  \
    case 3 * 16 + 2: return CALL(3, 2);                  \
    case 3 * 16 + 4: return CALL(3, 4);                  \
    case 3 * 16 + 8: return CALL(3, 8);                  \
    default: return HG_ERR_UNSUPPORTED;                  \
  }

}  // namespace hg

// ------------------------------------------------------------------ C ABI

extern "C" {

hg_status hashgrid_create(const hashgrid_config* cfg, hashgrid_t** out) {
  if (!cfg || !out) return HG_ERR_INVALID_ARG;
  const hashgrid_config& c = *cfg;
  if (c.d == 0 || c.L == 0 || c.F == 0 || c.T == 0 || c.N_min == 0 || c.N_max < c.N_min)
    return HG_ERR_INVALID_ARG;
  if (c.param_dtype > HG_F16 || c.io_dtype > HG_F16 || c.grad_dtype > HG_F16 || c.interp > HG_INTERP_SMOOTHSTEP)
    return HG_ERR_INVALID_ARG;
  if (c.d > 3 || c.L > HG_MAX_LEVELS) return HG_ERR_UNSUPPORTED;
  if (!(c.F == 1 || c.F == 2 || c.F == 4 || c.F == 8)) return HG_ERR_UNSUPPORTED;
  hashgrid* h = new (std::nothrow) hashgrid;
  if (!h) return HG_ERR_ALLOC;
  h->cfg = c;
  hg_status st = hg::build_levels(c, h->lv, h->total);
  if (st != HG_OK) {
    delete h;
    return st;
  }
  hg::build_bin_plan(h);
  *out = h;
  return HG_OK;
}

void hashgrid_destroy(hashgrid_t* hg) { delete hg; }

uint64_t hashgrid_n_entries(const hashgrid_t* hg) { return hg ? hg->total : 0; }

hg_status hashgrid_level_info(const hashgrid_t* hg, uint32_t l, uint32_t* N_l, uint64_t* entry_offset,
                              uint32_t* n_entries, int* is_dense) {
  if (!hg || l >= hg->lv.L) return HG_ERR_INVALID_ARG;
  if (N_l) *N_l = hg->lv.N[l];
  if (entry_offset) *entry_offset = hg->lv.offset[l];
  if (n_entries) *n_entries = hg->lv.size[l];
  if (is_dense) *is_dense = (int)((hg->lv.dense_mask >> l) & 1u);
  return HG_OK;
}

hg_status hashgrid_encode_fwd(const hashgrid_t* hg, uint32_t B, const float* x, const void* params, void* y,
                              void* stream) {
  if (!hg) return HG_ERR_INVALID_ARG;
  if (B == 0) return HG_OK;
  if (B > HG_MAX_BATCH) return HG_ERR_UNSUPPORTED;
  if (!x || !params || !y) return HG_ERR_INVALID_ARG;
  const hashgrid_config& c = hg->cfg;
  if (hg::misaligned(x, 4) || hg::misaligned(params, hg::entry_align(c.F, c.param_dtype)) ||
      hg::misaligned(y, hg::entry_align(c.F, c.io_dtype)))
    return HG_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const bool p16 = c.param_dtype == HG_F16, i16 = c.io_dtype == HG_F16;
#define HG_FWD(D, F)                                                                            \
  (p16 ? (i16 ? hg::launch_fwd<D, F, _Float16, _Float16>(hg, B, x, params, y, s)                \
              : hg::launch_fwd<D, F, _Float16, float>(hg, B, x, params, y, s))                  \
       : (i16 ? hg::launch_fwd<D, F, float, _Float16>(hg, B, x, params, y, s)                   \
              : hg::launch_fwd<D, F, float, float>(hg, B, x, params, y, s)))
  HG_DISPATCH_DF(c.d, c.F, HG_FWD)
#undef HG_FWD
}

hg_status hashgrid_encode_bwd(const hashgrid_t* hg, uint32_t B, const float* x, const void* dLdy,
                              void* grad_params, void* stream) {
  if (!hg) return HG_ERR_INVALID_ARG;
  if (B == 0) return HG_OK;
  if (B > HG_MAX_BATCH) return HG_ERR_UNSUPPORTED;
  if (!x || !dLdy || !grad_params) return HG_ERR_INVALID_ARG;
  const hashgrid_config& c = hg->cfg;
  if (hg::misaligned(x, 4) || hg::misaligned(dLdy, hg::entry_align(c.F, c.io_dtype)) ||
      hg::misaligned(grad_params, 4))
    return HG_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const bool i16 = c.io_dtype == HG_F16;
#define HG_BWD(D, F)                                                    \
  (i16 ? hg::launch_bwd<D, F, _Float16>(hg, B, x, dLdy, grad_params, s) \
       : hg::launch_bwd<D, F, float>(hg, B, x, dLdy, grad_params, s))
  HG_DISPATCH_DF(c.d, c.F, HG_BWD)
#undef HG_BWD
}

hg_status hashgrid_encode_bwd_input(const hashgrid_t* hg, uint32_t B, const float* x, const void* params,
                                    const void* dLdy, float* dLdx, void* stream) {
  if (!hg) return HG_ERR_INVALID_ARG;
  if (B == 0) return HG_OK;
  if (B > HG_MAX_BATCH) return HG_ERR_UNSUPPORTED;
  if (!x || !params || !dLdy || !dLdx) return HG_ERR_INVALID_ARG;
  const hashgrid_config& c = hg->cfg;
  if (hg::misaligned(x, 4) || hg::misaligned(dLdx, 4) ||
      hg::misaligned(params, hg::entry_align(c.F, c.param_dtype)) ||
      hg::misaligned(dLdy, hg::entry_align(c.F, c.io_dtype)))
    return HG_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const bool p16 = c.param_dtype == HG_F16, i16 = c.io_dtype == HG_F16;
#define HG_BWI(D, F)                                                                                    \
  (p16 ? (i16 ? hg::launch_bwd_input<D, F, _Float16, _Float16>(hg, B, x, params, dLdy, dLdx, s)         \
              : hg::launch_bwd_input<D, F, _Float16, float>(hg, B, x, params, dLdy, dLdx, s))           \
       : (i16 ? hg::launch_bwd_input<D, F, float, _Float16>(hg, B, x, params, dLdy, dLdx, s)            \
              : hg::launch_bwd_input<D, F, float, float>(hg, B, x, params, dLdy, dLdx, s)))
  HG_DISPATCH_DF(c.d, c.F, HG_BWI)
#undef HG_BWI
}

hg_status hashgrid_debug_indices(const hashgrid_t* hg, uint32_t B, const float* x, uint32_t level, uint32_t* idx,
                                 float* w, void* stream) {
  if (!hg || level >= hg->lv.L) return HG_ERR_INVALID_ARG;
  if (B == 0) return HG_OK;
  if (B > HG_MAX_BATCH) return HG_ERR_UNSUPPORTED;
  if (!x || hg::misaligned(x, 4) || hg::misaligned(idx, 4) || hg::misaligned(w, 4)) return HG_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const bool smooth = hg->cfg.interp == HG_INTERP_SMOOTHSTEP;
  dim3 grid((B + hg::kBlock - 1) / hg::kBlock);
  switch (hg->cfg.d) {
    case 1: hipLaunchKernelGGL((hg::indices_general<1>), grid, dim3(hg::kBlock), 0, s, hg->lv, smooth, B, x, level, idx, w); break;
    case 2: hipLaunchKernelGGL((hg::indices_general<2>), grid, dim3(hg::kBlock), 0, s, hg->lv, smooth, B, x, level, idx, w); break;
    case 3: hipLaunchKernelGGL((hg::indices_general<3>), grid, dim3(hg::kBlock), 0, s, hg->lv, smooth, B, x, level, idx, w); break;
    default: return HG_ERR_UNSUPPORTED;
  }
  return hg::launched();
}

hg_status hashgrid_debug_count_outside(const hashgrid_t* hg, uint32_t B, const float* x, uint32_t* count,
                                       void* stream) {
  if (!hg || !count || hg::misaligned(count, 4)) return HG_ERR_INVALID_ARG;
  if (B == 0) return HG_OK;
  if (B > HG_MAX_BATCH) return HG_ERR_UNSUPPORTED;
  if (!x || hg::misaligned(x, 4)) return HG_ERR_INVALID_ARG;
  const uint64_t n = (uint64_t)B * hg->cfg.d;
  const uint64_t wgs = (n + hg::kBlock - 1) / hg::kBlock;
  hipLaunchKernelGGL(hg::count_outside_unit, dim3((uint32_t)(wgs < 4096 ? wgs : 4096)), dim3(hg::kBlock), 0,
                     static_cast<hipStream_t>(stream), n, x, count);
  return hg::launched();
}

const char* hashgrid_strerror(hg_status s) {
  switch (s) {
    case HG_OK: return "ok";
    case HG_ERR_INVALID_ARG: return "invalid argument";
    case HG_ERR_UNSUPPORTED: return "unsupported configuration";
    case HG_ERR_ALLOC: return "host allocation failed";
    case HG_ERR_DEVICE: return "HIP launch failed";
  }
  return "unknown status";
}

}  // extern "C"
