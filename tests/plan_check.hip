// Host-side check of the plan of the sorted backward pass (no GPU): for every point, level and
// pair of corners along dimension 0 (or every corner, in plans that give each corner its own record), what rows_of hands to the count / scatter kernels must name,
// under the record's rules, exactly the two table entries that Section 3 / Eq. 4 of the paper give,
// inside the bounds the kernels rely on.  Compiled for the host only and linked against
// libhashgrid.so (for hashgrid_create, which builds the level table and the plan).
#include <stdint.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

#include "hashgrid.h"
#include "hashgrid_common.hpp"
#include "hashgrid_internal.hpp"
#include "bwd_bins.hpp"

namespace {

// with HG_PLAN_VERBOSE set, the first violations are printed with the line that found them
#define VIOLATION()                                                                                   \
  do {                                                                                                \
    if (bad < 10 && getenv("HG_PLAN_VERBOSE"))                                                        \
      fprintf(stderr, "plan_check line %d: point %u level %u x0 %.9g\n", __LINE__, b, l, (double)xp[0]); \
    ++bad;                                                                                            \
  } while (0)

// entry index of a vertex, written out from Section 3 (1:1) and Eq. 4 (hashed)
template <int D>
uint32_t entry_of(const hg::LevelTable& lv, uint32_t l, const uint32_t (&v)[D]) {
  if ((lv.dense_mask >> l) & 1u) {
    uint64_t idx = 0, stride = 1;
    for (int i = 0; i < D; ++i) {
      idx += v[i] * stride;
      stride *= lv.verts[l];
    }
    return (uint32_t)idx;
  }
  const uint32_t primes[3] = {1u, 2654435761u, 805459861u};
  uint32_t h = 0;
  for (int i = 0; i < D; ++i) h ^= v[i] * primes[i];
  return h % lv.T;
}

template <int D>
uint64_t check(const hashgrid* h, uint32_t B, const float* x, uint64_t* crossing) {
  const hg::LevelTable& lv = h->lv;
  const hg::BinPlan& bp = h->bp;
  const bool smooth = h->cfg.interp == HG_INTERP_SMOOTHSTEP;
  const uint32_t cl = bp.chunk_log2, cap = 1u << cl;
  uint64_t bad = 0;
  for (uint32_t b = 0; b < B; ++b) {
    float xp[D];
    for (int i = 0; i < D; ++i) xp[i] = x[(uint64_t)b * D + i];
    for (uint32_t l = 0; l < lv.L; ++l) {
      const bool dense = (lv.dense_mask >> l) & 1u;
      hg::Rows<D> rw, rc;
      hg::rows_of<D, false>(lv, bp, l, smooth, xp, rw);
      hg::rows_of<D, true>(lv, bp, l, smooth, xp, rc);  // what the count pass sees
      // the voxel, independently: one rounded multiply, optional half-voxel shift, floor
      uint32_t c0[D];
      for (int i = 0; i < D; ++i) {
        float p = xp[i] * (float)lv.N[l];
        if (smooth) p = p + 0.5f;
        c0[i] = (uint32_t)floorf(p);
      }
      if (rw.cross != rc.cross) VIOLATION();
      if (rw.cross) {
        ++*crossing;
        if (dense) VIOLATION();
      }
      if (!(rw.wf0 >= 0.0f && rw.wf0 < 1.0f) || rw.k > 15u) VIOLATION();
      if ((rw.k == 15u) != (c0[0] == 0u)) VIOLATION();
      // from the second voxel on the fraction is a multiple of 2^-23: the record keeps it exactly
      if (c0[0] != 0u && rw.wf0 * 0x1p23f != floorf(rw.wf0 * 0x1p23f)) VIOLATION();
      float wsum = 0.0f;
      for (uint32_t r = 0; r < (1u << (D - 1)); ++r) {
        uint32_t va[D], vb[D];
        va[0] = c0[0];
        vb[0] = c0[0] + 1u;
        for (int i = 1; i < D; ++i) va[i] = vb[i] = c0[i] + ((r >> (i - 1)) & 1u);
        const uint32_t ia = entry_of<D>(lv, l, va), ib = entry_of<D>(lv, l, vb);
        if (rw.bin[r] != rc.bin[r]) VIOLATION();
        if (rw.bin[r] < bp.bin_base[l] || rw.bin[r] >= bp.bin_base[l + 1]) {
          VIOLATION();
          continue;
        }
        const uint32_t bin = rw.bin[r] - bp.bin_base[l];
        // the chunk this bin stands for, as the accumulate pass lays it out
        uint64_t e0, e1;
        if (dense) {
          e0 = ((uint64_t)bin << bp.row_shift[l]) * lv.verts[l];
          e1 = e0 + ((uint64_t)lv.verts[l] << bp.row_shift[l]);
        } else {
          e0 = (uint64_t)bin << cl;
          e1 = e0 + cap;
        }
        if (e1 > lv.size[l]) e1 = lv.size[l];
        const uint32_t n_e = (uint32_t)(e1 - e0);
        if (n_e == 0 || n_e > cap) VIOLATION();
        if (rw.la[r] >= n_e || rw.la[r] >= 4096u || e0 + rw.la[r] != ia) VIOLATION();
        if (!rw.cross) {
          const uint32_t k = rw.k == 15u ? 0u : rw.k;  // the record's rule: 15 marks the first voxel, whose coordinate 0 has no trailing ones
          const uint32_t lb = dense ? rw.la[r] + 1u : rw.la[r] ^ (((2u << k) - 1u) & (n_e - 1u));
          if (lb >= n_e || e0 + lb != ib) VIOLATION();
        }
        // (a pair flagged as straddling is added with atomics instead of a record: always correct, so
        // the flag may be raised needlessly, as it is for tables of a single chunk; what matters is
        // that it is never missing, which the branch above checks)
        if (!(rw.wrow[r] >= 0.0f && rw.wrow[r] <= 1.0f)) VIOLATION();
        wsum += rw.wrow[r];
      }
      if (fabsf(wsum - 1.0f) > 1e-5f) VIOLATION();  // the rows' weights are a partition of unity
    }
  }
  return bad;
}

// Plans with one record per corner (BinPlan::corner_records): every corner's bin and chunk-local index
// must name the entry of Section 3 / Eq. 4, chunks being aligned blocks of the level's slice, and the
// corners' weights must be the interpolation weights (a partition of unity).
template <int D>
uint64_t check_corners(const hashgrid* h, uint32_t B, const float* x) {
  const hg::LevelTable& lv = h->lv;
  const hg::BinPlan& bp = h->bp;
  const bool smooth = h->cfg.interp == HG_INTERP_SMOOTHSTEP;
  const uint32_t cl = bp.chunk_log2, cap = 1u << cl;
  uint64_t bad = 0;
  for (uint32_t b = 0; b < B; ++b) {
    float xp[D];
    for (int i = 0; i < D; ++i) xp[i] = x[(uint64_t)b * D + i];
    for (uint32_t l = 0; l < lv.L; ++l) {
      hg::CornerRows<D> cr, cc;
      hg::corner_rows_of<D, false>(lv, bp, l, smooth, xp, cr);
      hg::corner_rows_of<D, true>(lv, bp, l, smooth, xp, cc);  // what the count pass sees
      uint32_t c0[D];
      double w[D];
      for (int i = 0; i < D; ++i) {
        float p = xp[i] * (float)lv.N[l];
        if (smooth) p = p + 0.5f;
        c0[i] = (uint32_t)floorf(p);
        const double f = (double)(p - floorf(p));
        w[i] = smooth ? f * f * (3.0 - 2.0 * f) : f;
      }
      float wsum = 0.0f;
      for (uint32_t m = 0; m < (1u << D); ++m) {
        uint32_t v[D];
        double wt = 1.0;
        for (int i = 0; i < D; ++i) {
          v[i] = c0[i] + ((m >> i) & 1u);
          wt *= ((m >> i) & 1u) ? w[i] : 1.0 - w[i];
        }
        const uint32_t ie = entry_of<D>(lv, l, v);
        if (cr.bin[m] != cc.bin[m]) VIOLATION();
        if (cr.bin[m] < bp.bin_base[l] || cr.bin[m] >= bp.bin_base[l + 1]) {
          VIOLATION();
          continue;
        }
        const uint64_t e0 = (uint64_t)(cr.bin[m] - bp.bin_base[l]) << cl;
        const uint64_t e1 = e0 + cap < lv.size[l] ? e0 + cap : lv.size[l];
        if (e0 >= e1 || cr.la[m] >= e1 - e0 || cr.la[m] >= 4096u || e0 + cr.la[m] != ie) VIOLATION();
        if (fabs((double)cr.weight[m] - wt) > 1e-6) VIOLATION();
        wsum += cr.weight[m];
      }
      if (fabsf(wsum - 1.0f) > 1e-5f) VIOLATION();
    }
  }
  return bad;
}

}  // namespace

// Number of violated invariants over B points (host pointer, [B, d] floats in [0,1)); *crossing counts
// the (point, level) pairs whose corners straddle two chunks.  UINT64_MAX when the configuration
// is not served by the sorted pass or cannot be created.
extern "C" uint64_t plan_check(const hashgrid_config* cfg, uint32_t B, const float* x, uint64_t* crossing) {
  hashgrid_t* h = nullptr;
  *crossing = 0;
  if (hashgrid_create(cfg, &h) != HG_OK) return UINT64_MAX;
  uint64_t bad = UINT64_MAX;
  if (h->bp.supported && h->bp.corner_records)
    bad = cfg->d == 3 ? check_corners<3>(h, B, x) : cfg->d == 2 ? check_corners<2>(h, B, x) : check_corners<1>(h, B, x);
  else if (h->bp.supported)
    bad = cfg->d == 3 ? check<3>(h, B, x, crossing) : check<2>(h, B, x, crossing);
  hashgrid_destroy(h);
  return bad;
}

// spread_in_run over every run length the scatter pass can see (a tile's records for one bin:
// at most 2^d * 512): number of run lengths for which it is not a bijection of [0, n), or puts
// two records that follow each other fewer than 64 slots apart in a run of 128 or more
// (cyclically: k * s mod n steps by s or s - n).
extern "C" uint32_t spread_check(uint32_t n_max) {
  uint32_t bad = 0;
  unsigned char* seen = (unsigned char*)malloc(n_max + 1);
  for (uint32_t n = 1; n <= n_max; ++n) {
    for (uint32_t i = 0; i < n; ++i) seen[i] = 0;
    bool ok = true;
    uint32_t prev = 0;
    for (uint32_t k = 0; k < n && ok; ++k) {
      const uint32_t p = hg::spread_in_run(k, n);
      if (p >= n || seen[p]) ok = false;
      else seen[p] = 1;
      if (ok && n >= 192 && k > 0) {
        const uint32_t dist = p > prev ? p - prev : prev - p;
        if (dist < 64) ok = false;
      }
      prev = p;
    }
    if (hg::spread_in_run(n, n) != n || hg::spread_in_run(n + 5, n) != n + 5) ok = false;  // out of range: left alone
    bad += ok ? 0 : 1;
  }
  free(seen);
  return bad;
}
