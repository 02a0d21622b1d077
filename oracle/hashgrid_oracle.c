/*
 * CPU oracle for the multiresolution hash encoding (paper Section 3, Eq. 2-4,
 * Fig. 3; Appendix A for the smoothstep variant).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, step-by-step transcription
 * of what the method computes, written to be checked against the paper by eye.
 * Only the test-suite, the smoke check and the benchmark's CPU-baseline leg may
 * call it.  It shares no code, header, table or constant with the GPU library.
 *
 * Arithmetic:
 *   - the level table (Eq. 2-3) is evaluated in fp64 on the host;
 *   - the scale / floor / fractional-weight step (Section 3, "rounding down and
 *     up", and the definition of the interpolation weight w_l) is evaluated in
 *     IEEE fp32, one rounded multiply per coordinate, because that step decides
 *     integers (voxel corners) and both sides must take the decision in the same
 *     precision;
 *   - everything after that (corner weights, products with table entries, sums,
 *     the backward accumulation) is fp64.  Table entries and upstream gradients
 *     arrive as fp64 (the caller widens fp16 / fp32 exactly).
 *
 * Readings of the paper where it leaves a choice (each also listed in the
 * design notes of the repository):
 *   - Eq. 2 is evaluated as floor(N_min * exp(l * (ln N_max - ln N_min)/(L-1)) + 1e-6):
 *     the geometric progression runs over [N_min, N_max] (Section 3), so level
 *     L-1 is N_max and levels whose real value is an exact integer keep it even
 *     when fp64 exp lands a few ulp below.
 *   - the upper corner of the voxel is floor(p)+1 in every case (when p is an
 *     integer ceil(p)=floor(p) would collapse the voxel; its weight is 0 there).
 *   - the 1:1 map on coarse levels ((N_l+1)^d <= T) is
 *     v_0 + v_1 (N_l+1) + v_2 (N_l+1)^2, dimension 0 fastest, in line with
 *     pi_1 = 1 in Eq. 4; such a level has exactly (N_l+1)^d entries, a hashed
 *     level exactly T.
 *   - Eq. 4 is evaluated in 32-bit unsigned wrap-around arithmetic.
 *   - colliding gradients are summed (Fig. 3 caption: "accumulated").
 *   - Appendix A (interp = 1): the smoothstep S(w) = w^2 (3 - 2w) replaces w in
 *     the corner weights and each level is shifted by half a voxel: the scaled
 *     position is x * N_l + 0.5 (fp32 multiply then fp32 add).  Corner
 *     coordinates then reach N_l + 1, so the shifted grid has N_l + 2 vertices
 *     per axis; to keep the coarse-level map 1:1 the dense criterion and the
 *     dense stride use N_l + 2 in place of N_l + 1 for this variant.  (The
 *     appendix does not say how the shifted grid is indexed; this is the
 *     reading taken here.  The smoothstep weights and their derivative are
 *     pinned by closed forms, and what this reading computes is pinned too
 *     (vertex exactness at x = (k - 1/2)/N_l, the map being one-to-one onto
 *     (N_l+2)^d entries, every corner's entry against the formula in integers).
 *     That the paper means this map and not another 1:1 map of the shifted grid
 *     is a choice nothing in the paper fixes: parity unpinned for that choice
 *     only.)
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define HGO_MAX_LEVELS 64
#define HGO_MAX_D 3

typedef struct {
  uint32_t d;      /* input dimensions, 1..3 (Eq. 4 names three primes)   */
  uint32_t L;      /* number of levels                                      */
  uint32_t F;      /* features per entry                                    */
  uint32_t T;      /* maximum entries per level                             */
  uint32_t N_min;  /* coarsest resolution                                   */
  uint32_t N_max;  /* finest resolution                                     */
  uint32_t interp; /* 0 = d-linear (Section 3), 1 = smoothstep (Appendix A) */
} hgo_config;

typedef struct {
  uint32_t N[HGO_MAX_LEVELS];      /* N_l, Eq. 2                                  */
  uint32_t verts[HGO_MAX_LEVELS];  /* grid vertices per axis: N_l+1 (N_l+2 shifted) */
  uint64_t offset[HGO_MAX_LEVELS]; /* first entry of level l in the concatenation */
  uint32_t size[HGO_MAX_LEVELS];   /* entries of level l                          */
  int32_t dense[HGO_MAX_LEVELS];   /* 1 when verts^d <= T                         */
  uint64_t total;                  /* sum of size[]                               */
} hgo_levels_t;

/* Eq. 4: pi_1 = 1, pi_2 = 2654435761, pi_3 = 805459861 */
static const uint32_t HGO_PI[HGO_MAX_D] = {1u, 2654435761u, 805459861u};

int hgo_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Threads the following calls may use (timing on one core next to all cores); no effect on results. */
void hgo_set_num_threads(int n) {
#ifdef _OPENMP
  if (n >= 1) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

/* Eq. 2-3 and the dense criterion of Section 3.  Returns 0, or -1 on a bad config. */
int hgo_levels(const hgo_config* c, hgo_levels_t* out) {
  if (!c || !out) return -1;
  if (c->d < 1 || c->d > HGO_MAX_D || c->L < 1 || c->L > HGO_MAX_LEVELS || c->F < 1 || c->T < 1 ||
      c->N_min < 1 || c->N_max < c->N_min || c->interp > 1)
    return -1;
  double log_b = 0.0; /* ln b, Eq. 3 */
  if (c->L > 1) log_b = (log((double)c->N_max) - log((double)c->N_min)) / (double)(c->L - 1);
  uint64_t off = 0;
  for (uint32_t l = 0; l < c->L; ++l) {
    double s = (double)c->N_min * exp((double)l * log_b); /* N_min * b^l */
    uint32_t N = (uint32_t)floor(s + 1e-6);               /* Eq. 2       */
    uint32_t per_axis = N + 1u + (c->interp == 1 ? 1u : 0u);
    uint64_t verts = 1;                                   /* (N_l+1)^d   */
    for (uint32_t i = 0; i < c->d; ++i) {
      verts *= (uint64_t)per_axis;
      if (verts > (uint64_t)c->T) { verts = (uint64_t)c->T + 1u; break; }
    }
    out->N[l] = N;
    out->verts[l] = per_axis;
    out->dense[l] = verts <= (uint64_t)c->T;
    out->size[l] = out->dense[l] ? (uint32_t)verts : c->T;
    out->offset[l] = off;
    off += out->size[l];
  }
  out->total = off;
  return 0;
}

/* Entry of a level's array for the integer vertex v (Section 3: 1:1 map on
 * coarse levels, Eq. 4 otherwise).  `verts` is the number of grid vertices per
 * axis of a dense level (N_l + 1 for the d-linear encoding). */
uint32_t hgo_index(uint32_t d, uint32_t verts, uint32_t T, int dense, const uint32_t* v) {
  if (dense) {
    uint64_t idx = 0, stride = 1;
    for (uint32_t i = 0; i < d; ++i) {
      idx += (uint64_t)v[i] * stride;
      stride *= (uint64_t)verts;
    }
    return (uint32_t)idx;
  }
  uint32_t h = 0;
  for (uint32_t i = 0; i < d; ++i) h ^= v[i] * HGO_PI[i]; /* 32-bit wrap-around */
  return h % T;
}

/* Scale one coordinate to level resolution N, split into voxel corner and
 * fractional position, all in fp32 (one rounded multiply; the subtraction of
 * the floor is exact).  interp = 1 adds the half-voxel shift of Appendix A. */
static void hgo_split(float x, uint32_t N, uint32_t interp, uint32_t* c0, float* w) {
  volatile float p = x * (float)N; /* volatile: keep the product rounded to fp32 */
  if (interp == 1) {
    volatile float q = p + 0.5f;
    p = q;
  }
  float fl = floorf(p);
  *c0 = (uint32_t)fl;
  *w = p - fl;
}

static double hgo_smooth(double w) { return w * w * (3.0 - 2.0 * w); }   /* Appendix A, S   */
static double hgo_dsmooth(double w) { return 6.0 * w * (1.0 - w); }      /* Appendix A, S'  */

/* Per point and level: the 2^d entry indices and their interpolation weights.
 * dweight[j][m], when asked for, is d(weight_m)/d(x_j) (chain rule on the
 * weight definition of Section 3; factor N_l from the scaling). */
static void hgo_corners(const hgo_config* c, const hgo_levels_t* lv, uint32_t l, const float* x,
                        uint32_t* idx, double* weight, double (*dweight)[1 << HGO_MAX_D]) {
  uint32_t c0[HGO_MAX_D];
  double w[HGO_MAX_D], dw[HGO_MAX_D];
  for (uint32_t i = 0; i < c->d; ++i) {
    float wf;
    hgo_split(x[i], lv->N[l], c->interp, &c0[i], &wf);
    if (c->interp == 1) {
      w[i] = hgo_smooth((double)wf);
      dw[i] = hgo_dsmooth((double)wf) * (double)lv->N[l];
    } else {
      w[i] = (double)wf;
      dw[i] = (double)lv->N[l];
    }
  }
  for (uint32_t m = 0; m < (1u << c->d); ++m) {
    uint32_t v[HGO_MAX_D];
    double wt = 1.0;
    for (uint32_t i = 0; i < c->d; ++i) {
      uint32_t bit = (m >> i) & 1u;
      v[i] = c0[i] + bit;
      wt *= bit ? w[i] : 1.0 - w[i];
    }
    idx[m] = hgo_index(c->d, lv->verts[l], c->T, lv->dense[l], v);
    weight[m] = wt;
    if (dweight) {
      for (uint32_t j = 0; j < c->d; ++j) {
        double g = ((m >> j) & 1u) ? dw[j] : -dw[j];
        for (uint32_t i = 0; i < c->d; ++i) {
          if (i == j) continue;
          g *= ((m >> i) & 1u) ? w[i] : 1.0 - w[i];
        }
        dweight[j][m] = g;
      }
    }
  }
}

/* Returns 0 when every coordinate is finite and in [0,1), else 1 + index of the
 * first offending scalar.  The encoding is defined on the unit cube only. */
uint64_t hgo_check_x(uint64_t n_scalars, const float* x) {
  for (uint64_t i = 0; i < n_scalars; ++i)
    if (!(x[i] >= 0.0f && x[i] < 1.0f)) return i + 1;
  return 0;
}

/* Forward (Section 3, Fig. 3 steps 1-4): y[b, l*F + f] = sum_m weight_m * theta_l[idx_m][f]. */
int hgo_fwd(const hgo_config* c, uint64_t B, const float* x, const double* theta, double* y) {
  hgo_levels_t lv;
  if (hgo_levels(c, &lv)) return -1;
  if (hgo_check_x(B * c->d, x)) return -2;
  const uint32_t d = c->d, F = c->F, L = c->L;
#pragma omp parallel for schedule(static)
  for (int64_t b = 0; b < (int64_t)B; ++b) {
    for (uint32_t l = 0; l < L; ++l) {
      uint32_t idx[1 << HGO_MAX_D];
      double wt[1 << HGO_MAX_D];
      hgo_corners(c, &lv, l, x + (uint64_t)b * d, idx, wt, NULL);
      for (uint32_t f = 0; f < F; ++f) {
        double acc = 0.0;
        for (uint32_t m = 0; m < (1u << d); ++m)
          acc += wt[m] * theta[(lv.offset[l] + idx[m]) * F + f];
        y[((uint64_t)b * L + l) * F + f] = acc;
      }
    }
  }
  return 0;
}

/* Backward to the tables (Fig. 3 caption): dtheta_l[idx_m][f] += weight_m * dy[b, l*F+f].
 * Levels are independent arrays, so the level loop is the parallel one and each
 * entry is summed in point order. */
int hgo_bwd(const hgo_config* c, uint64_t B, const float* x, const double* dy, double* dtheta) {
  hgo_levels_t lv;
  if (hgo_levels(c, &lv)) return -1;
  if (hgo_check_x(B * c->d, x)) return -2;
  const uint32_t d = c->d, F = c->F, L = c->L;
#pragma omp parallel for schedule(dynamic, 1)
  for (int32_t l = 0; l < (int32_t)L; ++l) {
    for (uint64_t b = 0; b < B; ++b) {
      uint32_t idx[1 << HGO_MAX_D];
      double wt[1 << HGO_MAX_D];
      hgo_corners(c, &lv, (uint32_t)l, x + b * d, idx, wt, NULL);
      for (uint32_t m = 0; m < (1u << d); ++m)
        for (uint32_t f = 0; f < F; ++f)
          dtheta[(lv.offset[l] + idx[m]) * F + f] += wt[m] * dy[(b * L + l) * F + f];
    }
  }
  return 0;
}

/* Gradient with respect to the input position:
 * dx[b, j] = sum_{l,f} dy[b, l*F+f] * sum_m d(weight_m)/d(x_j) * theta_l[idx_m][f]. */
int hgo_bwd_input(const hgo_config* c, uint64_t B, const float* x, const double* theta, const double* dy,
                  double* dx) {
  hgo_levels_t lv;
  if (hgo_levels(c, &lv)) return -1;
  if (hgo_check_x(B * c->d, x)) return -2;
  const uint32_t d = c->d, F = c->F, L = c->L;
#pragma omp parallel for schedule(static)
  for (int64_t b = 0; b < (int64_t)B; ++b) {
    double g[HGO_MAX_D] = {0.0, 0.0, 0.0};
    for (uint32_t l = 0; l < L; ++l) {
      uint32_t idx[1 << HGO_MAX_D];
      double wt[1 << HGO_MAX_D];
      double dwt[HGO_MAX_D][1 << HGO_MAX_D];
      hgo_corners(c, &lv, l, x + (uint64_t)b * d, idx, wt, dwt);
      for (uint32_t f = 0; f < F; ++f) {
        double up = dy[((uint64_t)b * L + l) * F + f];
        for (uint32_t j = 0; j < d; ++j) {
          double s = 0.0;
          for (uint32_t m = 0; m < (1u << d); ++m) s += dwt[j][m] * theta[(lv.offset[l] + idx[m]) * F + f];
          g[j] += up * s;
        }
      }
    }
    for (uint32_t j = 0; j < d; ++j) dx[(uint64_t)b * d + j] = g[j];
  }
  return 0;
}

/* The decisions taken in fp32 for one level: level-local entry indices [B, 2^d]
 * (corner m has bit i set when it is the upper corner along dimension i) and
 * the fractional positions w [B, d] before any smoothstep. */
int hgo_indices(const hgo_config* c, uint64_t B, const float* x, uint32_t l, uint32_t* idx, float* w) {
  hgo_levels_t lv;
  if (hgo_levels(c, &lv)) return -1;
  if (l >= c->L) return -1;
  if (hgo_check_x(B * c->d, x)) return -2;
  const uint32_t d = c->d;
  for (uint64_t b = 0; b < B; ++b) {
    /* the entries are the ones the forward and backward passes use: same routine */
    double wt[1 << HGO_MAX_D];
    hgo_corners(c, &lv, l, x + b * d, idx + b * (1u << d), wt, NULL);
    for (uint32_t i = 0; i < d; ++i) {
      uint32_t c0;
      hgo_split(x[b * d + i], lv.N[l], c->interp, &c0, &w[b * d + i]);
    }
  }
  return 0;
}

/* ---------------------------------------------------------------------------
 * Optimiser step on the tables (paper Section 4, "Training"): Adam (Kingma & Ba,
 * Algorithm 1, with bias correction) with beta1, beta2, eps as given by the
 * caller (the paper uses 0.9, 0.99, 1e-15), the paper's L2 regularisation (factor
 * l2: 1e-6 for the network's weights, 0 for table entries; read as the term
 * l2 * theta added to the gradient, the gradient of (l2 / 2) |theta|^2), and the
 * paper's rule that an entry whose gradient is exactly 0 is skipped: its moments
 * and its value are left untouched (with a regulariser: whose gradient
 * including that term is 0).
 *
 * Readings where the paper is silent: `step` (1-based) is one global counter
 * used for the bias corrections of every entry, skipped or not; "entry" is taken
 * per scalar (each of the F features of a table entry decides on its own
 * gradient).  All arithmetic fp64; theta is the full-precision master copy
 * (Section 4, "Performance considerations": the half-precision table is derived
 * from it by rounding, which the caller does).
 */
int hgo_adam_step(uint64_t n, double* theta, const double* grad, double* m, double* v, double lr, double beta1,
                  double beta2, double eps, double l2, uint32_t step) {
  if (!theta || !grad || !m || !v || step == 0) return -1;
  const double c1 = 1.0 - pow(beta1, (double)step); /* bias corrections */
  const double c2 = 1.0 - pow(beta2, (double)step);
  for (uint64_t i = 0; i < n; ++i) {
    const double g = grad[i] + l2 * theta[i];
    if (g == 0.0) continue; /* skipped entry */
    m[i] = beta1 * m[i] + (1.0 - beta1) * g;
    v[i] = beta2 * v[i] + (1.0 - beta2) * g * g;
    const double m_hat = m[i] / c1, v_hat = v[i] / c2;
    theta[i] -= lr * m_hat / (sqrt(v_hat) + eps);
  }
  return 0;
}
