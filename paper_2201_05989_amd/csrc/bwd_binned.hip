// Binned backward pass of the hash encoding (Fig. 3 caption of the paper: the
// gradient of the loss is accumulated in the looked-up feature vectors).
//
// Why not atomics: on this chip a device-scope fp32 atomic add costs one L2
// request per 64-byte block per wave instruction and all XCDs together retire
// about 21 G requests/s, whatever the table size; a fine hashed level needs at
// least 2^(d-1) requests per point, which bounds an atomic backward pass far
// below what the memory system can stream.  LDS fp32 atomics are slow as well
// (about 0.3 lane-ops per clock per CU) while LDS *integer* atomics run at about
// 3.6 64-bit adds per clock per CU.  So the scatter-add is done as a bucket
// sort followed by an owner-computes accumulation:
//
//   count      every (point, level) emits 2^(d-1) records, one per pair of
//              corners that differ only along dimension 0 (they are neighbours
//              in memory: index+1 on 1:1 levels, same small aligned block on
//              hashed levels because pi_1 = 1 in Eq. 4).  A record belongs to
//              the bin (chunk of the level's gradient slice, at most 2^chunk_log2
//              entries) that holds both corners.  This kernel only counts.
//   scan       per-bin totals and per-(workgroup, bin) write offsets.
//   scatter    recomputes the records, sorts them by bin in LDS one level at a
//              time and writes each to its slot.  A record names the two
//              chunk-local entries and carries the fractional position along
//              dimension 0, the weight of the other dimensions and dL/dy of the
//              level: 16 bytes when dL/dy is fp32, 12 bytes when it is fp16
//              (see Record below).  The passes that write and re-read the
//              records are bound by memory bandwidth, so the record size is
//              what sets their time.
//   accumulate one workgroup per bin (several for the few bins of coarse 1:1
//              levels, which receive very many records): sums its records into
//              LDS in 64-bit fixed point with integer atomics, then adds the
//              chunk to the fp32 gradient (plain read-modify-write when the bin
//              has a single owner).  The fixed-point scale comes from the
//              largest |dL/dy| of the call, with headroom for 8*B summands, so
//              the sum is exact and independent of the order of the records;
//              each summand is rounded once to 2^-min(62-H, 51) of the power of
//              two above that largest value (H = ceil(log2(8B))).
//
// Variants of the same plan: the forward pass can do the counting (hashgrid.hip,
// HG_BWD_COUNTED); plans with more than kMaxStagedBins chunks use tiles of
// kBigTileMult * 512 points and write their records unstaged (bin_scatter_direct);
// pairs whose corners lie in two chunks (hashed levels of resolution 2^chunk_log2
// or more) bypass the sort and are added with device atomics; with
// HG_BWD_OVERWRITE the owners store their sums instead of adding them, the scan
// kernel clears the levels that several workgroups share, and the atomics for the
// straddling pairs run as a last pass (bin_crossing).
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <atomic>
#include <type_traits>

#include "hashgrid.h"
#include "hashgrid_common.hpp"
#include "hashgrid_internal.hpp"
#include "bwd_bins.hpp"
#include "bwd_record.hpp"

namespace hg {

// Launch shapes, each the best of a sweep on the headline configuration.
constexpr int kScanThreads = 1024;
constexpr int kAccThreads = 1024;                // accumulate workgroup (512 x 2 per CU is slower)
constexpr uint32_t kFewBins = 32;                 // bins of a level up to which the scatter pass spreads a tile's records (bin_scatter)
constexpr int kAccUnroll = 4;                    // record loads in flight per lane in the tail of a long item
constexpr int kAccPreWords = 24;                 // registers per lane for records requested one item ahead
constexpr uint32_t kAccWgsPerCu = 1;             // its registers let one accumulate workgroup run per CU
constexpr uint32_t kTargetRecordsPerAccWg = 16384;
constexpr uint32_t kMaxParts = 4;                // level parts of the scatter grid (1, 2, 8: slower)
constexpr uint32_t kCountParts = 2;              // ... of the count grid (its workgroups are lighter)
// Level parts are doubled (up to one level per part) until one part's bins fit these bounds: a count
// workgroup keeps one LDS word per bin of its part, a scatter workgroup three, next to its staging area.
constexpr uint32_t kMaxCountPartBins = 4096, kMaxScatterPartBins = 4096;
// Beyond this many chunks in all, a tile is kBigTileMult * 512 points and the scatter pass does not
// stage (bin_scatter_direct, one LDS word per bin of its part).  One level of 4096 chunks per part: the grid runs
// part after part, so the records in flight then belong to two levels (200 MB at T = 2^24), not four (-3%).
constexpr uint32_t kMaxStagedBins = 16384, kBigTileMult = 8, kMaxDirectPartBins = 4096;
// A level may have this many chunks (one level is the smallest part): T up to 2^24 at 4096 entries per chunk.
constexpr uint32_t kMaxLevelBins = 4096;

static_assert(kChunkLog2 <= 12, "a record holds a 12-bit local index");

struct Workspace {
  uint32_t* counts;     // [n_tiles + 1][n_bins] counts, then exclusive prefix over tiles (last row: totals)
  uint32_t* bin_start;  // [n_bins] first record of the bin
  uint32_t* bin_total;  // [n_bins] records in the bin
  float* tile_max;      // [n_tiles * parts of the scatter grid (at most L)] largest |dL/dy| seen by each scatter workgroup
  uint32_t* item_counter;  // [1] next work item of the accumulate pass
  uint32_t* records;    // [B * L * rec_per_point] records (Record::kWords words each)
  uint32_t n_tiles;
  uint32_t n_bins;
};

static inline uint64_t align_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

// one count / scatter workgroup per tile and level part
static uint32_t tiles_for(const BinPlan& bp, uint32_t B) {
  const uint32_t points = kBinThreads * bp.tile_mult;
  return (uint32_t)(((uint64_t)B + points - 1) / points);
}

static uint64_t carve(const hashgrid* h, uint32_t B, uint8_t* base, Workspace* ws) {
  const uint32_t nt = tiles_for(h->bp, B), nb = h->bp.bin_base[h->lv.L];
  uint64_t off = 0;
  auto take = [&](uint64_t bytes) {
    uint64_t o = off;
    off = align_up(off + bytes, 256);
    return o;
  };
  const uint64_t o_counts = take((uint64_t)(nt + 1) * nb * 4), o_start = take((uint64_t)nb * 4),
                 o_total = take((uint64_t)nb * 4), o_max = take((uint64_t)nt * h->lv.L * 4), o_item = take(4),
                 o_rec = take((uint64_t)B * h->lv.L * h->bp.rec_per_point *
                              (8 + (h->cfg.F * (h->cfg.io_dtype == HG_F16 ? 2u : 4u) + 3u) / 4u * 4u));
  if (ws) {
    ws->counts = reinterpret_cast<uint32_t*>(base + o_counts);
    ws->bin_start = reinterpret_cast<uint32_t*>(base + o_start);
    ws->bin_total = reinterpret_cast<uint32_t*>(base + o_total);
    ws->tile_max = reinterpret_cast<float*>(base + o_max);
    ws->item_counter = reinterpret_cast<uint32_t*>(base + o_item);
    ws->records = reinterpret_cast<uint32_t*>(base + o_rec);
    ws->n_tiles = nt;
    ws->n_bins = nb;
  }
  return off;
}

// Chunking of every level's gradient slice.  1:1 levels are cut at grid-row
// boundaries (a row = all vertices that share the coordinates of dimensions
// 1..d-1, contiguous in memory), a power-of-two number of rows per chunk; hashed
// levels are cut into aligned blocks of 2^chunk_log2 entries, which the XOR with
// the low chunk_log2 bits of v_0 cannot leave.
void build_bin_plan(hashgrid* h) {
  BinPlan& bp = h->bp;
  bp = BinPlan{};
  const hashgrid_config& c = h->cfg;
  const LevelTable& lv = h->lv;
  bp.chunk_log2 = chunk_log2_of(c.F);
  // The pairing of the two corners along dimension 0 needs a power-of-two T (after Eq. 4's mod T
  // with another T the pair's entries are unrelated) and a second dimension to cut 1:1 levels by
  // grid rows; otherwise every corner gets a record of its own (twice the records).
  bp.corner_records = (c.d < 2 || !lv.T_is_pow2) ? 1u : 0u;
  bp.rec_per_point = bp.corner_records ? 1u << c.d : 1u << (c.d - 1);
  if (c.d < 1 || c.d > 3) return;  // F is 1, 2, 4 or 8 (hashgrid_create)
  const uint32_t cap = 1u << bp.chunk_log2;
  uint32_t bins = 0;
  for (uint32_t l = 0; l < lv.L; ++l) {
    const uint32_t verts = lv.verts[l];
    uint32_t nb;
    if (bp.corner_records) {
      nb = (lv.size[l] + cap - 1u) >> bp.chunk_log2;  // aligned blocks of the level's slice, the last one ragged
    } else if ((lv.dense_mask >> l) & 1u) {
      if (verts > cap) return;
      uint32_t s = 0;
      while (((uint64_t)verts << (s + 1)) <= cap) ++s;
      const uint64_t rows = c.d == 3 ? (uint64_t)verts * verts : verts;
      bp.row_shift[l] = (uint8_t)s;
      nb = (uint32_t)((rows + (1ull << s) - 1) >> s);
    } else {
      // The two corners of a pair share the bits above the chunk unless stepping v_0 carries out of
      // its low chunk_log2 bits, which needs a resolution of 2^chunk_log2 or more and then happens
      // for one voxel in 2^chunk_log2: those pairs bypass the sort (see bin_scatter).
      nb = lv.T > cap ? lv.T >> bp.chunk_log2 : 1u;
    }
    if (nb > kMaxLevelBins) return;
    bp.bin_base[l] = bins;
    bins += nb;
  }
  bp.bin_base[lv.L] = bins;
  auto max_part_bins = [&](uint32_t np) {
    uint32_t m = 0;
    for (uint32_t p = 0; p < np; ++p) {
      const uint32_t nbp = bp.bin_base[(p + 1) * lv.L / np] - bp.bin_base[p * lv.L / np];
      m = nbp > m ? nbp : m;
    }
    return m;
  };
  auto parts_for = [&](uint32_t start, uint32_t limit) {
    uint32_t np = lv.L < start ? lv.L : start;
    while (max_part_bins(np) > limit && np < lv.L) np = np * 2 < lv.L ? np * 2 : lv.L;
    return max_part_bins(np) <= limit ? np : 0u;
  };
  bp.count_parts = parts_for(kCountParts, kMaxCountPartBins);
  // With very many chunks a tile of 512 points leaves less than a record per chunk and level: the
  // per-chunk work of every count / scatter workgroup (and the count table) then outweighs the
  // records, and staging them for whole-line writes gains nothing.  Larger tiles, no staging.
  bp.tile_mult = bins > kMaxStagedBins ? kBigTileMult : 1u;
  bp.scatter_parts = bp.tile_mult > 1 ? parts_for(kMaxParts, kMaxDirectPartBins) : parts_for(kMaxParts, kMaxScatterPartBins);
  if (!bp.count_parts || !bp.scatter_parts) return;
  bp.supported = 1;
}

// Slices per bin of each level for a batch of B points: coarse 1:1 levels have
// few bins and receive B * 2^(d-1) records, so their bins are shared by several
// accumulate-workgroups.
static void plan_slices(BinPlan& bp, const LevelTable& lv, uint32_t B) {
  uint32_t wgs = 0;
  for (uint32_t l = 0; l < lv.L; ++l) {
    const uint32_t nb = bp.bin_base[l + 1] - bp.bin_base[l];
    const uint64_t per_bin = ((uint64_t)B * bp.rec_per_point + nb - 1) / nb;
    uint64_t s = (per_bin + kTargetRecordsPerAccWg - 1) / kTargetRecordsPerAccWg;
    if (!((lv.dense_mask >> l) & 1u) && s < 4) s = 1;  // hashed bins are evenly filled
    if (s > 256) s = 256;
    bp.slices[l] = (uint32_t)(s < 1 ? 1 : s);
    bp.wg_base[l] = wgs;
    wgs += nb * bp.slices[l];
  }
  bp.wg_base[lv.L] = wgs;
}

// ------------------------------------------------------------------ device

// The pairs of a hashed level whose two corners lie in different chunks (Rows::cross; one voxel
// in 2^chunk_log2 along dimension 0, and only at resolutions of 2^chunk_log2 or more) get no
// record: their 2^d products go to the gradient with device-scope atomics.  T is a power of two.
template <int D, int F>
__device__ __forceinline__ void add_crossing_pairs(const LevelTable& lv, uint32_t l, bool smooth, const float (&xp)[D],
                                                   const float (&g)[F], void* __restrict__ grad, const bool g16) {
  const float Nf = (float)lv.N[l];
  const float shift = smooth ? 0.5f : 0.0f;
  const float cmaxf = smooth ? Nf : Nf - 1.0f;
  uint32_t c0[D];
  float w[D], u[D];
#pragma unroll
  for (int i = 0; i < D; ++i) {
    float wf;
    split(xp[i], Nf, shift, cmaxf, c0[i], wf);
    w[i] = smooth ? smoothstep(wf) : wf;
    u[i] = smooth ? smoothstep(1.0f - wf) : 1.0f - wf;
  }
  const uint32_t tmask = lv.T - 1u;
  float* gl = static_cast<float*>(grad) + lv.offset[l] * F;          // (g16: the same entries, as halves)
  _Float16* gl16 = static_cast<_Float16*>(grad) + lv.offset[l] * F;
#pragma unroll
  for (uint32_t r = 0; r < (1u << (D - 1)); ++r) {
    float wr = 1.0f;
    uint32_t rt = 0;
#pragma unroll
    for (int i = 1; i < D; ++i) {
      const uint32_t up = (r >> (i - 1)) & 1u;
      wr *= up ? w[i] : u[i];
      rt ^= (c0[i] + up) * prime(i);
    }
    const uint32_t ia = (c0[0] ^ rt) & tmask, ib = ((c0[0] + 1u) ^ rt) & tmask;
#pragma unroll
    for (int f = 0; f < F; ++f) {
      if (g16) {  // uniform
        grad_atomic_add(gl16, F * (uint64_t)ia + f, u[0] * (wr * g[f]));
        grad_atomic_add(gl16, F * (uint64_t)ib + f, w[0] * (wr * g[f]));
      } else {
        grad_atomic_add(gl, F * (uint64_t)ia + f, u[0] * (wr * g[f]));
        grad_atomic_add(gl, F * (uint64_t)ib + f, w[0] * (wr * g[f]));
      }
    }
  }
}

template <int D>
__device__ __forceinline__ void load_x(const float* __restrict__ x, uint32_t b, float (&xp)[D]) {
#pragma unroll
  for (int i = 0; i < D; ++i) xp[i] = x[(uint64_t)b * D + i];
}

// Workgroup -> tile of points.  Workgroup i runs on XCD i mod 8 (each XCD has its
// own L2), so consecutive tiles are given to consecutive workgroups of one XCD:
// the runs two neighbouring tiles write into a bin are adjacent in memory, and
// the cache line they share is completed inside one L2 instead of being written
// back half-filled twice.  Returns n_tiles or more for surplus workgroups.
__device__ __forceinline__ uint32_t tile_of_workgroup(uint32_t wg, uint32_t n_tiles) {
  const uint32_t per_xcd = (n_tiles + 7u) / 8u;
  const uint32_t j = wg >> 3;
  return j < per_xcd ? (wg & 7u) * per_xcd + j : n_tiles;
}

// Levels are split into gridDim.y parts; a count / scatter workgroup serves one
// tile of points and one part.  More, lighter workgroups per CU hide the latency
// of the LDS atomics and of the per-level barriers.
__device__ __forceinline__ void part_levels(uint32_t L, uint32_t& l0, uint32_t& l1) {
  l0 = blockIdx.y * L / gridDim.y;
  l1 = (blockIdx.y + 1) * L / gridDim.y;
}

// count: records per (tile, bin).
template <int D, bool CORNERS>
__global__ __launch_bounds__(kBinThreads) void bin_count(const LevelTable lv, const BinPlan bp, const bool smooth,
                                                         const uint32_t B, const float* __restrict__ x,
                                                         uint32_t* __restrict__ counts, const uint32_t n_bins,
                                                         const uint32_t n_tiles) {
  extern __shared__ uint32_t hist[];  // bins of this part's levels
  const uint32_t tile = tile_of_workgroup(blockIdx.x, n_tiles);
  if (tile >= n_tiles) return;  // uniform: a surplus workgroup of the rounded-up grid
  uint32_t l0, l1;
  part_levels(lv.L, l0, l1);
  const uint32_t gb_a = bp.bin_base[l0], nbp = bp.bin_base[l1] - gb_a;
  for (uint32_t i = threadIdx.x; i < nbp; i += kBinThreads) hist[i] = 0;
  __syncthreads();
  for (uint32_t sub = 0; sub < bp.tile_mult; ++sub) {
    const uint64_t b64 = ((uint64_t)tile * bp.tile_mult + sub) * kBinThreads + threadIdx.x;
    if (b64 >= B) break;
    const uint32_t b = (uint32_t)b64;
    float xp[D];
    load_x<D>(x, b, xp);
    for (uint32_t l = l0; l < l1; ++l) {
      if constexpr (CORNERS) {
        CornerRows<D> cr;
        corner_rows_of<D, true>(lv, bp, l, smooth, xp, cr);
#pragma unroll
        for (uint32_t m = 0; m < (1u << D); ++m)
          count_one(hist, cr.bin[m] - gb_a);
      } else {
        Rows<D> rw;
        rows_of<D, true>(lv, bp, l, smooth, xp, rw);
        if (rw.cross) continue;
#pragma unroll
        for (uint32_t r = 0; r < (1u << (D - 1)); ++r)
          count_one(hist, rw.bin[r] - gb_a);
      }
    }
  }
  __syncthreads();
  for (uint32_t i = threadIdx.x; i < nbp; i += kBinThreads) counts[(uint64_t)tile * n_bins + gb_a + i] = hist[i];
}

// m = max(m, v) where a NaN on either side wins, so that one NaN in dL/dy is seen at the end
__device__ __forceinline__ float nan_max(float m, float v) { return (v > m || v != v) ? v : m; }

// Exclusive prefix sum of a[0..n) in LDS, in place, by all T threads of the
// workgroup (every thread must call it).  `tmp` holds T/64 words.
template <int T>
__device__ __forceinline__ void block_exclusive_scan(uint32_t* a, uint32_t n, uint32_t* tmp) {
  const uint32_t per = (n + T - 1) / T;
  const uint32_t begin = threadIdx.x * per < n ? threadIdx.x * per : n;
  const uint32_t end = begin + per < n ? begin + per : n;
  uint32_t sum = 0;
  for (uint32_t i = begin; i < end; ++i) sum += a[i];
  uint32_t inc = sum;  // inclusive scan across the wave
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t up = __shfl_up(inc, o);
    if ((threadIdx.x & 63) >= (uint32_t)o) inc += up;
  }
  if ((threadIdx.x & 63) == 63) tmp[threadIdx.x >> 6] = inc;
  __syncthreads();
  uint32_t wave_base = 0;
  for (uint32_t w = 0; w < (threadIdx.x >> 6); ++w) wave_base += tmp[w];
  uint32_t run = wave_base + inc - sum;
  for (uint32_t i = begin; i < end; ++i) {
    const uint32_t v = a[i];
    a[i] = run;
    run += v;
  }
  __syncthreads();
}

// scan: each workgroup takes kScanBins bins and turns their column of
// counts[tile][bin] into the exclusive prefix over tiles; it also writes the
// bin's record count.  Workgroup 0 clears the work counter of the accumulate pass.
constexpr int kScanBins = 32;  // 128-byte rows of the count table per load (16, 8: slower; 64: the same)
// With HG_BWD_OVERWRITE it also clears the gradient of the levels in zero_mask (those that the
// later passes add into, see launch_binned): it is the first kernel of the call to run.
__global__ __launch_bounds__(kScanThreads) void bin_scan(const uint32_t n_tiles, const uint32_t n_bins,
                                                         uint32_t* __restrict__ counts,
                                                         uint32_t* __restrict__ bin_total,
                                                         uint32_t* __restrict__ item_counter, const LevelTable lv,
                                                         const uint32_t zero_mask, const uint32_t F,
                                                         void* __restrict__ grad, const bool g16) {
  __shared__ uint32_t seg_sum[kScanThreads];
  if (blockIdx.x == 0 && threadIdx.x == 0) item_counter[0] = 0;  // the accumulate pass draws its work items from here
  for (uint32_t l = 0; zero_mask >> l; ++l) {  // uniform
    if (!((zero_mask >> l) & 1u)) continue;
    const uint64_t first = lv.offset[l] * F, n = (uint64_t)lv.size[l] * F;
    for (uint64_t i = (uint64_t)blockIdx.x * kScanThreads + threadIdx.x; i < n; i += (uint64_t)gridDim.x * kScanThreads) {
      if (g16) static_cast<_Float16*>(grad)[first + i] = (_Float16)0.0f;
      else static_cast<float*>(grad)[first + i] = 0.0f;
    }
  }
  constexpr uint32_t segs = kScanThreads / kScanBins;
  const uint32_t bin_in = threadIdx.x % kScanBins, seg = threadIdx.x / kScanBins;
  const uint32_t gb = blockIdx.x * kScanBins + bin_in;
  const bool active = gb < n_bins;
  const uint32_t tps = (n_tiles + segs - 1) / segs;
  const uint32_t t0 = seg * tps < n_tiles ? seg * tps : n_tiles;
  const uint32_t t1 = t0 + tps < n_tiles ? t0 + tps : n_tiles;
  uint32_t* col = counts + gb;
  // the loads of a column are independent: issue them eight at a time
  uint32_t s = 0;
  if (active) {
    uint32_t t = t0;
    for (; t + 8 <= t1; t += 8) {
      uint32_t c[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) c[j] = col[(uint64_t)(t + j) * n_bins];
#pragma unroll
      for (int j = 0; j < 8; ++j) s += c[j];
    }
    for (; t < t1; ++t) s += col[(uint64_t)t * n_bins];
  }
  seg_sum[threadIdx.x] = s;
  __syncthreads();
  if (active) {
    uint32_t pre = 0, total = 0;
    for (uint32_t q = 0; q < segs; ++q) {
      const uint32_t v = seg_sum[q * kScanBins + bin_in];
      pre += q < seg ? v : 0u;
      total += v;
    }
    if (seg == 0) {
      bin_total[gb] = total;
      col[(uint64_t)n_tiles * n_bins] = total;  // closes the prefix: count of tile t = row t+1 - row t
    }
    uint32_t run = pre;
    uint32_t t = t0;
    for (; t + 8 <= t1; t += 8) {
      uint32_t c[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) c[j] = col[(uint64_t)(t + j) * n_bins];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        col[(uint64_t)(t + j) * n_bins] = run;
        run += c[j];
      }
    }
    for (; t < t1; ++t) {
      const uint32_t c = col[(uint64_t)t * n_bins];
      col[(uint64_t)t * n_bins] = run;
      run += c;
    }
  }
}

// scatter: writes every record to its slot.  A bin's first record is the sum of
// the record counts of all bins before it (every level holds exactly
// B * rec_per_point records, so this is also level-major); inside a bin the
// tiles of 512 points follow each other.  Level by level the workgroup sorts the
// records of its points by bin in LDS and copies them out bin after bin, so that
// what reaches memory is runs of whole records that mostly fill whole cache
// lines; 16-byte stores scattered over a thousand open runs leave the L2 as
// partial lines and cost several times the bytes.
// Per-bin arrays in LDS, indexed by bin relative to the first bin of this part's levels:
// local[nbp + 1] exclusive prefix of this tile's counts (where a bin's records
// sit in the tile's sorted order), cur[nbp] the same, advanced as records are
// placed, delta[nbp] = global slot minus tile-local position.
// CROSS: this pass adds the pairs that straddle two chunks.  CORNERS: one record per corner (BinPlan::corner_records).
template <int D, typename IT, int F, bool CROSS, bool CORNERS = false>
__global__ __launch_bounds__(kBinThreads) void bin_scatter(const LevelTable lv, const BinPlan bp, const bool smooth,
                                                           const uint32_t B, const float* __restrict__ x,
                                                           const IT* __restrict__ dy,
                                                           const uint32_t* __restrict__ counts,
                                                           const uint32_t* __restrict__ bin_total,
                                                           uint32_t* __restrict__ bin_start,
                                                           uint32_t* __restrict__ records, const uint32_t n_bins,
                                                           const uint32_t n_records, const uint32_t n_tiles,
                                                           float* __restrict__ tile_max, void* __restrict__ grad, const bool g16) {
  constexpr uint32_t R = CORNERS ? 1u << D : 1u << (D - 1 > 0 ? D - 1 : 0);
  using Rec = Record<IT, F>;
  using Stored = typename Rec::Stored;
  Stored* out = reinterpret_cast<Stored*>(records);
  __shared__ uint32_t scan_tmp[kBinThreads / 64];
  // dynamic LDS: staging[R * kBinThreads] records, binv[R * kBinThreads] (part-relative bin of each
  // staged record, 16 bits), then the three per-bin arrays
  extern __shared__ uint32_t lds_u32[];
  Stored* staging = reinterpret_cast<Stored*>(lds_u32);
  uint16_t* binv = reinterpret_cast<uint16_t*>(lds_u32 + R * kBinThreads * Rec::kWords);
  uint32_t* bins_lds = lds_u32 + R * kBinThreads * Rec::kWords + R * kBinThreads / 2;

  const uint32_t tile = tile_of_workgroup(blockIdx.x, n_tiles);
  if (tile >= n_tiles) return;  // uniform: a surplus workgroup of the rounded-up grid
  uint32_t l0, l1;
  part_levels(lv.L, l0, l1);
  const uint32_t gb_a = bp.bin_base[l0], nbp = bp.bin_base[l1] - gb_a;
  uint32_t* delta = bins_lds;
  uint32_t* local = bins_lds + nbp;
  uint32_t* cur = bins_lds + 2 * nbp + 1;

  // records of all bins before this part
  uint32_t before = 0;
  for (uint32_t i = threadIdx.x; i < gb_a; i += kBinThreads) before += bin_total[i];
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) before += __shfl_xor(before, o);
  if ((threadIdx.x & 63) == 0) scan_tmp[threadIdx.x >> 6] = before;
  const uint32_t* row0 = counts + (uint64_t)tile * n_bins + gb_a;  // prefix over tiles before this one
  const uint32_t* row1 = row0 + n_bins;                             // ... including this one
  for (uint32_t i = threadIdx.x; i < nbp; i += kBinThreads) {
    delta[i] = bin_total[gb_a + i];
    local[i] = row1[i] - row0[i];
  }
  if (threadIdx.x == 0) local[nbp] = 0;
  __syncthreads();
  before = 0;
  for (int i = 0; i < kBinThreads / 64; ++i) before += scan_tmp[i];
  __syncthreads();
  block_exclusive_scan<kBinThreads>(delta, nbp, scan_tmp);
  block_exclusive_scan<kBinThreads>(local, nbp + 1, scan_tmp);
  for (uint32_t i = threadIdx.x; i < nbp; i += kBinThreads) {
    const uint32_t f = before + delta[i];  // first record of the bin
    if (tile == 0) bin_start[gb_a + i] = f;
    cur[i] = local[i];
    delta[i] = f + row0[i] - local[i];  // wrap-around arithmetic; undone when a position is added
  }
  __syncthreads();

  const uint64_t b64 = (uint64_t)tile * kBinThreads + threadIdx.x;
  const bool valid = b64 < B;
  const uint32_t b = valid ? (uint32_t)b64 : 0u;
  float xp[D];
  load_x<D>(x, b, xp);
  // dL/dy comes in as 16-byte pieces, K levels each when a level is narrower than that: a narrow
  // read per level with the stride of a row would cost the L1 a line per two lanes, L times over
  constexpr uint32_t kLevelBytes = F * sizeof(IT);
  constexpr uint32_t K = kLevelBytes >= 16 ? 1 : 16 / kLevelBytes;  // levels per piece
  constexpr uint32_t E = 16 / sizeof(IT);                           // scalars per piece
  constexpr uint32_t P = kLevelBytes >= 16 ? kLevelBytes / 16 : 1;  // pieces per level
  const IT* row = dy + (uint64_t)b * lv.L * F;
  const bool vec_ok = (lv.L % K == 0) && (l0 % K == 0) && ((reinterpret_cast<uintptr_t>(dy) & 15) == 0);
  Vec<IT, E> gv;
  float gmax = 0.0f;  // largest |dL/dy| this workgroup sees (idle lanes shadow point 0)
  for (uint32_t l = l0; l < l1; ++l) {
    const uint32_t rb0 = bp.bin_base[l] - gb_a, rb1 = bp.bin_base[l + 1] - gb_a;
    const uint32_t level_first = local[rb0], emitted = local[rb1] - level_first;  // <= R * kBinThreads
    IT g[F];
    if (vec_ok && K > 1) {  // uniform
      if ((l - l0) % K == 0) gv = *reinterpret_cast<const Vec<IT, E>*>(row + (uint64_t)l * F);
      const uint32_t k = (l - l0) % K;
#pragma unroll
      for (int f = 0; f < F; ++f) {
        g[f] = gv.v[f];
#pragma unroll
        for (uint32_t q = 1; q < K; ++q) g[f] = k == q ? gv.v[F * q + f] : g[f];
      }
    } else if (vec_ok) {
#pragma unroll
      for (uint32_t q = 0; q < P; ++q) {
        const Vec<IT, E> piece = *reinterpret_cast<const Vec<IT, E>*>(row + (uint64_t)l * F + q * E);
#pragma unroll
        for (uint32_t e = 0; e < E; ++e)
          if (q * E + e < (uint32_t)F) g[q * E + e] = piece.v[e];
      }
    } else {
#pragma unroll
      for (int f = 0; f < F; ++f) g[f] = row[(uint64_t)l * F + f];
    }
    float gf[F];
#pragma unroll
    for (int f = 0; f < F; ++f) {
      gf[f] = (float)g[f];
      gmax = nan_max(gmax, fabsf(gf[f]));
    }
    // Position of a new record of bin rb in the tile's sorted order.  On a level of few bins a wave's
    // lanes crowd into the same counters and a tile's run for a bin is long: there the wave draws
    // its slots with one add per bin (wave_add_one) and the run is filled with a stride
    // (spread_in_run), for the accumulate pass.  Levels of many bins take the plain atomic.
    const bool few_bins = rb1 - rb0 <= kFewBins;  // uniform
    auto take_slot = [&](const uint32_t rb) {
      if (!few_bins) return __hip_atomic_fetch_add(&cur[rb], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      const uint32_t first = local[rb];
      return first + spread_in_run(wave_add_one<true>(cur, rb) - first, local[rb + 1] - first);
    };
    if (valid) {
      if constexpr (CORNERS) {
        // a corner's record: all of its weight on the "lower" side of a pair whose upper weight is 0
        CornerRows<D> cr;
        corner_rows_of<D, false>(lv, bp, l, smooth, xp, cr);
#pragma unroll
        for (uint32_t m = 0; m < R; ++m) {
          const uint32_t rb = cr.bin[m] - gb_a;
          const uint32_t pos = take_slot(rb) - level_first;
          if (pos < R * kBinThreads) {
            staging[pos] = Rec::make(cr.la[m], 0u, 0.0f, cr.weight[m], g);
            binv[pos] = (uint16_t)rb;
          }
        }
      } else {
        Rows<D> rw;
        rows_of<D, false>(lv, bp, l, smooth, xp, rw);
        if (CROSS && rw.cross) add_crossing_pairs<D, F>(lv, l, smooth, xp, gf, grad, g16);
#pragma unroll
        for (uint32_t r = 0; r < R && !rw.cross; ++r) {
          const uint32_t rb = rw.bin[r] - gb_a;
          const uint32_t pos = take_slot(rb) - level_first;
          if (pos < R * kBinThreads) {  // holds when the count pass saw the same x
            staging[pos] = Rec::make(rw.la[r], rw.k, rw.wf0, rw.wrow[r], g, smooth);
            binv[pos] = (uint16_t)rb;
          }
        }
      }
    }
    __syncthreads();
    for (uint32_t j = threadIdx.x; j < emitted && j < R * kBinThreads; j += kBinThreads) {
      const uint32_t d = delta[binv[j]] + level_first + j;
      // the count pass saw the same inputs, so d < n_records; the check only keeps a
      // caller who changed x in between from writing out of bounds
      if (d < n_records) out[d] = staging[j];
    }
    __syncthreads();
  }
  // the accumulate pass scales its fixed point by the largest |dL/dy| of the call: one value per workgroup
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) gmax = nan_max(gmax, __shfl_xor(gmax, o));
  float* wave_max = reinterpret_cast<float*>(scan_tmp);  // free since the prologue
  if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = gmax;
  __syncthreads();
  if (threadIdx.x == 0) {
    float t = wave_max[0];
    for (int i = 1; i < kBinThreads / 64; ++i) t = nan_max(t, wave_max[i]);
    tile_max[tile * gridDim.y + blockIdx.y] = t;
  }
}

// scatter without staging, for plans of very many bins (BinPlan::tile_mult > 1): a tile is
// tile_mult * 512 points, which the workgroup walks 512 at a time, and every record goes
// straight to its slot.  The runs a tile writes are a few records long at best, so sorting them
// in LDS first would not make whole lines of them; what merges partial lines here is the L2,
// which keeps the tile's open runs (a few bytes per bin of the part) while the workgroup lasts.
// LDS: slot[nbp], the next free record slot of each bin of this part for this tile.
template <int D, typename IT, int F, bool CROSS, bool CORNERS = false>
__global__ __launch_bounds__(kBinThreads) void bin_scatter_direct(
    const LevelTable lv, const BinPlan bp, const bool smooth, const uint32_t B, const float* __restrict__ x,
    const IT* __restrict__ dy, const uint32_t* __restrict__ counts, const uint32_t* __restrict__ bin_total,
    uint32_t* __restrict__ bin_start, uint32_t* __restrict__ records, const uint32_t n_bins, const uint32_t n_records,
    const uint32_t n_tiles, float* __restrict__ tile_max, void* __restrict__ grad, const bool g16) {
  constexpr uint32_t R = CORNERS ? 1u << D : 1u << (D - 1 > 0 ? D - 1 : 0);
  using Rec = Record<IT, F>;
  using Stored = typename Rec::Stored;
  Stored* out = reinterpret_cast<Stored*>(records);
  __shared__ uint32_t scan_tmp[kBinThreads / 64];
  extern __shared__ uint32_t slot[];

  const uint32_t tile = tile_of_workgroup(blockIdx.x, n_tiles);
  if (tile >= n_tiles) return;  // uniform: a surplus workgroup of the rounded-up grid
  uint32_t l0, l1;
  part_levels(lv.L, l0, l1);
  const uint32_t gb_a = bp.bin_base[l0], nbp = bp.bin_base[l1] - gb_a;

  // first record of each bin = records of all bins before it; then the records of the tiles before this one
  uint32_t before = 0;
  for (uint32_t i = threadIdx.x; i < gb_a; i += kBinThreads) before += bin_total[i];
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) before += __shfl_xor(before, o);
  if ((threadIdx.x & 63) == 0) scan_tmp[threadIdx.x >> 6] = before;
  for (uint32_t i = threadIdx.x; i < nbp; i += kBinThreads) slot[i] = bin_total[gb_a + i];
  __syncthreads();
  before = 0;
  for (int i = 0; i < kBinThreads / 64; ++i) before += scan_tmp[i];
  __syncthreads();
  block_exclusive_scan<kBinThreads>(slot, nbp, scan_tmp);
  const uint32_t* row0 = counts + (uint64_t)tile * n_bins + gb_a;  // prefix over the tiles before this one
  for (uint32_t i = threadIdx.x; i < nbp; i += kBinThreads) {
    const uint32_t f = before + slot[i];
    if (tile == 0) bin_start[gb_a + i] = f;
    slot[i] = f + row0[i];
  }
  __syncthreads();

  float gmax = 0.0f;  // largest |dL/dy| this workgroup sees
  for (uint32_t sub = 0; sub < bp.tile_mult; ++sub) {
    const uint64_t b64 = ((uint64_t)tile * bp.tile_mult + sub) * kBinThreads + threadIdx.x;
    if (b64 >= B) break;  // no barrier inside this loop
    const uint32_t b = (uint32_t)b64;
    float xp[D];
    load_x<D>(x, b, xp);
    const IT* row = dy + (uint64_t)b * lv.L * F;
    for (uint32_t l = l0; l < l1; ++l) {
      IT g[F];
      float gf[F];
#pragma unroll
      for (int f = 0; f < F; ++f) {
        g[f] = row[(uint64_t)l * F + f];
        gf[f] = (float)g[f];
        gmax = nan_max(gmax, fabsf(gf[f]));
      }
      if constexpr (CORNERS) {
        CornerRows<D> cr;
        corner_rows_of<D, false>(lv, bp, l, smooth, xp, cr);
#pragma unroll
        for (uint32_t m = 0; m < R; ++m) {
          const uint32_t d =
              __hip_atomic_fetch_add(&slot[cr.bin[m] - gb_a], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
          if (d < n_records) out[d] = Rec::make(cr.la[m], 0u, 0.0f, cr.weight[m], g);
        }
      } else {
        Rows<D> rw;
        rows_of<D, false>(lv, bp, l, smooth, xp, rw);
        if (rw.cross) {
          if (CROSS) add_crossing_pairs<D, F>(lv, l, smooth, xp, gf, grad, g16);
          continue;
        }
#pragma unroll
        for (uint32_t r = 0; r < R; ++r) {
          const uint32_t d =
              __hip_atomic_fetch_add(&slot[rw.bin[r] - gb_a], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
          // the count pass saw the same inputs, so d < n_records; the check only keeps a caller
          // who changed x in between from writing out of bounds
          if (d < n_records) out[d] = Rec::make(rw.la[r], rw.k, rw.wf0, rw.wrow[r], g, smooth);
        }
      }
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) gmax = nan_max(gmax, __shfl_xor(gmax, o));
  __syncthreads();  // scan_tmp is free again
  float* wave_max = reinterpret_cast<float*>(scan_tmp);
  if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = gmax;
  __syncthreads();
  if (threadIdx.x == 0) {
    float t = wave_max[0];
    for (int i = 1; i < kBinThreads / 64; ++i) t = nan_max(t, wave_max[i]);
    tile_max[tile * gridDim.y + blockIdx.y] = t;
  }
}

// The pairs that straddle two chunks (add_crossing_pairs), as a pass of its own after the accumulate
// pass: with HG_BWD_OVERWRITE the owners of the chunks store their sums, so these atomic adds
// must come after them.  Only the levels in level_mask can have such pairs; one thread per point.
template <int D, typename IT, int F>
__global__ __launch_bounds__(kBinThreads) void bin_crossing(const LevelTable lv, const BinPlan bp, const bool smooth,
                                                            const uint32_t B, const float* __restrict__ x,
                                                            const IT* __restrict__ dy, const uint32_t level_mask,
                                                            void* __restrict__ grad, const bool g16) {
  const uint64_t b64 = (uint64_t)blockIdx.x * kBinThreads + threadIdx.x;
  if (b64 >= B) return;
  const uint32_t b = (uint32_t)b64;
  float xp[D];
  load_x<D>(x, b, xp);
  for (uint32_t l = 0; level_mask >> l; ++l) {  // uniform
    if (!((level_mask >> l) & 1u)) continue;
    Rows<D> rw;
    rows_of<D, true>(lv, bp, l, smooth, xp, rw);
    if (!rw.cross) continue;
    float gf[F];
#pragma unroll
    for (int f = 0; f < F; ++f) gf[f] = (float)dy[((uint64_t)b * lv.L + l) * F + f];
    add_crossing_pairs<D, F>(lv, l, smooth, xp, gf, grad, g16);
  }
}

// accumulate: work item = (bin, slice).  The grid is persistent: workgroup w
// starts with item w and then draws items from a device-wide counter, two items
// ahead, so that the first records and the count of the next item are fetched
// while the current one is streamed (the chain "offsets -> records" is paid once
// per workgroup, not once per bin) and workgroups that drew short items simply
// draw more of them: items differ in size by a factor of ten on 1:1 levels when
// the points crowd around a surface.  The LDS accumulators are re-zeroed by the
// lanes that have just read them.
// GT: type of the gradient scalars (float, or _Float16: the sums are still exact fixed point and are
// rounded to half precision once, where they are added to the gradient).
template <typename IT, int F, bool SMOOTH, typename GT = float>
__global__ __launch_bounds__(kAccThreads) void bin_accumulate(const LevelTable lv, const BinPlan bp,
                                                              const uint32_t B, const uint32_t n_items,
                                                              const uint32_t* __restrict__ bin_start,
                                                              const uint32_t* __restrict__ bin_total,
                                                              const float* __restrict__ tile_max,
                                                              const uint32_t n_max,
                                                              const uint32_t* __restrict__ records,
                                                              uint32_t* __restrict__ item_counter,
                                                              GT* __restrict__ grad, const uint32_t overwrite_mask) {
  // bit l of overwrite_mask: the owner of a chunk of level l stores its sums (HG_BWD_OVERWRITE, one
  // slice per chunk, no pairs that straddle chunks) instead of adding them to what is there
  __shared__ uint32_t s_ticket;
  extern __shared__ unsigned long long acc[];  // [F][2^chunk_log2] fixed point: feature 0 of every entry, then
                                               // feature 1 ..., so that consecutive entries map to consecutive banks
  // largest |dL/dy| of the call (NaN if any is NaN) from the scatter workgroups' maxima
  __shared__ float red[kAccThreads / 64];
  float m = 0.0f;
  for (uint32_t i = threadIdx.x; i < n_max; i += kAccThreads) m = nan_max(m, tile_max[i]);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) m = nan_max(m, __shfl_xor(m, o));
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
  __syncthreads();
  m = red[0];
#pragma unroll
  for (int i = 1; i < kAccThreads / 64; ++i) m = nan_max(m, red[i]);
  if (m == 0.0f && overwrite_mask == 0) return;  // every summand is zero (uniform: all lanes hold the same m)
  const bool finite = m < INFINITY;
  constexpr uint32_t cl = chunk_log2_of(F), cap = 1u << cl, cmask = cap - 1u;
  // fixed-point scale: |summand| <= m < 2^E, at most 8B summands per entry
  int E = 0;
  if (finite) (void)frexpf(m, &E);
  const int H = 3 + (32 - __builtin_clz(B > 1 ? B - 1 : 1));
  const int S = (62 - H < kFixedBits ? 62 - H : kFixedBits) - E;  // |summand| * 2^S < 2^min(62-H, 51)
  const double scale = ldexp(1.0, S), inv_scale = ldexp(1.0, -S);
  const uint32_t n_records = B * lv.L * bp.rec_per_point;  // < 2^32 (hashgrid_bwd_workspace_bytes)
  constexpr int kPer = (int)cap / kAccThreads;  // entries per lane
  struct alignas(F * sizeof(GT) > 16 ? 16 : F * sizeof(GT)) Entry {
    GT v[F];
  };

  // item_counter starts at 0 (bin_scan clears it); a ticket is the item it stands for
  auto draw = [&]() {
    return gridDim.x + __hip_atomic_fetch_add(item_counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  };
  if (threadIdx.x == 0) s_ticket = draw();
  for (uint32_t i = threadIdx.x; i < F * cap; i += kAccThreads) acc[i] = 0ull;
  __syncthreads();
  uint32_t next = s_ticket;  // every item number of n_items or more ends the loop, and tickets only grow

  // which level, bin and slice an item is
  auto decode = [&](uint32_t item, uint32_t& l, uint32_t& bin, uint32_t& slice) {
    l = 0;
    while (l + 1 < lv.L && item >= bp.wg_base[l + 1]) ++l;
    const uint32_t k = item - bp.wg_base[l];
    bin = k / bp.slices[l];
    slice = k - bin * bp.slices[l];
  };

  // Everything an item needs before its records can be used: where they are, which chunk of
  // the gradient it owns, and (software pipeline) its first kPre records per lane and its
  // gradient chunk, both requested while the previous item is still being flushed.
  struct Item {
    uint32_t l, n_sl, r0, r1, n_e;
    GT* gl;
    bool live, dense;
  };
  using Rec = Record<IT, F>;
  using Stored = typename Rec::Stored;
  constexpr int kPre = kAccPreWords / (int)Rec::kWords, kHalf = kPre / 2;
  // wide entries: the registers do not hold the next item's gradient chunk and several records in
  // flight as well, so the chunk is read when it is flushed and fewer records are unrolled
  constexpr bool kChunkAhead = F <= 2;
  constexpr int kUnroll = F <= 2 ? kAccUnroll : 2;
  auto describe = [&](uint32_t item, uint32_t start, uint32_t total, uint32_t l, uint32_t bin, uint32_t slice) {
    Item it;
    it.l = l;
    it.n_sl = bp.slices[l];
    const uint32_t per = (total + it.n_sl - 1) / it.n_sl;
    it.r0 = start + slice * per;
    it.r1 = (slice * per + per < total) ? it.r0 + per : start + total;
    // true for counts that belong to these points; keeps a caller who passed HG_BWD_COUNTED over
    // the counts of another batch from reading outside the records
    it.r0 = it.r0 < n_records ? it.r0 : n_records;
    it.r1 = it.r1 < n_records ? it.r1 : n_records;
    it.live = item < n_items && slice * per < total;
    uint32_t e0, e1;  // entries of this chunk in the level's slice
    it.dense = ((lv.dense_mask >> l) & 1u) && !bp.corner_records;  // (corner records: every level in aligned blocks)
    if (it.dense) {
      e0 = (bin << bp.row_shift[l]) * lv.verts[l];
      e1 = e0 + (lv.verts[l] << bp.row_shift[l]);
    } else {
      e0 = bin << cl;
      e1 = e0 + cap;
    }
    if (e1 > lv.size[l]) e1 = lv.size[l];
    it.n_e = e1 - e0;
    it.gl = grad + (lv.offset[l] + e0) * F;
    return it;
  };
  // records j0..j1-1 of each lane's share of the item
  auto request_records = [&](const Item& it, Stored (&pre)[kPre], const int j0, const int j1) {
    if (!it.live || !finite) return;
#pragma unroll
    for (int j = 0; j < kPre; ++j) {
      if (j < j0 || j >= j1) continue;
      const uint32_t i = it.r0 + threadIdx.x + j * kAccThreads;
      if (i < it.r1) pre[j] = Rec::load(records, i);
    }
  };
  auto overwrites = [&](const Item& it) { return ((overwrite_mask >> it.l) & 1u) != 0; };  // uniform
  auto request_chunk = [&](const Item& it, Entry (&cur)[kPer]) {
    if (!kChunkAhead || !it.live || !finite || overwrites(it)) return;
    if (it.n_sl == 1) {
#pragma unroll
      for (int j = 0; j < kPer; ++j) {
        const uint32_t e = threadIdx.x + j * kAccThreads;
        if (e < it.n_e) cur[j] = reinterpret_cast<const Entry*>(it.gl)[e];
      }
    }
  };

  uint32_t item = blockIdx.x;
  uint32_t l = 0, bin = 0, slice = 0, start = 0, total = 0;
  if (item < n_items) {
    decode(item, l, bin, slice);
    start = bin_start[bp.bin_base[l] + bin];
    total = bin_total[bp.bin_base[l] + bin];
  }
  Item it = describe(item, start, total, l, bin, slice);
  Stored pre[kPre];
  Entry cur[kPer];
  request_records(it, pre, 0, kPre);
  request_chunk(it, cur);
  while (item < n_items) {
    // the item after the next one, and the offsets of the next one: in flight while this one is processed
    uint32_t ticket = 0;
    if (threadIdx.x == 0) ticket = draw();
    uint32_t l_n = 0, bin_n = 0, slice_n = 0, start_n = 0, total_n = 0;
    if (next < n_items) {
      decode(next, l_n, bin_n, slice_n);
      start_n = bin_start[bp.bin_base[l_n] + bin_n];
      total_n = bin_total[bp.bin_base[l_n] + bin_n];
    }
    Item it_n;
    it_n.live = false;
    Entry cur_n[kPer];
    // HG_BWD_OVERWRITE: a chunk that gets no sums stored below is cleared by its owner
    auto clear_chunk = [&](const Item& c) {
      for (uint32_t q = threadIdx.x; q < c.n_e * F; q += kAccThreads) c.gl[q] = (GT)0.0f;
    };
    if (it.live && !finite) {
      if (overwrites(it)) {  // uniform
        clear_chunk(it);
        __threadfence();  // the zeros reach the L2 before any lane's atomics below
        __syncthreads();
      }
      // inf or NaN upstream: keep IEEE semantics with direct fp32 atomics (slow, rare)
      for (uint32_t i = it.r0 + threadIdx.x; i < it.r1; i += kAccThreads) {
        uint32_t la, lb;
        float w_lo, w_up;
        double G[F];
        bool first;
        Rec::unpack_scaled(Rec::load(records, i), it.dense, cmask, it.n_e - 1u, 1.0, la, lb, w_lo, w_up, first, G);
        const float wu = SMOOTH && !first ? smoothstep(w_up) : w_up, wl = SMOOTH && !first ? smoothstep(w_lo) : w_lo;
#pragma unroll
        for (int f = 0; f < F; ++f) {
          if (la < it.n_e) grad_atomic_add(it.gl, F * la + f, wl * (float)G[f]);
          if (lb < it.n_e) grad_atomic_add(it.gl, F * lb + f, wu * (float)G[f]);
        }
      }
      it_n = describe(next, start_n, total_n, l_n, bin_n, slice_n);
    } else if (!it.live) {
      if (overwrites(it)) clear_chunk(it);  // no records for this chunk (item < n_items inside the loop)
      it_n = describe(next, start_n, total_n, l_n, bin_n, slice_n);
      request_records(it_n, pre, 0, kPre);
      request_chunk(it_n, cur_n);
    } else {
      auto add_record = [&](const Stored& rec) {
        uint32_t la, lb;
        float w_lo, w_up;
        double G[F];
        bool first;
        Rec::unpack_scaled(rec, it.dense, cmask, it.n_e - 1u, scale, la, lb, w_lo, w_up, first, G);
        const float wu = SMOOTH && !first ? smoothstep(w_up) : w_up, wl = SMOOTH && !first ? smoothstep(w_lo) : w_lo;
#pragma unroll
        for (int f = 0; f < F; ++f) {
          __hip_atomic_fetch_add(&acc[f * cap + la], fixed_product(wl, G[f]), __ATOMIC_RELAXED,
                                 __HIP_MEMORY_SCOPE_WORKGROUP);
          __hip_atomic_fetch_add(&acc[f * cap + lb], fixed_product(wu, G[f]), __ATOMIC_RELAXED,
                                 __HIP_MEMORY_SCOPE_WORKGROUP);
        }
      };
      // The records requested ahead of time, in two halves: as soon as the first half has been
      // consumed its registers take the first half of the next item, so that loads stay in
      // flight while the LDS atomics of this item run, not only while it is flushed.
#pragma unroll
      for (int j = 0; j < kHalf; ++j)
        if (it.r0 + threadIdx.x + j * kAccThreads < it.r1) add_record(pre[j]);
      it_n = describe(next, start_n, total_n, l_n, bin_n, slice_n);
      request_records(it_n, pre, 0, kHalf);
#pragma unroll
      for (int j = kHalf; j < kPre; ++j)
        if (it.r0 + threadIdx.x + j * kAccThreads < it.r1) add_record(pre[j]);
      // the rest of a long item, kAccUnroll loads in flight per lane
      uint32_t i = it.r0 + threadIdx.x + kPre * kAccThreads;
      for (; i + (kUnroll - 1) * kAccThreads < it.r1; i += kUnroll * kAccThreads) {
        Stored rec[kUnroll];
#pragma unroll
        for (int j = 0; j < kUnroll; ++j) rec[j] = Rec::load(records, i + j * kAccThreads);
#pragma unroll
        for (int j = 0; j < kUnroll; ++j) add_record(rec[j]);
      }
      for (; i < it.r1; i += kAccThreads) add_record(Rec::load(records, i));
      // request the rest of the next item's records and its gradient chunk, then flush this one under them
      request_records(it_n, pre, kHalf, kPre);
      request_chunk(it_n, cur_n);
    }
    if (threadIdx.x == 0) s_ticket = ticket;
    __syncthreads();
    const uint32_t after_next = s_ticket;  // written before the barrier above, rewritten only after the one below
    if (it.live && finite) {
      if (it.n_sl == 1) {
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
          const uint32_t e = threadIdx.x + j * kAccThreads;
          long long a[F];
#pragma unroll
          for (int f = 0; f < F; ++f) {
            a[f] = (long long)acc[f * cap + e];
            acc[f * cap + e] = 0ull;  // ready for the next item
          }
          if (e >= it.n_e) continue;
          if (overwrites(it)) {
            // what adding to a cleared entry would leave
#pragma unroll
            for (int f = 0; f < F; ++f) cur[j].v[f] = (GT)(0.0f + (a[f] ? (float)((double)a[f] * inv_scale) : 0.0f));
          } else {
            if (!kChunkAhead) cur[j] = reinterpret_cast<const Entry*>(it.gl)[e];
            // an entry no record reached gets -0.0f added, which leaves every float (either zero,
            // NaNs included) exactly as it was; storing it anyway keeps the stores of a wave contiguous
#pragma unroll
            for (int f = 0; f < F; ++f)
              cur[j].v[f] = (GT)((float)cur[j].v[f] + (a[f] ? (float)((double)a[f] * inv_scale) : -0.0f));
          }
          reinterpret_cast<Entry*>(it.gl)[e] = cur[j];
        }
      } else if constexpr (sizeof(GT) == 2) {
        // several workgroups share this chunk, half-precision gradient: packed two-half atomics, one
        // lane per aligned pair of halves (two lanes that add to the halves of one word would be
        // served one after the other); the chunk may start on the odd half of a word
        const uint32_t par = (uint32_t)(reinterpret_cast<uintptr_t>(it.gl) >> 1) & 1u;
        const int n_h = (int)(it.n_e * F);
#pragma unroll
        for (int j = 0; j < (F * kPer) / 2 + 1; ++j) {
          const int p = (int)threadIdx.x + j * kAccThreads;
          const int q0 = 2 * p - (int)par;
          float v[2] = {0.0f, 0.0f};
#pragma unroll
          for (int t = 0; t < 2; ++t) {
            const int q = q0 + t;
            if (q < 0 || q >= F * (int)cap) continue;
            unsigned long long* slot = &acc[(q % F) * cap + q / F];
            const long long a = (long long)*slot;
            *slot = 0ull;
            if (q < n_h && a != 0) v[t] = (float)((double)a * inv_scale);
          }
          if (v[0] != 0.0f || v[1] != 0.0f) grad_atomic_add2(it.gl + q0, 0, v[0], v[1]);
        }
      } else {
        // several workgroups share this chunk: fp32 atomics, one lane per float so that the
        // features of an entry and its neighbours travel in the same 64-byte requests
#pragma unroll
        for (int j = 0; j < F * kPer; ++j) {
          const uint32_t q = threadIdx.x + j * kAccThreads;  // float index in the chunk
          const uint32_t e = q / F;
          unsigned long long* slot = &acc[(q % F) * cap + e];
          const long long a = (long long)*slot;
          *slot = 0ull;
          if (e < it.n_e && a != 0) grad_atomic_add(it.gl, q, (float)((double)a * inv_scale));
        }
      }
    }
    __syncthreads();
    item = next;
    next = after_next;
    it = it_n;
#pragma unroll
    for (int j = 0; j < kPer; ++j) cur[j] = cur_n[j];
  }
}

// Level parts of a count or scatter grid for a batch of n_tiles tiles: the plan's, doubled (up to one level per
// part) while the grid would leave most compute units without a workgroup.  A small batch is a few tiles, and a
// workgroup walks the levels of its part one after the other: 2^14 points at Table 1's sizes are 32 tiles, whose
// 128 scatter workgroups took 19 us for four levels each.
static uint32_t parts_for_batch(uint32_t plan_parts, uint32_t L, uint32_t n_tiles) {
  static const uint32_t cus = [] {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
      n = 256;
    return (uint32_t)n;
  }();
  uint32_t parts = plan_parts;
  while (parts < L && (uint64_t)n_tiles * parts < 2ull * cus) parts = parts * 2 < L ? parts * 2 : L;
  return parts;
}

// The count pass by itself: counts[tile][bin] for the B points (x only).
static hg_status launch_count(const hashgrid* h, uint32_t B, const float* x, const Workspace& ws, hipStream_t s) {
  const BinPlan& bp = h->bp;
  const uint32_t L = h->lv.L, cparts = parts_for_batch(bp.count_parts, L, ws.n_tiles);
  uint32_t max_bins = 0;
  for (uint32_t p = 0; p < cparts; ++p) {
    const uint32_t nbp = bp.bin_base[(p + 1) * L / cparts] - bp.bin_base[p * L / cparts];
    max_bins = nbp > max_bins ? nbp : max_bins;
  }
  const bool smooth = h->cfg.interp == HG_INTERP_SMOOTHSTEP;
  const dim3 grid((ws.n_tiles + 7u) / 8u * 8u, cparts);  // see tile_of_workgroup
#define HG_COUNT(D, C)                                                                                              \
  hipLaunchKernelGGL((bin_count<D, C>), grid, dim3(kBinThreads), (size_t)max_bins * 4, s, h->lv, bp, smooth, B, x, \
                     ws.counts, ws.n_bins, ws.n_tiles)
  if (bp.corner_records) {
    if (h->cfg.d == 3) HG_COUNT(3, true);
    else if (h->cfg.d == 2) HG_COUNT(2, true);
    else HG_COUNT(1, true);
  } else {
    if (h->cfg.d == 3) HG_COUNT(3, false);
    else HG_COUNT(2, false);
  }
#undef HG_COUNT
  return hipGetLastError() == hipSuccess ? HG_OK : HG_ERR_DEVICE;
}

template <int D, typename IT, int F, bool CORNERS>
static hg_status launch_binned(const hashgrid* h, uint32_t B, const float* x, const void* dy, void* grad,
                               const Workspace& ws, const bool counted, const bool overwrite, hipStream_t s) {
  const bool g16 = h->cfg.grad_dtype == HG_F16;
  using Rec = Record<IT, F>;
  constexpr uint32_t R = CORNERS ? 1u << D : 1u << (D - 1 > 0 ? D - 1 : 0);
  constexpr int DP = CORNERS ? 2 : D;  // (dimension of the kernels that only the pair records use: never D = 1)
  BinPlan bp = h->bp;
  plan_slices(bp, h->lv, B);
  const bool smooth = h->cfg.interp == HG_INTERP_SMOOTHSTEP;
  const uint32_t n_records = B * h->lv.L * bp.rec_per_point;
  const uint32_t L = h->lv.L, parts = parts_for_batch(bp.scatter_parts, L, ws.n_tiles);
  auto max_part_bins = [&](uint32_t np) {
    uint32_t m = 0;
    for (uint32_t p = 0; p < np; ++p) {
      const uint32_t nbp = bp.bin_base[(p + 1) * L / np] - bp.bin_base[p * L / np];
      m = nbp > m ? nbp : m;
    }
    return m;
  };
  // scatter: staging area, 16-bit bin of every staged record, three words per bin of the part
  constexpr size_t kStagingBytes = (size_t)R * kBinThreads * (Rec::kWords * 4 + 2);
  constexpr size_t kScatterLdsMax = kStagingBytes + (3 * (size_t)kMaxScatterPartBins + 1) * 4;
  // (eight 40-byte records per point do not fit the 160 KiB of a workgroup: such plans scatter unstaged)
  constexpr bool kStaged = kScatterLdsMax <= 160 * 1024;
  constexpr size_t kAccLds = (size_t)F * 8 << chunk_log2_of(F);
  // more dynamic LDS than the default limit of 64 KiB: opt in once per kernel
  static const hipError_t lds_ok = [] {
    hipError_t e = hipSuccess;
    if constexpr (kStaged) {
      if (!CORNERS && kScatterLdsMax > 64 * 1024)
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(bin_scatter<DP, IT, F, true, false>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)kScatterLdsMax);
      if (e == hipSuccess && kScatterLdsMax > 64 * 1024)
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(bin_scatter<D, IT, F, false, CORNERS>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)kScatterLdsMax);
    }
    if (e == hipSuccess && kAccLds > 48 * 1024)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(bin_accumulate<IT, F, false, float>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)kAccLds);
    if (e == hipSuccess && kAccLds > 48 * 1024)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(bin_accumulate<IT, F, true, float>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)kAccLds);
    if (e == hipSuccess && kAccLds > 48 * 1024)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(bin_accumulate<IT, F, false, _Float16>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)kAccLds);
    if (e == hipSuccess && kAccLds > 48 * 1024)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(bin_accumulate<IT, F, true, _Float16>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)kAccLds);
    return e;
  }();
  if (lds_ok != hipSuccess) return HG_ERR_DEVICE;
  const size_t lds_scatter = kStagingBytes + (3 * (size_t)max_part_bins(parts) + 1) * 4;
  const uint32_t tile_wgs = (ws.n_tiles + 7u) / 8u * 8u;  // see tile_of_workgroup
  if (!counted && launch_count(h, B, x, ws, s) != HG_OK) return HG_ERR_DEVICE;
  // HG_BWD_OVERWRITE: the owner of a chunk stores its sums, except on levels whose chunks are summed
  // by several workgroups; those levels are cleared first and added into as usual.  Pairs that
  // straddle two chunks (hashed levels of resolution 2^chunk_log2 or more) get their atomic adds
  // from a pass after the owners have stored.
  uint32_t add_mask = 0, cross_mask = 0;
  for (uint32_t l = 0; l < L; ++l) {
    const bool hashed = !((h->lv.dense_mask >> l) & 1u);
    if (bp.slices[l] > 1) add_mask |= 1u << l;
    if (!CORNERS && hashed && h->lv.N[l] + 1u >= (1u << bp.chunk_log2)) cross_mask |= 1u << l;
  }
  const uint32_t all_levels = L == 32 ? 0xffffffffu : (1u << L) - 1u;
  const uint32_t zero_mask = overwrite ? add_mask : 0u, overwrite_mask = overwrite ? all_levels & ~add_mask : 0u;
  const bool defer_cross = overwrite && cross_mask != 0;  // those atomic adds then follow the accumulate pass
  hipLaunchKernelGGL(bin_scan, dim3((ws.n_bins + kScanBins - 1) / kScanBins), dim3(kScanThreads), 0, s, ws.n_tiles,
                     ws.n_bins, ws.counts, ws.bin_total, ws.item_counter, h->lv, zero_mask, (uint32_t)F, grad, g16);
  auto scatter = [&](auto cross) {
    constexpr bool kCross = decltype(cross)::value;
    constexpr int DS = kCross ? DP : D;  // (the straddling pairs exist with pair records only)
    if (bp.tile_mult > 1 || !kStaged) {
      hipLaunchKernelGGL((bin_scatter_direct<DS, IT, F, kCross, CORNERS && !kCross>), dim3(tile_wgs, parts),
                         dim3(kBinThreads), (size_t)max_part_bins(parts) * 4, s, h->lv, bp, smooth, B, x,
                         static_cast<const IT*>(dy), ws.counts, ws.bin_total, ws.bin_start, ws.records, ws.n_bins,
                         n_records, ws.n_tiles, ws.tile_max, grad, g16);
    } else if constexpr (kStaged) {
      hipLaunchKernelGGL((bin_scatter<DS, IT, F, kCross, CORNERS && !kCross>), dim3(tile_wgs, parts),
                         dim3(kBinThreads), lds_scatter, s, h->lv, bp, smooth, B, x, static_cast<const IT*>(dy),
                         ws.counts, ws.bin_total, ws.bin_start, ws.records, ws.n_bins, n_records, ws.n_tiles,
                         ws.tile_max, grad, g16);
    }
  };
  if (CORNERS || defer_cross || cross_mask == 0)  // no such pairs at these resolutions, or bin_crossing takes them
    scatter(std::false_type{});
  else
    scatter(std::true_type{});
  const uint32_t n_items = bp.wg_base[h->lv.L];
  static const uint32_t acc_slots = [] {  // its registers let one 1024-thread workgroup run per CU; more would queue
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
      cus = 256;
    return (uint32_t)cus * kAccWgsPerCu;
  }();
  const dim3 acc_grid(n_items < acc_slots ? n_items : acc_slots);
  auto accumulate = [&](auto smooth_t, auto* g) {
    using GT = typename std::remove_pointer<decltype(g)>::type;
    hipLaunchKernelGGL((bin_accumulate<IT, F, decltype(smooth_t)::value, GT>), acc_grid, dim3(kAccThreads), kAccLds, s,
                       h->lv, bp, B, n_items, ws.bin_start, ws.bin_total, ws.tile_max, ws.n_tiles * parts, ws.records,
                       ws.item_counter, g, overwrite_mask);
  };
  if (g16) {
    if (smooth) accumulate(std::true_type{}, static_cast<_Float16*>(grad));
    else accumulate(std::false_type{}, static_cast<_Float16*>(grad));
  } else {
    if (smooth) accumulate(std::true_type{}, static_cast<float*>(grad));
    else accumulate(std::false_type{}, static_cast<float*>(grad));
  }
  if (defer_cross)
    hipLaunchKernelGGL((bin_crossing<DP, IT, F>), dim3((B + kBinThreads - 1) / kBinThreads), dim3(kBinThreads), 0, s,
                       h->lv, bp, smooth, B, x, static_cast<const IT*>(dy), cross_mask, grad, g16);
  return hipGetLastError() == hipSuccess ? HG_OK : HG_ERR_DEVICE;
}

template <int D, typename IT, bool CORNERS>
static hg_status launch_binned_f(const hashgrid* h, uint32_t B, const float* x, const void* dy, void* grad,
                                 const Workspace& ws, const bool counted, const bool overwrite, hipStream_t s) {
  switch (h->cfg.F) {
    case 1: return launch_binned<D, IT, 1, CORNERS>(h, B, x, dy, grad, ws, counted, overwrite, s);
    case 2: return launch_binned<D, IT, 2, CORNERS>(h, B, x, dy, grad, ws, counted, overwrite, s);
    case 4: return launch_binned<D, IT, 4, CORNERS>(h, B, x, dy, grad, ws, counted, overwrite, s);
    case 8: return launch_binned<D, IT, 8, CORNERS>(h, B, x, dy, grad, ws, counted, overwrite, s);
    default: return HG_ERR_UNSUPPORTED;
  }
}

template <typename IT>
static hg_status launch_binned_d(const hashgrid* h, uint32_t B, const float* x, const void* dy, void* grad,
                                 const Workspace& ws, const bool counted, const bool overwrite, hipStream_t s) {
  if (h->bp.corner_records) {
    switch (h->cfg.d) {
      case 1: return launch_binned_f<1, IT, true>(h, B, x, dy, grad, ws, counted, overwrite, s);
      case 2: return launch_binned_f<2, IT, true>(h, B, x, dy, grad, ws, counted, overwrite, s);
      default: return launch_binned_f<3, IT, true>(h, B, x, dy, grad, ws, counted, overwrite, s);
    }
  }
  return h->cfg.d == 3 ? launch_binned_f<3, IT, false>(h, B, x, dy, grad, ws, counted, overwrite, s)
                       : launch_binned_f<2, IT, false>(h, B, x, dy, grad, ws, counted, overwrite, s);
}

}  // namespace hg

extern "C" {

uint64_t hashgrid_bwd_workspace_bytes(const hashgrid_t* hg, uint32_t B) {
  if (!hg || !hg->bp.supported || B == 0 || B > HG_MAX_BATCH) return 0;
  if ((uint64_t)B * hg->lv.L * hg->bp.rec_per_point >= (1ull << 32)) return 0;
  return hg::carve(hg, B, nullptr, nullptr);
}

int hashgrid_bwd_ws_pays(const hashgrid_t* hg, uint32_t B) {
  if (hashgrid_bwd_workspace_bytes(hg, B) == 0) return 0;
  // Both passes in microseconds, from measurements on an MI355X.  Sorted pass: about 16 us of
  // launches, 0.017 us per chunk (every chunk of the gradient is visited and rewritten), then the
  // records, written once and read once: ~300 K records of 12 bytes per us, in proportion for
  // larger ones (wider entries, fp32 dL/dy) and twice as many where every corner has its own.
  // Atomic pass: ~6 us, then ~14.5 K pairs of corners per us (11 K at F = 4, 9 K at F = 8: their
  // requests are fatter), unless one 64-byte block of the gradient draws so many requests that
  // they queue up behind each other (~0.02 us each): the smallest level decides that, taking the
  // points as spread evenly over its entries.
  const uint32_t F = hg->cfg.F, d = hg->cfg.d;
  const double pairs = (double)B * hg->lv.L * (1u << (d - 1));
  const double records = (double)B * hg->lv.L * hg->bp.rec_per_point;
  const double rec_bytes = 8.0 + (F * (hg->cfg.io_dtype == HG_F16 ? 2u : 4u) + 3u) / 4u * 4u;
  double per_block = 0.0;
  for (uint32_t l = 0; l < hg->lv.L; ++l) {
    const double blocks = ceil((double)hg->lv.size[l] * F * sizeof(float) / 64.0);
    per_block = fmax(per_block, (double)B * (1u << (d - 1)) / blocks);
  }
  const double pairs_per_us = F <= 2 ? 14.5e3 : F == 4 ? 11e3 : 9e3;
  const double sorted_us = 16.0 + 0.017 * hg->bp.bin_base[hg->lv.L] + records * (rec_bytes / 12.0) / 300e3;
  const double atomic_us = 6.0 + fmax(pairs / pairs_per_us, 0.02 * per_block);
  return atomic_us > sorted_us ? 1 : 0;
}

// shared argument checks of the two entry points that take the scratch buffer
static hg_status check_workspace(const hashgrid_t* hg, uint32_t B, const void* workspace, uint64_t workspace_bytes) {
  const uint64_t need = hashgrid_bwd_workspace_bytes(hg, B);
  if (need == 0) return HG_ERR_UNSUPPORTED;
  if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255)) return HG_ERR_INVALID_ARG;
  return HG_OK;
}

hg_status hashgrid_encode_fwd_ws(const hashgrid_t* hg, uint32_t B, const float* x, const void* params, void* y,
                                 void* workspace, uint64_t workspace_bytes, void* stream) {
  if (!hg) return HG_ERR_INVALID_ARG;
  if (B == 0) return HG_OK;
  const hg_status ok = check_workspace(hg, B, workspace, workspace_bytes);
  if (ok != HG_OK) return ok;
  if (!x || !params || !y || (reinterpret_cast<uintptr_t>(x) & 3)) return HG_ERR_INVALID_ARG;
  hg::Workspace ws;
  hg::carve(hg, B, static_cast<uint8_t*>(workspace), &ws);
  hipStream_t s = static_cast<hipStream_t>(stream);
  // The counting kernel runs full workgroups (they cover whole tiles), which is slow for a batch that
  // cannot give every CU one: there the plain forward in small workgroups plus the count pass is
  // faster and leaves the workspace in the same state.
  // (So it is for plans with a record per corner, which the counting kernel does not serve.)
  if (hg->bp.corner_records || hg::point_major_block(B) < 1024u) {
    const hg_status st = hashgrid_encode_fwd(hg, B, x, params, y, stream);
    return st != HG_OK ? st : hg::launch_count(hg, B, x, ws, s);
  }
  return hg::launch_fwd_counting(hg, B, x, params, y, ws.counts, ws.n_bins, ws.n_tiles, s);
}

hg_status hashgrid_encode_bwd_ws(const hashgrid_t* hg, uint32_t B, const float* x, const void* dLdy,
                                 void* grad_params, void* workspace, uint64_t workspace_bytes, uint32_t flags,
                                 void* stream) {
  if (!hg || (flags & ~(uint32_t)(HG_BWD_COUNTED | HG_BWD_OVERWRITE))) return HG_ERR_INVALID_ARG;
  if (B == 0) return HG_OK;
  const hg_status ok = check_workspace(hg, B, workspace, workspace_bytes);
  if (ok != HG_OK) return ok;
  if (!x || !dLdy || !grad_params) return HG_ERR_INVALID_ARG;
  const size_t io = hg->cfg.io_dtype == HG_F16 ? 2 : 4, F = hg->cfg.F;
  const size_t gs = hg->cfg.grad_dtype == HG_F16 ? 2 : 4;
  // one entry's gradient, up to 16 bytes (and the 4 bytes of a packed atomic at least)
  const size_t grad_align = F * gs > 16 ? 16 : (F * gs < 4 ? 4 : F * gs);
  if ((reinterpret_cast<uintptr_t>(x) & 3) || (reinterpret_cast<uintptr_t>(dLdy) & (F * io - 1) & 15) ||
      (reinterpret_cast<uintptr_t>(grad_params) & (grad_align - 1)))
    return HG_ERR_INVALID_ARG;
  hg::Workspace ws;
  hg::carve(hg, B, static_cast<uint8_t*>(workspace), &ws);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const bool i16 = hg->cfg.io_dtype == HG_F16, counted = flags & HG_BWD_COUNTED, ow = flags & HG_BWD_OVERWRITE;
  return i16 ? hg::launch_binned_d<_Float16>(hg, B, x, dLdy, grad_params, ws, counted, ow, s)
             : hg::launch_binned_d<float>(hg, B, x, dLdy, grad_params, ws, counted, ow, s);
}

// ---------------------------------------------------------------- entry point that allocates nothing
//
// For callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses that
// forbid hipMalloc) and have no workspace to hand over: the scratch of the sorted pass lives in a
// fixed device array that every GPU holds from the moment the library is loaded.
static __device__ __align__(256) unsigned char scratch[HG_STATIC_SCRATCH_BYTES];

namespace hg {
constexpr int kMaxDevices = 64;
// Device address of `scratch` on each GPU (every GPU has its own copy of the array at its own
// address); looked up once per device, with that device current.  In host code the array's name is
// only a handle for this lookup, never an address a kernel could use.
static void* static_scratch_of_current_device() {
  static std::atomic<void*> ptr_of[kMaxDevices];
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  void* p = ptr_of[dev].load(std::memory_order_acquire);
  if (!p) {
    void* q = nullptr;
    if (hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)) != hipSuccess || !q) {
      (void)hipGetLastError();
      return nullptr;
    }
    ptr_of[dev].store(q, std::memory_order_release);  // (two threads racing here store the same address)
    p = q;
  }
  return p;
}
}  // namespace hg

hg_status hashgrid_encode_bwd_static(const hashgrid_t* hg, uint32_t B, const float* x, const void* dLdy,
                                     void* grad_params, uint32_t flags, void* stream) {
  if (!hg || (flags & ~(uint32_t)HG_BWD_OVERWRITE)) return HG_ERR_INVALID_ARG;
  if (B == 0) return HG_OK;
  const uint64_t need = hashgrid_bwd_workspace_bytes(hg, B);
  if (need == 0 || need > HG_STATIC_SCRATCH_BYTES) return HG_ERR_UNSUPPORTED;  // batch too large for the fixed array
  void* ws = hg::static_scratch_of_current_device();
  if (!ws) return HG_ERR_DEVICE;
  // every word of the scratch that a kernel reads is written earlier in the same call (counts by
  // bin_count, totals and the work counter by bin_scan, offsets, records and maxima by bin_scatter),
  // so what the previous call left behind needs no clearing
  return hashgrid_encode_bwd_ws(hg, B, x, dLdy, grad_params, ws, HG_STATIC_SCRATCH_BYTES, flags, stream);
}

}  // extern "C"
