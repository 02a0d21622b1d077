// Which bin (chunk of a level's gradient slice) each pair of corners of a point falls into:
// shared by the passes of the binned backward (bwd_binned.hip) and by the forward kernel that
// counts for it (hashgrid.hip).
#pragma once

#include "hashgrid_common.hpp"
#include "hashgrid_internal.hpp"

namespace hg {

constexpr int kBinThreads = 512;      // points of a tile = threads of a count / scatter workgroup (256 and 1024 are slower)
constexpr uint32_t kChunkLog2 = 12;  // log2 of the entries a chunk can hold, at most
// The accumulators of a chunk (F 64-bit words per entry) must fit the LDS of a workgroup: 128 KiB at F = 4 and 8.
__host__ __device__ constexpr uint32_t chunk_log2_of(uint32_t F) { return F <= 4 ? kChunkLog2 : kChunkLog2 - 1; }

template <int D>
struct Rows {
  uint32_t bin[1 << (D - 1)];    // global bin
  uint32_t la[1 << (D - 1)];     // chunk-local index of the lower corner along dimension 0
  float wrow[1 << (D - 1)];      // product of the weights of dimensions 1..d-1
  float wf0;                     // fractional position along dimension 0 (before any smoothstep)
  uint32_t k;                    // trailing one bits of the lower corner's coordinate along dimension 0 (at most 14);
                                 // 15: that coordinate is 0 (the record's k field, see bwd_record.hpp)
  bool cross;                    // hashed level: the pair's corners fall into different chunks (no record)
};

// (also compiled for the host: the plan's invariants are checked there, point by point, without a GPU)
template <int D, bool COUNT_ONLY>
__host__ __device__ __forceinline__ void rows_of(const LevelTable& lv, const BinPlan& bp, uint32_t l, bool smooth,
                                        const float (&xp)[D], Rows<D>& out) {
  const uint32_t N = lv.N[l], verts = lv.verts[l];
  const bool dense = (lv.dense_mask >> l) & 1u;
  const float Nf = (float)N;
  const float shift = smooth ? 0.5f : 0.0f;
  const float cmaxf = smooth ? Nf : Nf - 1.0f;
  uint32_t c0[D];
  float w[D], u[D];
#pragma unroll
  for (int i = 0; i < D; ++i) {
    float wf;
    split(xp[i], Nf, shift, cmaxf, c0[i], wf);
    if (i == 0) out.wf0 = wf;
    w[i] = smooth ? smoothstep(wf) : wf;
    u[i] = smooth ? smoothstep(1.0f - wf) : 1.0f - wf;
  }
  const uint32_t cl = bp.chunk_log2, cmask = (1u << cl) - 1u;
  const uint32_t gb0 = bp.bin_base[l];
  out.cross = !dense && (c0[0] & cmask) == cmask;  // v_0 + 1 carries out of the chunk's index bits
  if (!COUNT_ONLY) {
    // trailing ones of the coordinate; 12 or more never reaches a record (the pair then straddles two
    // chunks); 15 marks the first voxel, whose fractional position the record stores in its second form
    const uint32_t ones = (uint32_t)__builtin_ctz(~c0[0] | 0x4000u);
    out.k = c0[0] == 0u ? 15u : ones;
#pragma unroll
    for (uint32_t r = 0; r < (1u << (D - 1)); ++r) {
      float wr = 1.0f;
#pragma unroll
      for (int i = 1; i < D; ++i) wr *= ((r >> (i - 1)) & 1u) ? w[i] : u[i];
      out.wrow[r] = wr;
    }
  }
  // the level kind is uniform: a scalar branch, not per-lane selects between the two maps
  if (dense) {
    const uint32_t sh = bp.row_shift[l];
#pragma unroll
    for (uint32_t r = 0; r < (1u << (D - 1)); ++r) {
      uint32_t row = c0[1] + (r & 1u);
      if (D == 3) row += (c0[D - 1] + (r >> 1)) * verts;
      const uint32_t bin = row >> sh;
      out.bin[r] = gb0 + bin;
      if (!COUNT_ONLY) {
        const uint32_t la = c0[0] + (row - (bin << sh)) * verts;
        out.la[r] = la;
      }
    }
  } else {
    const uint32_t tmask = lv.T - 1u;
    uint32_t t1[2], t2[2];
    t1[0] = c0[1] * prime(1);
    t1[1] = t1[0] + prime(1);
    t2[0] = D == 3 ? c0[D - 1] * prime(2) : 0u;
    t2[1] = t2[0] + prime(2);
#pragma unroll
    for (uint32_t r = 0; r < (1u << (D - 1)); ++r) {
      const uint32_t rt = D == 3 ? t1[r & 1u] ^ t2[r >> 1] : t1[r & 1u];
      const uint32_t ia = (c0[0] ^ rt) & tmask;
      out.bin[r] = gb0 + (ia >> cl);
      if (!COUNT_ONLY) {
        out.la[r] = ia & cmask;
      }
    }
  }
}

// One record per corner (plans with BinPlan::corner_records: a table size that is not a power of
// two, where the two corners of a pair land in unrelated chunks after Eq. 4's mod T, and d = 1):
// every level's slice is cut into aligned blocks of 2^chunk_log2 entries, a corner belongs to the
// block of its entry.  bin / la as in Rows; weight = the corner's whole interpolation weight.
template <int D>
struct CornerRows {
  uint32_t bin[1 << D];
  uint32_t la[1 << D];
  float weight[1 << D];
};

template <int D, bool COUNT_ONLY>
__host__ __device__ __forceinline__ void corner_rows_of(const LevelTable& lv, const BinPlan& bp, uint32_t l, bool smooth,
                                                        const float (&xp)[D], CornerRows<D>& out) {
  const uint32_t verts = lv.verts[l];
  const bool dense = (lv.dense_mask >> l) & 1u;
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
  const uint32_t cl = bp.chunk_log2, cmask = (1u << cl) - 1u, gb0 = bp.bin_base[l];
#pragma unroll
  for (uint32_t m = 0; m < (1u << D); ++m) {
    uint32_t idx = 0, stride = 1;
    float wt = 1.0f;
#pragma unroll
    for (int i = 0; i < D; ++i) {
      const uint32_t v = c0[i] + ((m >> i) & 1u);
      idx = dense ? idx + v * stride : idx ^ (v * prime(i));
      stride *= verts;
      wt *= ((m >> i) & 1u) ? w[i] : u[i];
    }
    if (!dense) idx = lv.T_is_pow2 ? idx & (lv.T - 1u) : idx % lv.T;
    out.bin[m] = gb0 + (idx >> cl);
    if (!COUNT_ONLY) {
      out.la[m] = idx & cmask;
      out.weight[m] = wt;
    }
  }
}

// Where the k-th record that a tile places into a bin goes inside the tile's run of n records for
// that bin: k * s mod n for a prime s that does not divide n, a bijection of [0, n).  Points that
// follow each other in the batch often share a voxel (samples along a ray), their records would
// sit next to each other, and the accumulate pass, whose 64 lanes take 64 consecutive records,
// would add them to one LDS address in one instruction, served one lane after the other.  With
// the stride such records are at least 67 slots apart.  Short runs (fine levels, where neighbours
// in the batch do not share voxels) stay in order.  n <= 2^12, so every product is below 2^24
// and the float quotient is off by one at most, which the two corrections undo.
__host__ __device__ __forceinline__ uint32_t spread_in_run(const uint32_t k, const uint32_t n) {
  if (n < 128u || k >= n) return k;
  const uint32_t s = (n % 67u) ? 67u : 71u;
  const uint32_t t = k * s;
#if defined(__HIP_DEVICE_COMPILE__)
  const float inv = __builtin_amdgcn_rcpf((float)n);
#else
  const float inv = 1.0f / (float)n;
#endif
  const uint32_t q = (uint32_t)((float)t * inv);
  int32_t m = (int32_t)(t - q * n);
  m = m < 0 ? m + (int32_t)n : m;
  m = m >= (int32_t)n ? m - (int32_t)n : m;
  return (uint32_t)m;
}

// counters[bin] += 1 from every lane that calls (LDS counters, any subset of the wave's lanes);
// returns what a fetch-and-add of 1 would have returned to the lane, in some order of the lanes.
// Lanes that name the same counter in one LDS atomic instruction are served one after the other,
// and neighbouring points of a batch often fall into one bin (all points on a coarse level with
// few bins; samples along a ray).  So the largest groups of the wave, found by comparing with the
// first pending lane's bin, send one add of the group's size each and share out the slots by lane
// rank; the lanes that are left use plain atomics.
constexpr uint32_t kAggregateFrom = 20;  // lanes with one bin from which a common add pays (measured: 8 costs random batches 1%)
template <bool RETURN>
__device__ __forceinline__ uint32_t wave_add_one(uint32_t* counters, const uint32_t bin) {
  uint32_t slot = 0;
  bool todo = true;
#pragma unroll
  for (int round = 0; round < 2; ++round) {
    const uint64_t pending = __ballot(todo);
    if (pending == 0) return slot;  // uniform over the calling lanes
    const uint32_t leader = (uint32_t)__builtin_ctzll(pending);
    const uint32_t bin_l = (uint32_t)__builtin_amdgcn_readlane((int)bin, (int)leader);
    const bool mine = todo && bin == bin_l;
    const uint64_t group = __ballot(mine);
    const uint32_t n = (uint32_t)__popcll(group);
    if (n < kAggregateFrom) break;
    const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(group >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)group, 0u));
    uint32_t base = 0;
    if (mine && rank == 0) base = __hip_atomic_fetch_add(&counters[bin_l], n, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    if (RETURN) {
      base = (uint32_t)__builtin_amdgcn_readlane((int)base, (int)__builtin_ctzll(group));
      slot = mine ? base + rank : slot;
    }
    todo = todo && !mine;
  }
  if (todo) slot = __hip_atomic_fetch_add(&counters[bin], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  return slot;
}

// counters[bin] += 1 from every calling lane (LDS counters), for the histograms of the count pass.
// Points that follow each other in the batch often share a voxel and with it a bin (samples along
// a ray), and lanes that add to one address in one instruction are served one after the other.  So
// where many neighbouring lanes (within a row of 16) name the same bin, only the first lane of a run
// adds, the length of its run; a wave in which few do takes the plain atomic.
constexpr int kRunsFrom = 16;  // lanes of a wave that repeat their neighbour's bin from which the runs are folded
__device__ __forceinline__ void count_one(uint32_t* counters, const uint32_t bin) {
  const uint32_t prev = (uint32_t)__builtin_amdgcn_update_dpp((int)0xffffffffu, (int)bin, 0x111 /* row_shr:1 */, 0xf, 0xf, false);
  // lanes that repeat the bin of their left neighbour in the row of 16, where that neighbour takes part in the
  // call (the register of a lane that does not may hold anything)
  const uint64_t calling = __ballot(true);
  const uint64_t runs = __ballot(prev == bin) & (calling << 1) & 0xfffefffefffefffeull;
  if (__popcll(runs) < kRunsFrom) {  // uniform over the calling lanes
    __hip_atomic_fetch_add(&counters[bin], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    return;
  }
  const uint32_t lane = __lane_id();
  if (!((runs >> lane) & 1ull)) {  // the first lane of a run adds the run's length
    const uint64_t above = lane == 63u ? 0ull : runs >> (lane + 1u);
    __hip_atomic_fetch_add(&counters[bin], 1u + (uint32_t)__builtin_ctzll(~above), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_WORKGROUP);
  }
}

}  // namespace hg
