// Host-side handle shared by the translation units of libhashgrid.
#pragma once

#include "hashgrid.h"
#include "hashgrid_common.hpp"

namespace hg {

// Plan of the binned backward pass (see bwd_binned.hip): how each level's
// gradient slice is cut into chunks that fit the LDS of one workgroup.
struct BinPlan {
  uint32_t bin_base[HG_MAX_LEVELS + 1];  // first global bin of the level; [L] = number of bins
  uint32_t wg_base[HG_MAX_LEVELS + 1];   // first accumulate-workgroup of the level; [L] = their number
  uint32_t slices[HG_MAX_LEVELS];        // workgroups that share one bin of the level
  uint8_t row_shift[HG_MAX_LEVELS];      // 1:1 levels: log2 of grid rows per chunk
  uint32_t chunk_log2;                   // log2 of the entries a chunk can hold
  uint32_t rec_per_point;                // records per (point, level): 2^(d-1) pairs of corners, or 2^d corners
  uint32_t corner_records;               // 1: one record per corner and every level cut into aligned blocks of
                                         // 2^chunk_log2 entries (T not a power of two, or d = 1); 0: one per pair
  uint32_t count_parts, scatter_parts;   // level parts (gridDim.y) of the count and scatter grids
  uint32_t tile_mult;                    // a tile of the sort = tile_mult * 512 points; above 1: no staging (bin_scatter_direct)
  uint32_t supported;                    // 0: configuration not served by the binned path
};

}  // namespace hg

struct hashgrid {
  hashgrid_config cfg;
  hg::LevelTable lv;
  uint64_t total;
  hg::BinPlan bp;
};

namespace hg {
void build_bin_plan(hashgrid* h);
// hashgrid.hip: threads (= points) per workgroup of the point-major kernels for a batch of B points
uint32_t point_major_block(uint32_t B);
// hashgrid.hip: forward pass that also fills counts[n_tiles][n_bins] of the binned backward pass
hg_status launch_fwd_counting(const hashgrid* h, uint32_t B, const float* x, const void* params, void* y,
                              uint32_t* counts, uint32_t n_bins, uint32_t n_tiles, hipStream_t s);
}
