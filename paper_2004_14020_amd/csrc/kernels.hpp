// Launch wrappers for the gfx950 kernels.
#pragma once

#include <hip/hip_runtime.h>

#include "tiles.hpp"

namespace caramel {

struct ReduceArgs {
  const ReduceTile* tiles;  // device
  const uint64_t* rows;     // device: (n_rows x W) base pointers
  uint32_t begin, count;    // tile range
  uint32_t world;
  bool bf16;
  bool nontemporal;
  bool tree;          // add as a balanced pairwise tree (halving-doubling) instead of a chain
  uint32_t unroll;    // vectors in flight per lane and worker: 1, 2 or 4 (0 = choose from W)
  uint32_t max_grid;  // 0 = one workgroup per tile
  uint32_t block;     // lanes per workgroup: 256, 512 or 1024
  uint32_t stream_major;  // 0: fetch all workers at once; 2, 4 or 8: walk the workers one by one with
                          // (up to) that many vectors per lane; 8 exists for fp32 chains of at most
                          // 8 workers, everything else gets 4
};

struct CopyArgs {
  const CopyTile* tiles;  // device
  const uint64_t* rows;   // device
  uint32_t begin, count;
  uint32_t world;
  uint32_t fused_row;
  bool bf16;
  bool unpack;  // false: tensors -> fused buffers; true: fused buffers -> tensors
  bool nontemporal;  // streaming loads and stores (for copies too large to stay in the caches)
};

// Ring reduce-scatter arithmetic + 1/W scaling + all-gather for a range of tiles.
hipError_t launch_ring_reduce(const ReduceArgs& a, hipStream_t stream);
// Whether the kernel that launch_ring_reduce picks for this world size handles tiles that straddle
// a segment boundary (ReduceTile::split != 0).  The tile tables must hold none otherwise.
bool reduce_handles_split_tiles(uint32_t world);
// Segmented gather (pack) or scatter (unpack) driven by the copy-tile table.
hipError_t launch_copy(const CopyArgs& a, hipStream_t stream);

}  // namespace caramel
