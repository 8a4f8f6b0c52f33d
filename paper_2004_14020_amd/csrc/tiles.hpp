// Descriptor tables that drive the kernels.  Built on the host from a HostPlan, uploaded at
// bind time.  All offsets are in 16-byte vectors relative to a "pointer row": row t < n_tensors
// is tensor t (one base pointer per worker), row n_tensors is the fused workspace.
#pragma once

#include <cstdint>
#include <vector>

#include "plan.hpp"

namespace caramel {

// One workgroup's share of the ring reduction: a piece of one row that lies inside one ring
// segment, or straddles the boundary between two consecutive ones.  Inside a segment the chain of
// workers is the same for every lane; the sums of the next segment start one worker later.
struct ReduceTile {
  uint32_t row;      // pointer row
  uint32_t first;    // worker whose value is read first: (segment + 1) mod W for the ring, else 0
  uint32_t vec_off;  // offset of the piece inside the row, in 16-byte vectors
  uint32_t n_elems;  // elements in the piece; only a piece that ends a tensor may be ragged
  uint32_t split;    // 0, or the number of elements that belong to the first of two segments (a
                     // multiple of the vector size): the sums of the elements from `split` on
                     // start at worker first + 1 (mod W)
  uint32_t pad_[3];
};

// One workgroup's share of pack / unpack: a run of one batch member.
struct CopyTile {
  uint32_t row;        // tensor row
  uint32_t t_vec_off;  // offset inside the tensor, in vectors
  uint32_t f_vec_off;  // offset inside a replica's fused buffer, in vectors
  uint32_t n_elems;    // elements to copy
  uint32_t n_zero;     // padding elements that follow in the fused buffer (pack writes +0.0)
  uint32_t pad_[3];
};

struct Range {
  uint32_t begin = 0, count = 0;
};

// A run is a maximal contiguous piece of one row (a tensor, or the fused buffer) that belongs to
// one unit: a whole chunk, a whole member of a batch unit reduced in place, or a batch unit's
// region of the fused buffer.  It consists of one part per ring segment it crosses.  Runs are
// cut into tiles along aligned blocks of memory, whatever the segment boundaries; a tile that
// contains a boundary carries its position (`split`), and where a tile would contain two, it
// ends at the second.  Long runs are cut into long tiles, for 1024-lane workgroups that walk the
// replicas one after the other; the rest into small tiles, for 256-lane workgroups that fetch
// all replicas at once.
struct TileShape {
  uint32_t long_vecs = 0;              // vectors per long tile; 0 (options only) = chosen at bind: 4096 or 8192
  uint32_t small_vecs = 256;           // vectors per small tile
  uint64_t long_run_bytes = 0;         // a run of at least this many bytes per replica is long; 0 (options only) = chosen at bind
  uint32_t copy_vecs = 1024;           // vectors per copy tile: one per lane of the copy kernel's workgroup
  // Where every replica of a run has the same address modulo the tile size, the first tile of
  // the run is shortened so that all later ones start on multiples of the tile size in memory
  // (bit 0: small tiles, bit 1: long tiles).
  uint32_t align_tiles = 3;
  bool split_tiles = false;  // tiles may straddle a segment boundary (set at bind if the kernel handles them)
  // The last `tail_tiles` long tiles of every stream are cut into pieces of `tail_vecs` vectors:
  // when a launch runs out of tiles the workgroups still at work finish at different times, and
  // with short pieces at the end that drain is short.
  uint32_t tail_tiles = 128;
  uint32_t tail_vecs = 1024;
};

enum { kLong = 0, kSmall = 1 };


struct UnitTiles {
  Range tiles[2];                // [class] range in the table
  uint64_t elems[2] = {0, 0};    // [class] elements covered
};

struct TileTables {
  // Both reduce tables are ordered class by class, stream by stream, unit by unit: the long
  // tiles of the units of stream 0, of stream 1, then the small tiles likewise.  So the tiles of
  // one class of consecutive units of a stream are adjacent.
  std::vector<ReduceTile> staged;  // batch units on the fused row, chunk units on tensor rows
  std::vector<ReduceTile> direct;  // batch units addressed through their member tensors
  std::vector<CopyTile> copy;      // stream by stream, unit by unit
  std::vector<uint32_t> order[2];  // [stream] -> its units, in plan order
  std::vector<UnitTiles> staged_unit, direct_unit;
  std::vector<Range> copy_unit;
  Range copy_stream[2];            // copy tiles of all batch units of a stream
};

// `row_addr`, if given, holds (n_tensors + 1) x W base addresses, row-major (the last row is
// the fused workspace; zeros if there is none): needed to cut tiles on aligned blocks.
void build_tiles(const HostPlan& p, const TileShape& ts, TileTables& out, const uint64_t* row_addr = nullptr);

}  // namespace caramel
