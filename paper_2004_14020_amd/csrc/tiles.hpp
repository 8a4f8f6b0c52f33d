// Descriptor tables that drive the kernels.  Built on the host from a HostPlan, uploaded at
// bind time.  All offsets are in 16-byte vectors relative to a "pointer row": row t < n_tensors
// is tensor t (one base pointer per worker), row n_tensors is the fused workspace.
#pragma once

#include <cstdint>
#include <vector>

#include "plan.hpp"

namespace caramel {

// One workgroup's share of the ring reduction: a run of elements that lies inside ONE ring
// segment, so the chain of workers is the same for every lane.
struct ReduceTile {
  uint32_t row;      // pointer row
  uint32_t first;    // worker whose value is read first: (segment + 1) mod W for the ring, else 0
  uint32_t vec_off;  // offset of the run inside the row, in 16-byte vectors
  uint32_t n_elems;  // elements in the run; only a run that ends a tensor may be ragged
};

// One wavefront's share of pack / unpack: a run of one batch member.
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

struct TileShape {
  uint32_t large_vecs = 4096;        // vectors per reduce tile of a large chunk unit (long launches)
  uint32_t medium_vecs = 1024;       // ... when a stream has too few large units for long launches
  uint32_t small_vecs = 256;         // ... of every other unit
  uint64_t large_bytes = 4u << 20;   // a chunk unit of at least this many bytes per replica is "large"
  uint64_t long_bytes = 64u << 20;   // a stream whose large units total at least this much gets long launches
  uint32_t copy_vecs = 512;          // vectors per copy tile
  uint32_t align_tiles = 1;          // bit 0: small tiles, bit 1: medium tiles start on multiples of their size in memory where possible
};

// A unit whose tiles have the large shape: long uniform runs, worth 1024-lane workgroups.
// Batch units are cut at member boundaries into many short runs and get the small shape.
inline bool is_large_unit(const HostPlan& p, uint32_t unit, const TileShape& ts) {
  const caramel_unit& u = p.units[unit];
  return u.kind == CARAMEL_KIND_CHUNK && u.elems * p.elem_size() >= ts.large_bytes;
}

enum { kLarge = 0, kSmall = 1 };

struct TileTables {
  std::vector<ReduceTile> staged;  // batch units on the fused row, chunk units on tensor rows
  std::vector<ReduceTile> direct;  // batch units addressed through their member tensors
  std::vector<CopyTile> copy;
  // Units appear in the tables class by class, stream by stream: the large units of stream 0,
  // of stream 1, then the small units of stream 0, of stream 1 -- each in unit order.  So the
  // tiles of consecutive units of one class and stream are adjacent, and so are all tiles of
  // one class.
  std::vector<uint32_t> order[2][2];  // [class][stream] -> unit indices
  bool long_launches[2] = {false, false};  // per stream: large units use large_vecs tiles (else medium_vecs)
  std::vector<Range> staged_unit, direct_unit, copy_unit;  // tile range of every unit
};

// `row0_addr`, if given, holds (n_tensors x W) base addresses, tensor-major: large tiles are used
// for a stream only if every large unit of it starts on a multiple of the large tile size in
// every replica (the stream-major kernel is markedly slower on misaligned runs).
void build_tiles(const HostPlan& p, const TileShape& ts, TileTables& out, const uint64_t* row_addr = nullptr);

}  // namespace caramel
