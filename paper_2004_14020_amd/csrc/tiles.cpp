#include "tiles.hpp"

#include <algorithm>

namespace caramel {
namespace {

// One ring segment's part of a run.
struct Part {
  uint32_t first;  // worker whose value is read first
  uint64_t n;      // elements
};

struct Run {
  uint32_t row;
  uint64_t row_elem;  // start inside the row, in elements
  uint64_t n;         // length = sum of the parts
  std::vector<Part> parts;
};

// The tile [at, at + len) of a run: first worker and split position.  Requires that the tile
// touches at most two parts (cut_run cuts it that way).
ReduceTile make_tile(const Run& r, uint64_t at, uint64_t len, uint64_t vec_elems) {
  ReduceTile t{};
  t.row = r.row;
  t.vec_off = uint32_t((r.row_elem + at) / vec_elems);
  t.n_elems = uint32_t(len);
  uint64_t part_begin = 0;
  for (const Part& pt : r.parts) {
    if (at < part_begin + pt.n) {
      t.first = pt.first;
      const uint64_t in_part = part_begin + pt.n - at;  // elements of the tile inside this part
      t.split = in_part < len ? uint32_t(in_part) : 0;
      break;
    }
    part_begin += pt.n;
  }
  return t;
}

// Cut a run into tiles of `tile_elems`.  `phase_elems` is the position of the run's start
// inside a tile-sized block of memory (0 if unknown or not to be used): the first tile is
// shortened so that every later tile starts on a multiple of the tile size in memory.  A tile
// ends early at the second part boundary it would contain (or, without split tiles, at the
// first).  `phases` receives for every tile the position of its start inside such a block.
void cut_run(std::vector<ReduceTile>& out, const Run& r, uint64_t vec_elems, uint64_t tile_elems,
             uint64_t phase_elems, bool split_tiles, uint32_t world, std::vector<uint64_t>& phases) {
  std::vector<uint64_t> bounds;  // ends of the parts, relative to the run
  uint64_t acc = 0;
  for (const Part& pt : r.parts) bounds.push_back(acc += pt.n);
  uint64_t phase = phase_elems % tile_elems;
  for (uint64_t at = 0; at < r.n;) {
    uint64_t len = std::min(tile_elems - phase, r.n - at);
    // the part ends after `at`: the tile may run past the first of them if the sums of the next
    // part start exactly one worker later (what the kernels assume of a split tile)
    const auto lo = std::upper_bound(bounds.begin(), bounds.end(), at);
    const size_t part = size_t(lo - bounds.begin());
    const bool next_is_one_later =
        part + 1 < r.parts.size() && r.parts[part + 1].first == (r.parts[part].first + 1) % world;
    const size_t allowed = split_tiles && next_is_one_later ? 1 : 0;
    if (size_t(bounds.end() - lo) > allowed && lo[allowed] < at + len) len = lo[allowed] - at;
    out.push_back(make_tile(r, at, len, vec_elems));
    phases.push_back(phase);
    at += len;
    phase = (phase + len) % tile_elems;
  }
}

// Cut the last `n_tail` tiles of tiles[begin..] into pieces of at most `piece_elems` elements
// (pieces of a tile stay where the tile was, in order) and move the tile ranges of the units
// along.  phases[i - begin] is the position of tile i's start inside a tile-sized block of
// memory; if the piece size divides the tile size, pieces are cut on multiples of the piece size
// in memory (the first piece of a tile that starts inside such a block is shortened).
void split_tail(std::vector<ReduceTile>& tiles, size_t begin, const std::vector<uint64_t>& phases, uint32_t n_tail,
                uint64_t piece_elems, bool align_pieces, uint64_t vec_elems, uint32_t world,
                std::vector<UnitTiles>& per_unit, const std::vector<uint32_t>& units) {
  const size_t n = tiles.size() - begin;
  if (n == 0) return;
  const size_t first = begin + (n > n_tail ? n - n_tail : 0);
  std::vector<ReduceTile> cut;
  std::vector<uint32_t> grew(tiles.size() - first, 0);  // pieces added per original tile
  for (size_t i = first; i < tiles.size(); ++i) {
    const ReduceTile& t = tiles[i];
    uint32_t pieces = 0;
    const uint64_t ph = align_pieces ? phases[i - begin] % piece_elems : 0;
    uint64_t len = ph ? piece_elems - ph : piece_elems;
    for (uint64_t at = 0; at < t.n_elems; at += len, len = piece_elems, ++pieces) {
      ReduceTile q = t;
      q.vec_off = uint32_t(t.vec_off + at / vec_elems);
      q.n_elems = uint32_t(std::min<uint64_t>(len, t.n_elems - at));
      // where the piece lies relative to the tile's segment boundary
      if (t.split && at >= t.split) {
        q.first = (t.first + 1) % world;
        q.split = 0;
      } else if (t.split && at + q.n_elems > t.split) {
        q.split = uint32_t(t.split - at);
      } else {
        q.split = 0;
      }
      cut.push_back(q);
    }
    grew[i - first] = pieces - 1;
  }
  // unit ranges: a unit's begin moves by the pieces added before it, its count by those inside
  for (uint32_t u : units) {
    Range& r = per_unit[u].tiles[kLong];
    uint32_t before = 0, inside = 0;
    for (size_t i = first; i < tiles.size(); ++i) {
      if (i < r.begin) before += grew[i - first];
      else if (i < size_t(r.begin) + r.count) inside += grew[i - first];
    }
    r.begin += before;
    r.count += inside;
  }
  tiles.resize(first);
  tiles.insert(tiles.end(), cut.begin(), cut.end());
}

}  // namespace

void build_tiles(const HostPlan& p, const TileShape& ts, TileTables& out, const uint64_t* row_addr) {
  out = TileTables{};
  const uint32_t W = p.cfg.world;
  const uint64_t es = p.elem_size();
  const uint64_t ve = 16 / es;  // elements per 16-byte vector
  const uint64_t copy_elems = uint64_t(ts.copy_vecs) * ve;
  const uint32_t fused_row = uint32_t(p.tensor_elems.size());
  const size_t nu = p.units.size();
  out.staged_unit.resize(nu);
  out.direct_unit.resize(nu);
  out.copy_unit.resize(nu);
  for (uint32_t ui = 0; ui < nu; ++ui) out.order[p.units[ui].stream].push_back(ui);

  // Position of a row's element inside an aligned block of `block_elems` elements of memory.
  // Normally it is the same in every replica (tensors at the same offsets of equally aligned
  // arenas); if not, the position most replicas share is taken (the first such, for a tie), so
  // that as many replicas as possible see aligned tiles.  Without addresses: 0.
  std::vector<uint64_t> ph(W);
  auto common_phase = [&](uint32_t row, uint64_t elem, uint64_t block_elems) -> uint64_t {
    if (!row_addr) return 0;
    const uint64_t block_b = block_elems * es;
    for (uint32_t w = 0; w < W; ++w) ph[w] = (row_addr[size_t(row) * W + w] + elem * es) % block_b;
    uint64_t best = ph[0];
    uint32_t best_n = 0;
    for (uint32_t w = 0; w < W; ++w) {
      uint32_t n = 0;
      for (uint32_t x = 0; x < W; ++x) n += ph[x] == ph[w];
      if (n > best_n) best = ph[w], best_n = n;
    }
    return best / es;
  };

  // The runs of a unit in one table, in memory order: a chunk, the unit's region of the fused
  // buffer, or (batch unit reduced in place) each member; every run with its part per segment.
  // Without split tiles a run ends where the first worker changes.
  std::vector<Run> runs;
  auto unit_runs = [&](uint32_t ui, bool direct) {
    runs.clear();
    const caramel_unit& u = p.units[ui];
    const uint64_t* seg = p.segments(ui);
    const caramel_entry* ent = &p.entries[u.first_entry];
    // ring: the chain of segment c starts at worker c+1; the other patterns add in an order
    // that does not depend on the segment and read the workers from 0
    auto first_of = [&](uint32_t c) { return p.cfg.pattern == CARAMEL_PATTERN_RING ? (c + 1) % W : 0u; };
    // [lo, hi) in unit positions, starting at element `row_elem` of `row`
    auto add_run = [&](uint32_t row, uint64_t row_elem, uint64_t lo, uint64_t hi) {
      Run r{row, row_elem, hi - lo, {}};
      for (uint32_t c = 0; c < W; ++c) {
        const uint64_t a = std::max(lo, seg[c]), b = std::min(hi, seg[c + 1]);
        if (a >= b) continue;
        // equal first workers need no boundary between them
        if (!r.parts.empty() && r.parts.back().first == first_of(c)) r.parts.back().n += b - a;
        else r.parts.push_back({first_of(c), b - a});
      }
      if (!r.n) return;
      if (ts.split_tiles) {
        runs.push_back(std::move(r));
        return;
      }
      // tiles that end at segment boundaries: every part is a run of its own
      uint64_t at = 0;
      for (const Part& pt : r.parts) {
        runs.push_back(Run{row, row_elem + at, pt.n, {pt}});
        at += pt.n;
      }
    };
    if (u.kind == CARAMEL_KIND_CHUNK) {
      add_run(ent[0].tensor, ent[0].tensor_off, 0, u.elems);
    } else if (!direct) {
      add_run(fused_row, u.fused_off, 0, u.elems);
    } else {
      for (uint32_t k = 0; k < u.n_entries; ++k)
        add_run(ent[k].tensor, ent[k].tensor_off, ent[k].unit_off, ent[k].unit_off + ent[k].elems);
    }
  };

  for (int table = 0; table < 2; ++table) {
    const bool direct = table == 1;
    std::vector<ReduceTile>& tiles = direct ? out.direct : out.staged;
    std::vector<UnitTiles>& per_unit = direct ? out.direct_unit : out.staged_unit;
    for (int cls = 0; cls < 2; ++cls) {
      const uint64_t tile_elems = uint64_t(cls == kLong ? ts.long_vecs : ts.small_vecs) * ve;
      const bool align = (ts.align_tiles & (cls == kSmall ? 1u : 2u)) != 0;
      for (uint32_t s = 0; s < p.cfg.num_streams; ++s) {
        const size_t stream_begin = tiles.size();
        std::vector<uint64_t> phases;
        for (uint32_t ui : out.order[s]) {
          unit_runs(ui, direct);
          UnitTiles& ut = per_unit[ui];
          ut.tiles[cls].begin = uint32_t(tiles.size());
          for (const Run& r : runs) {
            if ((r.n * es >= ts.long_run_bytes) != (cls == kLong)) continue;
            cut_run(tiles, r, ve, tile_elems, align ? common_phase(r.row, r.row_elem, tile_elems) : 0,
                    ts.split_tiles, W, phases);
            ut.elems[cls] += r.n;
          }
          ut.tiles[cls].count = uint32_t(tiles.size()) - ut.tiles[cls].begin;
        }
        if (cls == kLong && ts.tail_tiles && ts.tail_vecs && ts.tail_vecs < ts.long_vecs)
          split_tail(tiles, stream_begin, phases, ts.tail_tiles, uint64_t(ts.tail_vecs) * ve,
                     align && ts.long_vecs % ts.tail_vecs == 0, ve, W, per_unit, out.order[s]);
      }
    }
  }

  for (uint32_t s = 0; s < p.cfg.num_streams; ++s) {
    out.copy_stream[s].begin = uint32_t(out.copy.size());
    for (uint32_t ui : out.order[s]) {
      const caramel_unit& u = p.units[ui];
      out.copy_unit[ui].begin = uint32_t(out.copy.size());
      if (u.kind == CARAMEL_KIND_BATCH) {
        const caramel_entry* ent = &p.entries[u.first_entry];
        for (uint32_t k = 0; k < u.n_entries; ++k) {
          const caramel_entry& e = ent[k];
          const uint64_t next = (k + 1 < u.n_entries) ? ent[k + 1].unit_off : u.elems;
          for (uint64_t at = 0; at < e.elems; at += copy_elems) {
            CopyTile t{};
            t.row = e.tensor;
            t.t_vec_off = uint32_t((e.tensor_off + at) / ve);
            t.f_vec_off = uint32_t((u.fused_off + e.unit_off + at) / ve);
            t.n_elems = uint32_t(std::min(copy_elems, e.elems - at));
            t.n_zero = (at + copy_elems >= e.elems) ? uint32_t(next - (e.unit_off + e.elems)) : 0;
            out.copy.push_back(t);
          }
        }
      }
      out.copy_unit[ui].count = uint32_t(out.copy.size()) - out.copy_unit[ui].begin;
    }
    out.copy_stream[s].count = uint32_t(out.copy.size()) - out.copy_stream[s].begin;
  }
}

}  // namespace caramel
