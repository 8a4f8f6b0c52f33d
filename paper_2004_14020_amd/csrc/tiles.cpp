#include "tiles.hpp"

#include <algorithm>

namespace caramel {
namespace {

// Cut the run of `n` elements that starts at element `row_elem` of a row into tiles.  `phase` is
// the byte address of the run's start modulo the tile size (0 if unknown): the first tile is
// shortened so that every later tile starts on a multiple of the tile size in memory.
void cut_run(std::vector<ReduceTile>& out, uint32_t row, uint32_t first, uint64_t row_elem, uint64_t n,
             uint64_t vec_elems, uint64_t tile_elems, uint64_t phase_elems) {
  uint64_t len = phase_elems ? tile_elems - phase_elems : tile_elems;
  for (uint64_t at = 0; at < n; at += len, len = tile_elems) {
    ReduceTile t;
    t.row = row;
    t.first = first;
    t.vec_off = uint32_t((row_elem + at) / vec_elems);
    t.n_elems = uint32_t(std::min(len, n - at));
    out.push_back(t);
  }
}

}  // namespace

void build_tiles(const HostPlan& p, const TileShape& ts, TileTables& out, const uint64_t* row_addr) {
  out = TileTables{};
  const uint32_t W = p.cfg.world;
  const uint64_t ve = 16 / p.elem_size();  // elements per 16-byte vector
  const uint64_t copy_elems = uint64_t(ts.copy_vecs) * ve;
  const uint32_t fused_row = uint32_t(p.tensor_elems.size());
  const size_t nu = p.units.size();
  out.staged_unit.resize(nu);
  out.direct_unit.resize(nu);
  out.copy_unit.resize(nu);
  uint64_t large_total[2] = {0, 0};
  bool aligned[2] = {true, true};
  const uint64_t tile_bytes = uint64_t(ts.large_vecs) * 16;
  for (uint32_t ui = 0; ui < nu; ++ui) {
    const bool large = is_large_unit(p, ui, ts);
    const uint32_t s = p.units[ui].stream;
    out.order[large ? kLarge : kSmall][s].push_back(ui);
    if (!large) continue;
    large_total[s] += p.units[ui].elems * p.elem_size();
    if (row_addr) {
      const caramel_entry& e = p.entries[p.units[ui].first_entry];
      for (uint32_t w = 0; w < W; ++w)
        if ((row_addr[size_t(e.tensor) * W + w] + e.tensor_off * p.elem_size()) % tile_bytes) aligned[s] = false;
    }
  }
  for (int s = 0; s < 2; ++s)
    out.long_launches[s] = large_total[s] >= ts.long_bytes && large_total[s] > 0 && aligned[s];

  // Position of a row's element inside an aligned tile-sized block of memory, in elements, if it
  // is the same in every replica (else, or without addresses, 0: tiles start where the run starts).
  auto phase = [&](uint32_t row, uint64_t elem, uint64_t tile_elems, int cls) -> uint64_t {
    if (!row_addr || !(ts.align_tiles & (cls == kSmall ? 1u : 2u))) return 0;
    const uint64_t tile_b = tile_elems * p.elem_size();
    const uint64_t ph = (row_addr[size_t(row) * W] + elem * p.elem_size()) % tile_b;
    for (uint32_t w = 1; w < W; ++w)
      if ((row_addr[size_t(row) * W + w] + elem * p.elem_size()) % tile_b != ph) return 0;
    return ph / p.elem_size();
  };

  for (int cls = 0; cls < 2; ++cls)
    for (uint32_t s = 0; s < p.cfg.num_streams; ++s)
      for (uint32_t ui : out.order[cls][s]) {
        const caramel_unit& u = p.units[ui];
        const uint64_t* seg = p.segments(ui);
        const caramel_entry* ent = &p.entries[u.first_entry];
        const uint64_t tile_elems =
            uint64_t(cls == kSmall ? ts.small_vecs : (out.long_launches[s] ? ts.large_vecs : ts.medium_vecs)) * ve;
        out.staged_unit[ui].begin = uint32_t(out.staged.size());
        out.direct_unit[ui].begin = uint32_t(out.direct.size());
        out.copy_unit[ui].begin = uint32_t(out.copy.size());

        for (uint32_t c = 0; c < W; ++c) {
          const uint64_t a = seg[c], b = seg[c + 1];
          if (a == b) continue;
          // ring: the chain of segment c starts at worker c+1; the other patterns add in an
          // order that does not depend on the segment and read the workers from 0
          const uint32_t first = p.cfg.pattern == CARAMEL_PATTERN_RING ? (c + 1) % W : 0;
          if (u.kind == CARAMEL_KIND_CHUNK) {
            const uint64_t ph = phase(ent[0].tensor, ent[0].tensor_off + a, tile_elems, cls);
            cut_run(out.staged, ent[0].tensor, first, ent[0].tensor_off + a, b - a, ve, tile_elems, ph);
            cut_run(out.direct, ent[0].tensor, first, ent[0].tensor_off + a, b - a, ve, tile_elems, ph);
            continue;
          }
          cut_run(out.staged, fused_row, first, u.fused_off + a, b - a, ve, tile_elems,
                  phase(fused_row, u.fused_off + a, tile_elems, cls));
          for (uint32_t k = 0; k < u.n_entries; ++k) {
            const caramel_entry& e = ent[k];
            const uint64_t lo = std::max(a, e.unit_off), hi = std::min(b, e.unit_off + e.elems);
            if (lo >= hi) continue;
            const uint64_t te = e.tensor_off + (lo - e.unit_off);
            cut_run(out.direct, e.tensor, first, te, hi - lo, ve, tile_elems, phase(e.tensor, te, tile_elems, cls));
          }
        }

        if (u.kind == CARAMEL_KIND_BATCH) {
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
        out.staged_unit[ui].count = uint32_t(out.staged.size()) - out.staged_unit[ui].begin;
        out.direct_unit[ui].count = uint32_t(out.direct.size()) - out.direct_unit[ui].begin;
        out.copy_unit[ui].count = uint32_t(out.copy.size()) - out.copy_unit[ui].begin;
      }
}

}  // namespace caramel
