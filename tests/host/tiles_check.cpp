// Host-only check of the planner and the tile tables, built with AddressSanitizer and UBSan.
// For random configurations it verifies what the kernels rely on: every tile stays inside
// its row, starts on a 16-byte vector, lies inside one ring segment with the right first
// worker -- or straddles one boundary between two segments whose chains start one worker apart,
// at the position the tile names --, and the tiles of a table cover every element exactly once.
#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <map>
#include <random>
#include <string>
#include <vector>

#include "plan.hpp"
#include "schedule.hpp"
#include "tiles.hpp"

using namespace caramel;

static int fails = 0;
#define CHECK(c)                                                        \
  do {                                                                  \
    if (!(c)) {                                                         \
      std::printf("FAIL %s:%d  %s\n", __FILE__, __LINE__, #c);          \
      if (++fails > 20) std::exit(1);                                   \
    }                                                                   \
  } while (0)

static void check_case(const caramel_config& cfg, const std::vector<uint64_t>& elems, uint32_t tile_vecs,
                       uint32_t small_vecs, uint64_t long_run_bytes, uint32_t copy_vecs, uint64_t addr_seed) {
  HostPlan p;
  std::string why;
  const int rc = build_host_plan(cfg, elems.data(), uint32_t(elems.size()), nullptr, 0.0, 0.0, p, why);
  CHECK(rc == CARAMEL_OK);
  if (rc != CARAMEL_OK) return;
  TileTables tt;
  TileShape shape;
  shape.long_vecs = tile_vecs;
  shape.small_vecs = small_vecs;
  shape.long_run_bytes = long_run_bytes;
  shape.copy_vecs = copy_vecs;
  shape.align_tiles = uint32_t(addr_seed >> 8) & 3u;
  shape.tail_tiles = (addr_seed >> 10) & 1 ? 0 : uint32_t(1 + (addr_seed >> 11) % 40);
  shape.tail_vecs = (addr_seed >> 17) & 1 ? 64 : 16;
  shape.split_tiles = ((addr_seed >> 18) & 1) != 0;
  // addr_seed 0: no addresses (tiles start where runs start).  Otherwise made-up base addresses,
  // aligned as bind demands; odd seeds give every replica the same position inside a tile-sized
  // block (tiles must then start on multiples of the tile size), even seeds different ones.
  const uint64_t es = p.elem_size(), ve = 16 / es, W = cfg.world;
  const uint32_t fused_row = uint32_t(elems.size());
  std::vector<uint64_t> addr;
  if (addr_seed) {
    std::mt19937_64 ar(addr_seed);
    addr.resize((elems.size() + 1) * W);
    for (size_t row = 0; row <= elems.size(); ++row) {
      const uint64_t common = (ar() % 4096) * cfg.align_bytes;
      for (uint64_t w = 0; w < W; ++w)
        addr[row * W + w] = (uint64_t(1) << 40) * (w + 1) + (uint64_t(row) << 32) +
                            ((addr_seed & 1) ? common : (ar() % 4096) * cfg.align_bytes);
    }
  }
  build_tiles(p, shape, tt, addr_seed ? addr.data() : nullptr);
  auto row_elems = [&](uint32_t row) { return row == fused_row ? p.fused_elems : elems[row]; };

  for (int table = 0; table < 2; ++table) {
    const std::vector<ReduceTile>& tiles = table ? tt.direct : tt.staged;
    const std::vector<UnitTiles>& per_unit = table ? tt.direct_unit : tt.staged_unit;
    // coverage counters per row
    std::map<uint32_t, std::vector<uint8_t>> seen;
    uint64_t total_tiles = 0;
    for (uint32_t u = 0; u < p.units.size(); ++u) {
      const caramel_unit& un = p.units[u];
      const uint64_t* seg = p.segments(u);
      uint64_t covered[2] = {0, 0};
      for (int cls = 0; cls < 2; ++cls) {
        const Range r = per_unit[u].tiles[cls];
        const uint64_t cap = uint64_t(cls == kLong ? tile_vecs : small_vecs);
        CHECK(uint64_t(r.begin) + r.count <= tiles.size());
        total_tiles += r.count;
        uint32_t prev_row = ~0u, prev_last_first = ~0u;
        uint64_t prev_end = ~0ull;
        // first worker of a tile's last element
        auto last_first = [&](const ReduceTile& t) { return t.split ? (t.first + 1) % uint32_t(W) : t.first; };
        // consecutive tiles of one run: adjacent in the same row and, where tiles end at segment
        // boundaries, of the same segment (a ring run's first worker identifies its segment; the
        // other patterns have first == 0 everywhere and their segments form one run)
        auto same_run = [&](const ReduceTile& a, const ReduceTile& b) {
          return a.row == b.row && uint64_t(a.vec_off) * ve + a.n_elems == uint64_t(b.vec_off) * ve &&
                 (shape.split_tiles || last_first(a) == b.first);
        };
        auto run_len = [&](uint32_t i) {
          uint32_t lo = i, hi = i;
          while (lo > r.begin && same_run(tiles[lo - 1], tiles[lo])) --lo;
          while (hi + 1 < r.begin + r.count && same_run(tiles[hi], tiles[hi + 1])) ++hi;
          uint64_t n = 0;
          for (uint32_t k = lo; k <= hi; ++k) n += tiles[k].n_elems;
          return n;
        };
        for (uint32_t i = r.begin; i < r.begin + r.count; ++i) {
          const ReduceTile& t = tiles[i];
          CHECK(t.n_elems > 0 && t.n_elems <= cap * ve);
          CHECK(t.first < W);
          CHECK(t.row <= fused_row);
          const uint64_t e0 = uint64_t(t.vec_off) * ve, e1 = e0 + t.n_elems;
          CHECK(e1 <= row_elems(t.row));
          covered[cls] += t.n_elems;
          // ragged only at the very end of a tensor row (the fused row is whole granules)
          if (t.n_elems % ve) CHECK(t.row != fused_row && e1 == elems[t.row]);
          // position inside the unit -> segment -> first worker
          uint64_t unit_pos = ~0ull;
          if (un.kind == CARAMEL_KIND_CHUNK) {
            const caramel_entry& e = p.entries[un.first_entry];
            CHECK(t.row == e.tensor && e0 >= e.tensor_off && e1 <= e.tensor_off + e.elems);
            unit_pos = e0 - e.tensor_off;
          } else if (t.row == fused_row) {
            CHECK(table == 0 && e0 >= un.fused_off && e1 <= un.fused_off + un.elems);
            unit_pos = e0 - un.fused_off;
          } else {
            CHECK(table == 1);
            bool found = false;
            for (uint32_t k = 0; k < un.n_entries; ++k) {
              const caramel_entry& e = p.entries[un.first_entry + k];
              if (e.tensor == t.row) {
                CHECK(e0 >= e.tensor_off && e1 <= e.tensor_off + e.elems);
                unit_pos = e.unit_off + (e0 - e.tensor_off);
                found = true;
              }
            }
            CHECK(found);
          }
          // every element's segment -> the worker its sum starts at
          CHECK(t.split % ve == 0 && t.split < t.n_elems);
          if (!shape.split_tiles) CHECK(t.split == 0);
          uint32_t c = 0;
          for (uint64_t k = 0; k < t.n_elems; ++k) {
            while (c + 1 < W && seg[c + 1] <= unit_pos + k) ++c;
            CHECK(unit_pos + k >= seg[c] && unit_pos + k < seg[c + 1]);
            const uint32_t want = cfg.pattern == CARAMEL_PATTERN_RING ? uint32_t((c + 1) % W) : 0u;
            const uint32_t have = (t.split && k >= t.split) ? uint32_t((t.first + 1) % W) : t.first;
            if (have != want) {
              CHECK(have == want);
              break;
            }
          }
          // a boundary the tile names is a real one
          if (t.split) CHECK(cfg.pattern == CARAMEL_PATTERN_RING && W > 1);
          // the class follows the length of the run
          const uint64_t rl = run_len(i) * es;
          if (cls == kLong) CHECK(rl >= long_run_bytes);
          else CHECK(rl < long_run_bytes);
          if ((addr_seed & 1) && (shape.align_tiles & (cls == kLong ? 2u : 1u))) {
            // same phase in every replica: a tile that does not begin its run begins an aligned
            // block, unless the tile before it had to end at a segment boundary (a tile holds at
            // most one)
            const bool at_boundary = std::find(seg, seg + W + 1, unit_pos) != seg + W + 1;
            const bool continues = i > r.begin && prev_row == t.row && prev_end == e0 && !at_boundary &&
                                   (shape.split_tiles || prev_last_first == t.first);
            // (pieces of the tiles cut up at the end of a stream start on multiples of the piece size)
            const uint64_t block = cls == kLong && shape.tail_tiles ? std::min<uint64_t>(cap, shape.tail_vecs) : cap;
            if (continues) CHECK((addr[size_t(t.row) * W] + e0 * es) % (block * 16) == 0);
          }
          prev_row = t.row;
          prev_end = e1;
          prev_last_first = last_first(t);
          std::vector<uint8_t>& s = seen[t.row];
          if (s.empty()) s.assign(row_elems(t.row), 0);
          for (uint64_t e = e0; e < e1; ++e) {
            CHECK(s[e] == 0);
            s[e] = 1;
          }
        }
        CHECK(covered[cls] == per_unit[u].elems[cls]);
      }
      // a unit's tiles cover its elements (the padding of a batch unit only in the fused buffer)
      uint64_t want = un.elems;
      if (un.kind == CARAMEL_KIND_BATCH && table == 1) {
        want = 0;
        for (uint32_t k = 0; k < un.n_entries; ++k) want += p.entries[un.first_entry + k].elems;
      }
      CHECK(covered[0] + covered[1] == want);
    }
    CHECK(total_tiles == tiles.size());
    // tensors: every element exactly once, except members of batch units in the staged table
    std::vector<bool> in_batch(elems.size(), false);
    for (const caramel_entry& e : p.entries)
      if (p.units[e.unit].kind == CARAMEL_KIND_BATCH) in_batch[e.tensor] = true;
    for (uint32_t t = 0; t < elems.size(); ++t) {
      const bool expect = table == 1 || !in_batch[t];
      const std::vector<uint8_t>& s = seen[t];
      if (!expect) {
        CHECK(s.empty());
        continue;
      }
      CHECK(s.size() == elems[t]);
      CHECK(std::all_of(s.begin(), s.end(), [](uint8_t b) { return b == 1; }));
    }
    if (table == 0 && p.fused_elems) {
      const std::vector<uint8_t>& s = seen[fused_row];
      CHECK(s.size() == p.fused_elems && std::all_of(s.begin(), s.end(), [](uint8_t b) { return b == 1; }));
    }
    // the unit ranges follow one another in the documented order: long tiles of the units of
    // stream 0, of stream 1, then the small tiles likewise
    uint32_t at = 0;
    for (int cls = 0; cls < 2; ++cls)
      for (uint32_t s = 0; s < cfg.num_streams; ++s)
        for (uint32_t u : tt.order[s]) {
          CHECK(p.units[u].stream == s);
          CHECK(per_unit[u].tiles[cls].begin == at);
          at += per_unit[u].tiles[cls].count;
        }
    CHECK(at == tiles.size());
  }

  // copy tiles: members of batch units, with the zero padding that follows each member
  std::vector<uint8_t> fused_seen(p.fused_elems, 0);
  for (const CopyTile& t : tt.copy) {
    CHECK(t.row < fused_row && t.n_elems > 0 && t.n_elems <= uint64_t(copy_vecs) * ve);
    const uint64_t t0 = uint64_t(t.t_vec_off) * ve, f0 = uint64_t(t.f_vec_off) * ve;
    CHECK(t0 + t.n_elems <= elems[t.row]);
    CHECK(f0 + t.n_elems + t.n_zero <= p.fused_elems);
    if (t.n_elems % ve) CHECK(t0 + t.n_elems == elems[t.row]);
    for (uint64_t e = f0; e < f0 + t.n_elems + t.n_zero; ++e) {
      CHECK(fused_seen[e] == 0);
      fused_seen[e] = 1;
    }
  }
  CHECK(std::all_of(fused_seen.begin(), fused_seen.end(), [](uint8_t b) { return b == 1; }));
}

// The scheduler on random inputs: one slot per group, inside its boundary, no two slots of a
// window overlapping -- and no out-of-bounds access or undefined behaviour on the way.
void check_schedule(std::mt19937_64& rng) {
  const uint32_t n = uint32_t(rng() % 60);
  const double bp = double(1 + rng() % 40), fp = double(1 + rng() % 40);
  std::vector<uint64_t> bytes(n);
  std::vector<double> ready(n), need(n);
  for (uint32_t g = 0; g < n; ++g) {
    bytes[g] = 1 + rng() % 5000;
    ready[g] = bp * double(rng() % 1000) / 999.0;
    need[g] = fp * double(rng() % 1000) / 999.0;
    if (ready[g] > bp) ready[g] = bp;
    if (need[g] > fp) need[g] = fp;
  }
  std::vector<caramel_slot> slots(n);
  caramel_schedule_summary sum{};
  std::string why;
  const double a = double(rng() % 4) * 0.25, b = 1e-3 * double(1 + rng() % 8);
  CHECK(schedule_transfers(bytes.data(), ready.data(), need.data(), n, bp, fp, a, b, slots.data(), &sum, why) ==
        CARAMEL_OK);
  for (uint32_t g = 0; g < n; ++g) {
    const caramel_slot& s = slots[g];
    CHECK(s.stage == 2 || s.stage == 3);
    CHECK(s.end > s.start);
    if (s.bin == CARAMEL_BIN_BACKWARD) {
      CHECK(s.start >= ready[g] && (s.stage == 3 || s.end <= bp));
    } else {
      CHECK(s.bin == CARAMEL_BIN_FORWARD && s.end <= need[g] && (s.stage == 3 || s.start >= 0.0));
    }
    for (uint32_t h = 0; h < g; ++h)
      CHECK(slots[h].bin != s.bin || !(slots[h].start < s.end && s.start < slots[h].end));
  }
  CHECK(sum.iteration_time >= sum.compute_time && sum.utilization <= 1.0);
  CHECK(schedule_transfers(bytes.data(), ready.data(), need.data(), n, -1.0, fp, a, b, slots.data(), &sum, why) ==
        CARAMEL_EINVAL);
}

int main() {
  std::mt19937_64 rng(20041402);
  for (int it = 0; it < 300; ++it) check_schedule(rng);
  auto pick = [&](std::initializer_list<uint64_t> xs) {
    std::vector<uint64_t> v(xs);
    return v[rng() % v.size()];
  };
  for (int it = 0; it < 600; ++it) {
    caramel_config cfg{};
    cfg.world = uint32_t(pick({1, 2, 3, 4, 5, 7, 8, 16, 33, 64}));
    cfg.dtype = uint32_t(rng() % 2);
    cfg.align_bytes = uint32_t(pick({16, 16, 32, 64, 256}));
    cfg.batch_threshold_bytes = pick({0, 64, 256, 1024, 4096, 1000, 65536});
    cfg.split_mode = uint32_t(rng() % 3);
    cfg.max_depth = uint32_t(pick({1, 2, 8}));
    cfg.split_bytes = cfg.split_mode ? pick({1, 2, 4, 16, 64}) * std::max<uint64_t>(cfg.align_bytes, 64) : 0;
    cfg.num_streams = uint32_t(1 + rng() % 2);
    cfg.pattern = uint32_t(rng() % 3);
    if (cfg.pattern == CARAMEL_PATTERN_HALVING_DOUBLING) cfg.world = uint32_t(pick({1, 2, 4, 8, 16, 32, 64}));
    std::vector<uint64_t> elems(1 + rng() % 14);
    for (uint64_t& e : elems) e = pick({1, 2, 3, 5, 8, 17, 64, 100, 255, 256, 257, 1000, 4096, 5000, 70000});
    check_case(cfg, elems, uint32_t(pick({64, 256, 1024, 4096})), uint32_t(pick({64, 256, 1024})),
               pick({0, 256, 1024, 16384, 65536, 1u << 22}), uint32_t(pick({64, 512})), it % 3 == 0 ? 0 : rng());
  }
  // rejected configurations must not crash
  HostPlan p;
  std::string why;
  caramel_config bad{};
  uint64_t one = 1;
  CHECK(build_host_plan(bad, &one, 1, nullptr, 0.0, 0.0, p, why) == CARAMEL_EINVAL);
  CHECK(build_host_plan(bad, nullptr, 1, nullptr, 0.0, 0.0, p, why) == CARAMEL_EINVAL);
  if (fails) {
    std::printf("%d checks failed\n", fails);
    return 1;
  }
  std::printf("tiles_check ok\n");
  return 0;
}
