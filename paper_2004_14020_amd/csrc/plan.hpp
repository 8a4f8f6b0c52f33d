// Host-side transfer planner: batching (paper section 4.2), chunking (section 4.4)
// and ring segmentation (sections 2 / 4.4).  Pure C++, no GPU calls.
#pragma once

#include <cstdint>
#include <string>
#include <vector>

#include "caramel.h"

namespace caramel {

struct HostPlan {
  caramel_config cfg{};
  std::vector<uint64_t> tensor_elems;
  std::vector<caramel_unit> units;
  std::vector<caramel_entry> entries;
  std::vector<uint64_t> seg;  // (world + 1) offsets per unit, unit-major
  uint64_t fused_elems = 0;
  // timing-aware plans only (section 4.2): per unit, when it was queued, started and finished
  std::vector<double> enqueue_time, start_time, finish_time;

  uint32_t elem_size() const { return cfg.dtype == CARAMEL_F32 ? 4u : 2u; }
  uint64_t granule() const { return cfg.align_bytes / elem_size(); }
  const uint64_t* segments(uint32_t unit) const { return &seg[size_t(unit) * (cfg.world + 1)]; }
};

// Returns CARAMEL_OK or CARAMEL_EINVAL (with `why` filled in).
// `ready_time` may be NULL (size-only batching); otherwise n non-decreasing update times, and a
// transfer of d bytes is modelled to take net_a + net_b * d.
int build_host_plan(const caramel_config& cfg, const uint64_t* elems, uint32_t n, const double* ready_time,
                    double net_a, double net_b, HostPlan& out, std::string& why);

// Smallest integer x >= 1 with f(2x) / (2 f(x)) > 0.8 for f(d) = a + b*d, decided exactly.
// Returns false if a < 0, b <= 0, a value is not finite, or the result does not fit 64 bits.
bool threshold_from_model(double a, double b, uint64_t& out);

// Canonical little-endian byte image.
std::vector<uint8_t> serialize(const HostPlan& p);

}  // namespace caramel
