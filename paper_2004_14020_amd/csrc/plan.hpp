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

  uint32_t elem_size() const { return cfg.dtype == CARAMEL_F32 ? 4u : 2u; }
  uint64_t granule() const { return cfg.align_bytes / elem_size(); }
  const uint64_t* segments(uint32_t unit) const { return &seg[size_t(unit) * (cfg.world + 1)]; }
};

// Returns CARAMEL_OK or CARAMEL_EINVAL (with `why` filled in).
int build_host_plan(const caramel_config& cfg, const uint64_t* elems, uint32_t n, HostPlan& out,
                    std::string& why);

// Canonical little-endian byte image.
std::vector<uint8_t> serialize(const HostPlan& p);

}  // namespace caramel
