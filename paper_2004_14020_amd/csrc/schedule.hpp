// Network transfer scheduler (paper section 4.3): greedy packing of the transfer units into
// the backward-pass and forward-pass windows.  Pure C++, no GPU calls.
#pragma once

#include <cstdint>
#include <string>
#include <vector>

#include "caramel.h"
#include "plan.hpp"

namespace caramel {

// Per unit of a plan: its byte size, the update time of its member updated last and the read
// time of its member read first (the unit's transfer boundaries).
void unit_windows(const HostPlan& p, const double* ready_time, const double* read_time, uint64_t* bytes,
                  double* ready, double* need);

// Returns CARAMEL_OK or CARAMEL_EINVAL (with `why` filled in).  `slots` has n entries.
int schedule_transfers(const uint64_t* bytes, const double* ready, const double* need, uint32_t n, double bp_len,
                       double fp_len, double net_a, double net_b, caramel_slot* slots,
                       caramel_schedule_summary* summary, std::string& why);

}  // namespace caramel
