// Network transfer scheduler (paper section 4.3).
//
// The network carries one transfer at a time.  Each window keeps its placed transfers as a
// list of disjoint intervals sorted by time, and a new transfer is slid from its boundary
// away from it -- later in the backward pass, earlier in the forward pass -- past every
// interval it collides with, until it lies in free time.  The two windows are mirror images:
// the forward window is handled by the same sweep on negated times.
#include "schedule.hpp"

#include <algorithm>
#include <limits>
#include <numeric>

namespace caramel {
namespace {

struct Interval {
  double from, to;  // in the window's own direction: from <= to
};

// One window, seen in the direction in which transfers are pushed away from their boundary.
// Backward pass: x = t.  Forward pass: x = -t, so "at or before the read time" becomes "at or
// after -read time" and "not before the pass starts" becomes "x <= 0".
class Window {
 public:
  // Nearest free position at or beyond `boundary` for a transfer of length `dur`.
  double slide(double boundary, double dur) const {
    double x = boundary;
    for (const Interval& iv : busy_) {            // sorted by `from`
      if (iv.from < x + dur && x < iv.to) x = iv.to;
    }
    return x;
  }
  void occupy(double from, double to) {
    Interval iv{from, to};
    busy_.insert(std::upper_bound(busy_.begin(), busy_.end(), iv,
                                  [](const Interval& a, const Interval& b) { return a.from < b.from; }),
                 iv);
    reach_ = std::max(reach_, to);
  }
  // Farthest point any transfer reaches, at least `floor`.
  double reach(double floor) const { return std::max(floor, reach_); }

 private:
  std::vector<Interval> busy_;
  double reach_ = -std::numeric_limits<double>::infinity();
};

}  // namespace

void unit_windows(const HostPlan& p, const double* ready_time, const double* read_time, uint64_t* bytes,
                  double* ready, double* need) {
  for (size_t u = 0; u < p.units.size(); ++u) {
    const caramel_unit& un = p.units[u];
    double last_update = -std::numeric_limits<double>::infinity();
    double first_read = std::numeric_limits<double>::infinity();
    for (uint32_t k = 0; k < un.n_entries; ++k) {
      const uint32_t t = p.entries[un.first_entry + k].tensor;
      last_update = std::max(last_update, ready_time[t]);
      first_read = std::min(first_read, read_time[t]);
    }
    bytes[u] = un.elems * p.elem_size();
    ready[u] = last_update;
    need[u] = first_read;
  }
}

int schedule_transfers(const uint64_t* bytes, const double* ready, const double* need, uint32_t n, double bp_len,
                       double fp_len, double net_a, double net_b, caramel_slot* slots,
                       caramel_schedule_summary* summary, std::string& why) {
  auto bad = [&](const char* m) {
    why = m;
    return CARAMEL_EINVAL;
  };
  if (n > 0 && (!bytes || !ready || !need || !slots)) return bad("NULL argument");
  if (!(bp_len >= 0.0) || !(fp_len >= 0.0) || !(net_a >= 0.0) || !(net_b >= 0.0))
    return bad("pass lengths and model coefficients must be non-negative");
  std::vector<double> dur(n);
  for (uint32_t g = 0; g < n; ++g) {
    if (!(0.0 <= ready[g] && ready[g] <= bp_len)) return bad("an update time lies outside the backward pass");
    if (!(0.0 <= need[g] && need[g] <= fp_len)) return bad("a read time lies outside the forward pass");
    dur[g] = net_a + net_b * double(bytes[g]);
    if (!(dur[g] > 0.0)) return bad("a transfer takes no time");
  }

  // largest first; equal sizes keep their queue order
  std::vector<uint32_t> order(n);
  std::iota(order.begin(), order.end(), 0u);
  std::stable_sort(order.begin(), order.end(), [&](uint32_t x, uint32_t y) { return bytes[x] > bytes[y]; });

  Window back, fwd;  // fwd in negated time
  std::vector<uint32_t> left;
  auto put_back = [&](uint32_t g, double x, uint32_t stage) {
    back.occupy(x, x + dur[g]);
    slots[g] = caramel_slot{CARAMEL_BIN_BACKWARD, stage, x, x + dur[g]};
  };
  auto put_fwd = [&](uint32_t g, double x, uint32_t stage) {  // x = -(end time)
    const double end = -x, start = end - dur[g];
    fwd.occupy(x, -start);
    slots[g] = caramel_slot{CARAMEL_BIN_FORWARD, stage, start, end};
  };

  // beside the computation: the backward pass first, then the forward pass
  for (uint32_t g : order) {
    const double xb = back.slide(ready[g], dur[g]);
    if (xb + dur[g] <= bp_len) {
      put_back(g, xb, 2);
      continue;
    }
    const double xf = fwd.slide(-need[g], dur[g]);
    if (-xf - dur[g] >= 0.0) {
      put_fwd(g, xf, 2);
      continue;
    }
    left.push_back(g);
  }
  // the rest lengthens the iteration: take the side where it lengthens it less
  for (uint32_t g : left) {
    const double xb = back.slide(ready[g], dur[g]);
    const double xf = fwd.slide(-need[g], dur[g]);
    const double end_now = back.reach(bp_len);
    const double begin_now = -fwd.reach(0.0);
    const double grow_back = std::max(0.0, (xb + dur[g]) - end_now);
    const double grow_fwd = std::max(0.0, begin_now - (-xf - dur[g]));
    if (grow_back <= grow_fwd)
      put_back(g, xb, 3);
    else
      put_fwd(g, xf, 3);
  }

  if (summary) {
    double comm = 0.0;
    for (uint32_t g = 0; g < n; ++g) comm += dur[g];
    const double compute = bp_len + fp_len;
    const double over_back = back.reach(bp_len) - bp_len;
    const double over_fwd = 0.0 - (-fwd.reach(0.0));
    const double total = compute + over_back + over_fwd;
    const double lesser = std::min(comm, compute);
    summary->comm_time = comm;
    summary->compute_time = compute;
    summary->bp_overrun = over_back;
    summary->fp_overrun = over_fwd;
    summary->iteration_time = total;
    summary->overlap = lesser > 0.0 ? (comm + compute - total) / lesser : 0.0;
    summary->utilization = total > 0.0 ? compute / total : 0.0;
  }
  return CARAMEL_OK;
}

}  // namespace caramel
