// Host-side transfer planner (no GPU calls).
//
// Section 4.2 (Parameter Batcher): parameters are visited in ascending update time; one whose
// size reaches the threshold goes out alone, a smaller one joins the open batch, and the
// batch goes out as soon as it has reached the threshold.  Units are numbered in the order
// they enter the transfer queue.
// Section 4.4 (Adaptive Depth Enforcer): a large transfer becomes `depth` chunks that are
// aggregated independently; unit u is handled by internal stream u mod num_streams.
// Sections 2 / 4.4 (ring pattern): each unit is divided into W segments, one per owner.
#include "plan.hpp"

#include <algorithm>
#include <cmath>
#include <cstring>

namespace caramel {
namespace {

inline uint64_t round_up(uint64_t x, uint64_t m) { return (x + m - 1) / m * m; }
inline uint64_t ceil_div(uint64_t x, uint64_t m) { return (x + m - 1) / m; }

class Queue {
 public:
  Queue(const caramel_config& c, HostPlan& p, bool timed, double a, double b)
      : cfg_(c), plan_(p), es_(p.elem_size()), gran_(p.granule()), timed_(timed), a_(a), b_(b) {}

  // Update time of the parameter being visited (timing-aware plans).
  void set_now(double t) { now_ = t; }
  // When everything queued so far will have been transferred.
  double free_at() const { return free_at_; }

  // A transfer that goes out on its own, possibly cut into chunks.
  void send_alone(uint32_t tensor, uint64_t elems) {
    const uint64_t piece = chunk_elems(elems);
    for (uint64_t at = 0; at < elems; at += piece) {
      const uint64_t n = std::min(piece, elems - at);
      caramel_entry e{tensor, next_unit(), at, 0, n};
      plan_.entries.push_back(e);
      push_unit(CARAMEL_KIND_CHUNK, uint32_t(plan_.entries.size() - 1), 1, n, 0);
    }
  }

  // A small parameter joins the open batch; the batch leaves once it is large enough.
  // Returns true if the batch is now large enough and has been sent.
  bool join_batch(uint32_t tensor, uint64_t elems) {
    const uint64_t at = round_up(fill_, gran_);
    pending_.push_back(caramel_entry{tensor, 0, 0, at, elems});
    fill_ = at + elems;
    if (round_up(fill_, gran_) * es_ < cfg_.batch_threshold_bytes) return false;
    flush();
    return true;
  }

  void flush() {
    if (pending_.empty()) return;
    const uint32_t u = next_unit();
    const uint32_t first = uint32_t(plan_.entries.size());
    for (caramel_entry& e : pending_) {
      e.unit = u;
      plan_.entries.push_back(e);
    }
    const uint64_t padded = round_up(fill_, gran_);
    push_unit(CARAMEL_KIND_BATCH, first, uint32_t(pending_.size()), padded, plan_.fused_elems);
    plan_.fused_elems += padded;
    pending_.clear();
    fill_ = 0;
  }

 private:
  uint32_t next_unit() const { return uint32_t(plan_.units.size()); }

  uint64_t chunk_elems(uint64_t elems) const {
    const uint64_t bytes = elems * es_;
    if (cfg_.split_mode == CARAMEL_SPLIT_NONE || bytes <= cfg_.split_bytes) return elems;
    if (cfg_.split_mode == CARAMEL_SPLIT_FIXED) return cfg_.split_bytes / es_;
    uint64_t depth = bytes / cfg_.split_bytes;
    depth = std::max<uint64_t>(1, std::min<uint64_t>(depth, cfg_.max_depth));
    return round_up(ceil_div(elems, depth), gran_);
  }

  void push_unit(uint32_t kind, uint32_t first, uint32_t count, uint64_t elems, uint64_t fused_off) {
    caramel_unit u{};
    u.kind = kind;
    u.stream = next_unit() % cfg_.num_streams;
    u.first_entry = first;
    u.n_entries = count;
    u.elems = elems;
    u.fused_off = fused_off;
    plan_.units.push_back(u);
    if (timed_) {
      // one transfer at a time, in queue order
      const double begin = now_ > free_at_ ? now_ : free_at_;
      free_at_ = begin + (a_ + b_ * double(elems * es_));
      plan_.enqueue_time.push_back(now_);
      plan_.start_time.push_back(begin);
      plan_.finish_time.push_back(free_at_);
    }
    // ring segments: granules dealt out as evenly as possible, the surplus to the first owners
    const uint64_t W = cfg_.world;
    const uint64_t q = ceil_div(elems, gran_);
    const uint64_t each = q / W, extra = q % W;
    uint64_t g = 0;
    for (uint64_t c = 0; c <= W; ++c) {
      plan_.seg.push_back(std::min(g * gran_, elems));
      g += each + (c < extra ? 1 : 0);
    }
  }

  const caramel_config& cfg_;
  HostPlan& plan_;
  const uint64_t es_, gran_;
  const bool timed_;
  const double a_, b_;
  double now_ = 0.0, free_at_ = 0.0;
  std::vector<caramel_entry> pending_;
  uint64_t fill_ = 0;
};

}  // namespace

int build_host_plan(const caramel_config& cfg, const uint64_t* elems, uint32_t n, const double* ready_time,
                    double net_a, double net_b, HostPlan& out, std::string& why) {
  auto bad = [&](const char* m) {
    why = m;
    return CARAMEL_EINVAL;
  };
  if (!elems) return bad("tensor_elems is NULL");
  if (n == 0) return bad("n_tensors is 0");
  if (cfg.world < 1 || cfg.world > CARAMEL_MAX_WORLD) return bad("world out of range");
  if (cfg.dtype != CARAMEL_F32 && cfg.dtype != CARAMEL_BF16) return bad("unknown dtype");
  if (cfg.split_mode > CARAMEL_SPLIT_ADAPTIVE) return bad("unknown split_mode");
  const uint32_t a = cfg.align_bytes;
  if (a < 16 || (a & (a - 1)) != 0) return bad("align_bytes must be a power of two >= 16");
  if (cfg.num_streams != 1 && cfg.num_streams != 2) return bad("num_streams must be 1 or 2");
  if (cfg.split_mode != CARAMEL_SPLIT_NONE) {
    if (cfg.split_bytes == 0 || cfg.split_bytes % a != 0)
      return bad("split_bytes must be a positive multiple of align_bytes");
    if (cfg.split_mode == CARAMEL_SPLIT_ADAPTIVE && cfg.max_depth == 0) return bad("max_depth is 0");
  }
  if (cfg.pattern > CARAMEL_PATTERN_SHUFFLE) return bad("unknown pattern");
  if (cfg.reserved != 0) return bad("reserved field must be 0");
  if (cfg.pattern == CARAMEL_PATTERN_HALVING_DOUBLING) {
    if (cfg.world & (cfg.world - 1)) return bad("halving-doubling needs a power-of-two world");
  }
  const uint64_t es = cfg.dtype == CARAMEL_F32 ? 4 : 2;
  // 32-bit offsets in units of 16 bytes address at most 64 GiB inside one tensor
  const uint64_t max_elems = (uint64_t(1) << 36) / es - a;
  for (uint32_t i = 0; i < n; ++i) {
    if (elems[i] == 0) return bad("zero-element tensor");
    if (elems[i] > max_elems) return bad("tensor larger than 64 GiB");
  }

  const bool timed = ready_time != nullptr;
  if (timed) {
    if (!(net_a >= 0.0) || !(net_b >= 0.0)) return bad("network model coefficients must be non-negative");
    for (uint32_t i = 0; i + 1 < n; ++i)
      if (!(ready_time[i] <= ready_time[i + 1])) return bad("ready_time must be non-decreasing");
    if (!(ready_time[n - 1] == ready_time[n - 1])) return bad("ready_time holds a NaN");
  }

  out = HostPlan{};
  out.cfg = cfg;
  out.tensor_elems.assign(elems, elems + n);
  Queue q(cfg, out, timed, net_a, net_b);
  for (uint32_t i = 0; i < n; ++i) {
    if (timed) q.set_now(ready_time[i]);
    const bool large = cfg.batch_threshold_bytes == 0 || elems[i] * es >= cfg.batch_threshold_bytes;
    if (large) {
      q.send_alone(i, elems[i]);
      continue;
    }
    const bool sent = q.join_batch(i, elems[i]);
    // section 4.2: the batch also goes out if the queue will have drained before the next
    // parameter is updated -- waiting for more members would leave the network idle
    if (!sent && timed && i + 1 < n && q.free_at() <= ready_time[i + 1]) q.flush();
  }
  q.flush();
  if (out.fused_elems > max_elems) return bad("fused buffer larger than 64 GiB per replica");
  if (out.units.size() > 0xFFFFFFF0ull) return bad("too many units");
  return CARAMEL_OK;
}

bool threshold_from_model(double a, double b, uint64_t& out) {
  if (!(a >= 0.0) || !(b > 0.0) || !std::isfinite(a) || !std::isfinite(b)) return false;
  if (a == 0.0) {
    out = 1;
    return true;
  }
  // a = ma * 2^ea, b = mb * 2^eb with 53-bit integer mantissas; the condition
  // (a + 2bx) / (2a + 2bx) > 4/5  <=>  2bx > 3a  <=>  x > 3 ma 2^(ea - eb - 1) / mb
  int ea = 0, eb = 0;
  const unsigned __int128 ma = (unsigned __int128)std::ldexp(std::frexp(a, &ea), 53);
  const unsigned __int128 mb = (unsigned __int128)std::ldexp(std::frexp(b, &eb), 53);
  const int d = ea - eb - 1;
  unsigned __int128 num = 3 * ma, den = mb;
  if (d >= 0) {
    if (d > 70) return false;  // far beyond 2^64
    num <<= d;
  } else {
    if (-d > 70) {             // 3a / 2b is below 1
      out = 1;
      return true;
    }
    den <<= -d;
  }
  const unsigned __int128 x = num / den + 1;
  if (x >> 64) return false;
  out = uint64_t(x);
  return true;
}

namespace {
template <typename T>
void put(std::vector<uint8_t>& b, T v) {
  for (size_t i = 0; i < sizeof(T); ++i) b.push_back(uint8_t(uint64_t(v) >> (8 * i)));
}
}  // namespace

std::vector<uint8_t> serialize(const HostPlan& p) {
  std::vector<uint8_t> b;
  const char magic[8] = {'C', 'A', 'R', 'A', 'M', 'E', 'L', '1'};
  b.insert(b.end(), magic, magic + 8);
  put<uint32_t>(b, p.cfg.world);
  put<uint32_t>(b, p.cfg.dtype);
  put<uint64_t>(b, p.cfg.batch_threshold_bytes);
  put<uint32_t>(b, p.cfg.split_mode);
  put<uint32_t>(b, p.cfg.max_depth);
  put<uint64_t>(b, p.cfg.split_bytes);
  put<uint32_t>(b, p.cfg.align_bytes);
  put<uint32_t>(b, p.cfg.num_streams);
  put<uint32_t>(b, p.cfg.pattern);
  put<uint32_t>(b, uint32_t(p.tensor_elems.size()));
  put<uint32_t>(b, uint32_t(p.units.size()));
  put<uint32_t>(b, uint32_t(p.entries.size()));
  put<uint64_t>(b, p.fused_elems);
  for (uint64_t e : p.tensor_elems) put<uint64_t>(b, e);
  for (const caramel_unit& u : p.units) {
    put<uint32_t>(b, u.kind);
    put<uint32_t>(b, u.stream);
    put<uint32_t>(b, u.first_entry);
    put<uint32_t>(b, u.n_entries);
    put<uint64_t>(b, u.elems);
    put<uint64_t>(b, u.fused_off);
  }
  for (const caramel_entry& e : p.entries) {
    put<uint32_t>(b, e.tensor);
    put<uint32_t>(b, e.unit);
    put<uint64_t>(b, e.tensor_off);
    put<uint64_t>(b, e.unit_off);
    put<uint64_t>(b, e.elems);
  }
  for (uint64_t s : p.seg) put<uint64_t>(b, s);
  return b;
}

}  // namespace caramel
