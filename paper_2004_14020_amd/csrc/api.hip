// C ABI of the library: plan objects, binding of device memory, stream pipeline, timing.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "caramel.h"
#include "kernels.hpp"
#include "plan.hpp"
#include "schedule.hpp"
#include "tiles.hpp"

using namespace caramel;

// Table space of caramel_allreduce_static: one copy per GPU the library runs on, held until the
// process ends.  On the host this name is only a handle for hipGetSymbolAddress; the device
// address it stands for is looked up once per device and used everywhere else.
static __device__ __align__(256) unsigned char scratch[CARAMEL_STATIC_TABLE_BYTES];

namespace {

thread_local std::string g_err;

int fail(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}

#define HIP_TRY(expr)                                                                         \
  do {                                                                                        \
    hipError_t e_ = (expr);                                                                   \
    if (e_ != hipSuccess) return fail(CARAMEL_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

// No exception leaves the library: allocation failures inside an entry point become ENOMEM.
template <typename F>
int guarded(F&& body) {
  try {
    return body();
  } catch (const std::bad_alloc&) {
    return fail(CARAMEL_ENOMEM, "out of host memory");
  } catch (const std::exception& e) {
    return fail(CARAMEL_ESTATE, "unexpected failure: %s", e.what());
  }
}

struct Options {
  uint32_t launch_mode = CARAMEL_LAUNCH_AUTO;
  uint32_t batch_path = CARAMEL_BATCH_DIRECT;
  TileShape shape;
  uint32_t max_grid = 0;
  uint32_t nontemporal = 1;
  uint32_t unroll = 0;
  uint32_t block = 1024;        // workgroup of launches over long tiles
  uint32_t small_block = 256;   // ... over small tiles
  uint32_t stream_major = 8;    // most vectors per lane of the stream-major kernel for long tiles (0 = off)
  uint64_t launch_min_bytes = 4u << 20;        // launches over small tiles: units share one up to this size
  uint64_t long_launch_min_bytes = 64u << 20;  // launches over long tiles likewise
  uint64_t pipeline_min_bytes = ~uint64_t(0);  // AUTO never pipelines unless told to
  uint64_t merge_small_bytes = 1u << 20;       // one launch per stream: small tiles up to this total join the long ones
  bool split_tiles = true;                     // tiles across segment boundaries where the kernel handles them
};

// Fork/join events order work between streams of the same device; no timing, and no system-scope
// fence (device scope is enough: every producer and consumer is a kernel on this GPU).
constexpr unsigned kOrderOnly = hipEventDisableTiming | hipEventDisableSystemFence;

// One reduce launch: consecutive tiles of one class that belong to consecutive units of one lane.
struct LaunchGroup {
  uint32_t lane, first_unit;
  int cls;  // kLong or kSmall
  Range reduce;
  uint64_t elems;  // elements per replica the launch covers
};

// CARAMEL_TRACE=1 in the environment: one line on stderr per bound unit and per kernel launch
// (what is launched where, over which tiles).  Read once.
bool tracing() {
  static const bool on = [] {
    const char* v = std::getenv("CARAMEL_TRACE");
    return v && *v && std::strcmp(v, "0") != 0;
  }();
  return on;
}

struct TimedLaunch {
  int kind;
  uint64_t call;
  hipEvent_t start, stop;
};

// What binding a plan to a set of gradient pointers produces on the host.
struct Binding {
  TileShape shape;             // the shape the tables were built with
  std::vector<uint64_t> rows;  // (n_tensors + 1) x W base addresses
  TileTables tt;
  std::vector<LaunchGroup> groups[2];  // [0] staged tables, [1] direct tables
  bool groups_stale[2] = {true, true};
  bool groups_pipelined[2] = {false, false};
};

// Where the kernels find the tables of a binding.
struct DeviceTables {
  const uint64_t* rows = nullptr;
  const ReduceTile* staged = nullptr;
  const ReduceTile* direct = nullptr;
  const CopyTile* copy = nullptr;
};

}  // namespace

struct caramel_plan {
  HostPlan host;
  Options opt;
  // device side (valid when bound)
  bool bound = false;
  bool has_ws = false;
  int device = -1;  // the device that was current at bind: tables, stream and events live there
  Binding bind;
  uint64_t* d_rows = nullptr;
  ReduceTile* d_staged = nullptr;
  ReduceTile* d_direct = nullptr;
  CopyTile* d_copy = nullptr;
  hipStream_t streams[2] = {nullptr, nullptr};
  hipEvent_t ev_fork = nullptr;
  hipEvent_t ev_join[2] = {nullptr, nullptr};
  // caramel_allreduce_static keeps its own host tables; their device copy lives in the
  // library's static array
  Binding fixed;
  bool fixed_valid = false;
  uint64_t fixed_generation = 0;  // identifies the contents of `fixed` among all plans
  // timing
  int profiling = 0;  // 0 off, 1 one event pair per stream sequence, 2 one pair per launch
  uint64_t call_no = 0;
  std::vector<TimedLaunch> pending;
  std::vector<hipEvent_t> spare;
  std::vector<std::pair<uint64_t, hipEvent_t>> call_base;
  caramel_kernel_stat stats[CARAMEL_K_COUNT] = {};

  DeviceTables tables() const { return DeviceTables{d_rows, d_staged, d_direct, d_copy}; }
};

namespace {

void release_device(caramel_plan* p) {
  if (p->d_rows) (void)hipFree(p->d_rows);
  if (p->d_staged) (void)hipFree(p->d_staged);
  if (p->d_direct) (void)hipFree(p->d_direct);
  if (p->d_copy) (void)hipFree(p->d_copy);
  p->d_rows = nullptr;
  p->d_staged = p->d_direct = nullptr;
  p->d_copy = nullptr;
  p->bound = false;
}

void drop_events(caramel_plan* p) {
  for (TimedLaunch& t : p->pending) {
    (void)hipEventDestroy(t.start);
    (void)hipEventDestroy(t.stop);
  }
  for (auto& b : p->call_base) (void)hipEventDestroy(b.second);
  for (hipEvent_t e : p->spare) (void)hipEventDestroy(e);
  p->pending.clear();
  p->call_base.clear();
  p->spare.clear();
}

template <typename T>
int upload(const std::vector<T>& v, T** dst) {
  *dst = nullptr;
  if (v.empty()) return CARAMEL_OK;
  HIP_TRY(hipMalloc(reinterpret_cast<void**>(dst), v.size() * sizeof(T)));
  HIP_TRY(hipMemcpy(*dst, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice));
  return CARAMEL_OK;
}

hipEvent_t take_event(caramel_plan* p) {
  if (!p->spare.empty()) {
    hipEvent_t e = p->spare.back();
    p->spare.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  // timing only: no system-scope fence, which would cost a cache write-back per record
  if (hipEventCreateWithFlags(&e, hipEventDisableSystemFence) != hipSuccess) return nullptr;
  return e;
}

// Wraps a kernel launch (or a stream's whole sequence) in a pair of timing events on the
// launch stream when profiling.
struct Timed {
  caramel_plan* p;
  hipStream_t s;
  TimedLaunch t{};
  bool on = false;
  Timed(caramel_plan* plan, int kind, hipStream_t stream, uint64_t elems = 0) : p(plan), s(stream) {
    if (!p->profiling) return;
    if (kind != CARAMEL_K_SEQUENCE) {
      p->stats[kind].launches += 1;
      p->stats[kind].elements += elems;
      if (p->profiling < 2) return;
    }
    t.kind = kind;
    t.call = p->call_no;
    t.start = take_event(p);
    t.stop = take_event(p);
    if (!t.start || !t.stop) return;
    p->pending.reserve(p->pending.size() + 4);  // the destructor must not have to allocate
    on = hipEventRecord(t.start, s) == hipSuccess;
  }
  ~Timed() {
    if (!on) return;
    (void)hipEventRecord(t.stop, s);
    p->pending.push_back(t);
  }
};

int run_reduce(caramel_plan* p, const Binding& bd, const DeviceTables& dt, bool direct, const LaunchGroup& g,
               hipStream_t s, bool timed = true) {
  const Range r = g.reduce;
  const int cls = g.cls;
  if (r.count == 0) return CARAMEL_OK;
  ReduceArgs a{};
  a.tiles = direct ? dt.direct : dt.staged;
  a.rows = dt.rows;
  a.begin = r.begin;
  a.count = r.count;
  a.world = p->host.cfg.world;
  a.bf16 = p->host.cfg.dtype == CARAMEL_BF16;
  a.nontemporal = p->opt.nontemporal != 0;
  a.tree = p->host.cfg.pattern == CARAMEL_PATTERN_HALVING_DOUBLING;
  // by default a workgroup takes a whole tile in one go: vectors per lane = tile / workgroup size
  const bool lng = cls == kLong;
  a.block = lng ? p->opt.block : p->opt.small_block;
  const uint32_t tile_vecs = lng ? bd.shape.long_vecs : bd.shape.small_vecs;
  a.unroll = p->opt.unroll ? p->opt.unroll : std::max(1u, tile_vecs / a.block);
  // stream-major walk: as many vectors per lane as a whole tile has rows of lanes (2, 4 or 8)
  a.stream_major = 0;
  if (lng && p->opt.stream_major) {
    const uint32_t rows = tile_vecs / a.block;
    a.stream_major = std::min(p->opt.stream_major, rows >= 8 ? 8u : (rows >= 4 ? 4u : 2u));
  }
  a.max_grid = p->opt.max_grid;
  if (tracing())
    std::fprintf(stderr,
                 "caramel: call %llu reduce  stream %p (plan stream %u, from unit %u) %s tiles [%u, %u) %s, %u lanes, "
                 "%u vectors per lane and worker, %llu bytes per replica\n",
                 (unsigned long long)p->call_no, (void*)s, g.lane, g.first_unit, lng ? "long" : "small", r.begin,
                 r.begin + r.count, direct ? "in place" : "staged", a.block, a.stream_major ? a.stream_major : a.unroll,
                 (unsigned long long)(g.elems * p->host.elem_size()));
  if (!timed) {
    HIP_TRY(launch_ring_reduce(a, s));
    return CARAMEL_OK;
  }
  Timed timer(p, lng ? CARAMEL_K_REDUCE : CARAMEL_K_REDUCE_SMALL, s, g.elems);
  HIP_TRY(launch_ring_reduce(a, s));
  return CARAMEL_OK;
}

int run_copy(caramel_plan* p, const DeviceTables& dt, bool unpack, Range r, hipStream_t s) {
  if (r.count == 0) return CARAMEL_OK;
  CopyArgs a{};
  a.tiles = dt.copy;
  a.rows = dt.rows;
  a.begin = r.begin;
  a.count = r.count;
  a.world = p->host.cfg.world;
  a.fused_row = uint32_t(p->host.tensor_elems.size());
  a.bf16 = p->host.cfg.dtype == CARAMEL_BF16;
  a.unpack = unpack;
  // Measured on MI355X: with 0.9 GB of fused buffers (Inception-v3, Transformer) streaming loads and
  // stores are 3 to 5 points of peak faster; with 52 MB (ResNet-50), which the last-level cache
  // holds, 10 points slower.
  a.nontemporal = p->opt.nontemporal != 0 &&
                  p->host.fused_elems * p->host.elem_size() * p->host.cfg.world >= (uint64_t(256) << 20);
  if (tracing())
    std::fprintf(stderr, "caramel: call %llu %s stream %p copy tiles [%u, %u)\n", (unsigned long long)p->call_no,
                 unpack ? "unpack " : "pack   ", (void*)s, r.begin, r.begin + r.count);
  Timed timer(p, unpack ? CARAMEL_K_UNPACK : CARAMEL_K_PACK, s);
  HIP_TRY(launch_copy(a, s));
  return CARAMEL_OK;
}

int begin_call(caramel_plan* p, hipStream_t user) {
  ++p->call_no;
  if (p->profiling) {
    hipEvent_t e = take_event(p);
    if (e && hipEventRecord(e, user) == hipSuccess) p->call_base.emplace_back(p->call_no, e);
  }
  return CARAMEL_OK;
}

// Stream 0 of the plan is the caller's stream itself; stream 1 is an internal stream that starts
// after everything already queued on the caller's stream ...
int fork_streams(caramel_plan* p, hipStream_t user, hipStream_t* lane, bool pipelined) {
  lane[0] = lane[1] = user;
  if (!pipelined) return CARAMEL_OK;
  HIP_TRY(hipEventRecord(p->ev_fork, user));
  HIP_TRY(hipStreamWaitEvent(p->streams[1], p->ev_fork, 0));
  lane[1] = p->streams[1];
  return CARAMEL_OK;
}

// ... and the caller's stream continues after the internal stream has drained.
int join_streams(caramel_plan* p, hipStream_t user, bool pipelined) {
  if (!pipelined) return CARAMEL_OK;
  HIP_TRY(hipEventRecord(p->ev_join[1], p->streams[1]));
  HIP_TRY(hipStreamWaitEvent(user, p->ev_join[1], 0));
  return CARAMEL_OK;
}

// A reduce launch covers the tiles of one class (long or small) of consecutive units of one
// stream; they are adjacent in the tables, so a launch is one tile range.  PER_UNIT: units are
// added until the launch covers at least the class's minimum bytes per replica.  PER_STREAM: one
// launch per class and stream.  The order in which a stream's launches are issued does not
// affect results.  AUTO: the two-stream pipeline pays a fixed price for its fork and join (tens
// of microseconds of cross-stream signalling), so it is used only when a call moves enough
// bytes to win that back; smaller calls go out as one launch per class on the caller's stream.
bool use_pipeline(const caramel_plan* p) {
  if (p->host.cfg.num_streams != 2) return false;
  if (p->opt.launch_mode != CARAMEL_LAUNCH_AUTO) return true;
  uint64_t elems = 0;
  for (uint64_t e : p->host.tensor_elems) elems += e;
  return 2 * uint64_t(p->host.cfg.world) * elems * p->host.elem_size() >= p->opt.pipeline_min_bytes;
}

// PER_UNIT or PER_STREAM: what the launch mode comes to for this plan.
uint32_t effective_mode(const caramel_plan* p, bool pipelined) {
  if (p->opt.launch_mode != CARAMEL_LAUNCH_AUTO) return p->opt.launch_mode;
  return pipelined ? CARAMEL_LAUNCH_PER_UNIT : CARAMEL_LAUNCH_PER_STREAM;
}

const std::vector<LaunchGroup>& launch_groups(const caramel_plan* p, Binding& bd, bool direct, bool pipelined) {
  const int ti = direct ? 1 : 0;
  std::vector<LaunchGroup>& out = bd.groups[ti];
  if (!bd.groups_stale[ti] && bd.groups_pipelined[ti] == pipelined) return out;
  out.clear();
  const TileTables& tt = bd.tt;
  const std::vector<UnitTiles>& unit_tiles = direct ? tt.direct_unit : tt.staged_unit;
  const uint32_t mode = effective_mode(p, pipelined);
  const uint64_t es = p->host.elem_size();
  // Without the pipeline both plan streams run on the caller's stream: treat them as one lane.
  const uint32_t lanes = pipelined ? p->host.cfg.num_streams : 1;
  for (int cls = 0; cls < 2; ++cls) {
    const uint64_t min_bytes = cls == kLong ? p->opt.long_launch_min_bytes : p->opt.launch_min_bytes;
    for (uint32_t lane = 0; lane < lanes; ++lane) {
      LaunchGroup g{};
      uint64_t bytes = 0;
      bool open = false;
      const size_t mine = out.size();  // launches of this class and lane start here
      for (uint32_t s = 0; s < p->host.cfg.num_streams; ++s) {
        if (pipelined && s != lane) continue;
        for (uint32_t u : tt.order[s]) {
          const UnitTiles& ut = unit_tiles[u];
          if (ut.tiles[cls].count == 0) continue;
          if (!open) {
            g = LaunchGroup{lane, u, cls, Range{ut.tiles[cls].begin, 0}, 0};
            bytes = 0;
            open = true;
          }
          g.reduce.count += ut.tiles[cls].count;
          g.elems += ut.elems[cls];
          bytes += ut.elems[cls] * es;
          if (mode == CARAMEL_LAUNCH_PER_UNIT && bytes >= min_bytes) {
            out.push_back(g);
            open = false;
          }
        }
      }
      if (open) {
        // what is left over at the end is rarely worth a launch of its own: less than half the
        // minimum joins the launch before it (its tiles follow that launch's in the table)
        LaunchGroup* prev = out.size() > mine ? &out.back() : nullptr;
        if (prev && bytes < min_bytes / 2 && prev->reduce.begin + prev->reduce.count == g.reduce.begin) {
          prev->reduce.count += g.reduce.count;
          prev->elems += g.elems;
        } else {
          out.push_back(g);
        }
      }
    }
  }
  // One launch per class on one stream: if the short runs are few, their tiles (which follow the
  // long tiles in the table) join the launch over the long tiles, whose kernel takes a tile of up
  // to one vector per lane in a single pass.  That saves a launch of a few microseconds; the
  // small tiles come last in the grid and fill the tail of the long ones.
  if (mode == CARAMEL_LAUNCH_PER_STREAM && lanes == 1 && out.size() == 2 && out[0].cls == kLong &&
      out[1].cls == kSmall && out[1].elems * es <= p->opt.merge_small_bytes &&
      out[0].reduce.begin + out[0].reduce.count == out[1].reduce.begin &&
      bd.shape.small_vecs <= p->opt.block) {
    out[0].reduce.count += out[1].reduce.count;
    out[0].elems += out[1].elems;
    out.pop_back();
  }
  // issue in the order of the first unit, which alternates between the streams ...
  std::stable_sort(out.begin(), out.end(),
                   [](const LaunchGroup& a, const LaunchGroup& b) { return a.first_unit < b.first_unit; });
  // ... but every stream issues its launches over small tiles first: a call then ends with the
  // long, evenly sized launches running on both streams, and the streams finish together
  std::stable_sort(out.begin(), out.end(), [](const LaunchGroup& a, const LaunchGroup& b) { return a.cls > b.cls; });
  bd.groups_stale[ti] = false;
  bd.groups_pipelined[ti] = pipelined;
  return out;
}

// Shared body of caramel_ring_reduce (reduce only, staged tables) and caramel_allreduce.  In
// staged mode every lane packs all its batch units, reduces, and unpacks them, in stream order.
int pipeline(caramel_plan* p, hipStream_t user, bool with_copies, bool direct) {
  begin_call(p, user);
  hipStream_t lane[2] = {nullptr, nullptr};
  const bool pipelined = use_pipeline(p);
  int rc = fork_streams(p, user, lane, pipelined);
  if (rc) return rc;
  const bool copies = with_copies && !direct;
  const DeviceTables dt = p->tables();
  const TileTables& tt = p->bind.tt;
  const uint32_t n_lanes = pipelined ? 2u : 1u;
  // the copy tiles of a lane: of its stream, or of both streams when there is one lane
  Range copy_of[2] = {tt.copy_stream[0], tt.copy_stream[1]};
  if (!pipelined) copy_of[0].count = tt.copy_stream[0].count + tt.copy_stream[1].count;
  // one event pair around everything a stream does in this call
  std::unique_ptr<Timed> seq[2];
  if (p->profiling)
    for (uint32_t s = 0; s < n_lanes; ++s) seq[s].reset(new Timed(p, CARAMEL_K_SEQUENCE, lane[s]));
  if (copies)
    for (uint32_t s = 0; s < n_lanes && !rc; ++s) rc = run_copy(p, dt, false, copy_of[s], lane[s]);
  if (!rc)
    for (const LaunchGroup& g : launch_groups(p, p->bind, direct, pipelined)) {
      rc = run_reduce(p, p->bind, dt, direct, g, lane[g.lane]);
      if (rc) break;
    }
  if (copies)
    for (uint32_t s = 0; s < n_lanes && !rc; ++s) rc = run_copy(p, dt, true, copy_of[s], lane[s]);
  for (auto& q : seq) q.reset();
  // join even after a failed launch so the caller's stream stays ordered
  const int jc = join_streams(p, user, pipelined);
  return rc ? rc : jc;
}

int need_bound(const caramel_plan* p, bool needs_ws) {
  if (!p) return fail(CARAMEL_EINVAL, "plan is NULL");
  if (!p->bound) return fail(CARAMEL_ESTATE, "plan is not bound to device memory");
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev != p->device)
    return fail(CARAMEL_ESTATE, "plan was bound with device %d current, now device %d is", p->device, dev);
  if (needs_ws && p->host.fused_elems > 0 && !p->has_ws)
    return fail(CARAMEL_ESTATE, "this call needs the fused workspace, but none was bound");
  return CARAMEL_OK;
}

}  // namespace

extern "C" {

namespace {
int create_plan(const caramel_config* cfg, const uint64_t* tensor_elems, uint32_t n_tensors,
                const double* ready_time, double net_a, double net_b, caramel_plan** out);
}

int caramel_plan_create(const caramel_config* cfg, const uint64_t* tensor_elems, uint32_t n_tensors,
                        caramel_plan** out) {
  return create_plan(cfg, tensor_elems, n_tensors, nullptr, 0.0, 0.0, out);
}

int caramel_plan_create_timed(const caramel_config* cfg, const uint64_t* tensor_elems, uint32_t n_tensors,
                              const double* ready_time, double net_a, double net_b, caramel_plan** out) {
  if (!ready_time) return fail(CARAMEL_EINVAL, "ready_time is NULL");
  return create_plan(cfg, tensor_elems, n_tensors, ready_time, net_a, net_b, out);
}

int caramel_plan_times(const caramel_plan* p, double* enqueue, double* start, double* finish, uint32_t cap) {
  if (!p) return fail(CARAMEL_EINVAL, "plan is NULL");
  const HostPlan& h = p->host;
  if (h.start_time.size() != h.units.size()) return fail(CARAMEL_ESTATE, "not a timing-aware plan");
  if (cap < h.units.size()) return fail(CARAMEL_EINVAL, "capacity %u < %zu units", cap, h.units.size());
  if (enqueue) std::copy(h.enqueue_time.begin(), h.enqueue_time.end(), enqueue);
  if (start) std::copy(h.start_time.begin(), h.start_time.end(), start);
  if (finish) std::copy(h.finish_time.begin(), h.finish_time.end(), finish);
  return CARAMEL_OK;
}

int caramel_net_model_fit(uint64_t bytes1, double time1, uint64_t bytes2, double time2, double* a, double* b) {
  if (!a || !b) return fail(CARAMEL_EINVAL, "NULL argument");
  if (bytes1 == bytes2) return fail(CARAMEL_EINVAL, "the two sizes must differ");
  if (!std::isfinite(time1) || !std::isfinite(time2)) return fail(CARAMEL_EINVAL, "times must be finite");
  const double slope = (time2 - time1) / (double(bytes2) - double(bytes1));
  const double icpt = time1 - slope * double(bytes1);
  if (!(slope > 0.0) || !(icpt >= 0.0))
    return fail(CARAMEL_EINVAL,
                "the probes (%llu B in %g, %llu B in %g) give the line %g + %g * bytes: a transfer-time model "
                "needs a >= 0 and b > 0 (time must grow with size); measure again",
                (unsigned long long)bytes1, time1, (unsigned long long)bytes2, time2, icpt, slope);
  *b = slope;
  *a = icpt;
  return CARAMEL_OK;
}

int caramel_threshold_estimate(double a, double b, uint64_t* threshold_bytes) {
  if (!threshold_bytes) return fail(CARAMEL_EINVAL, "NULL argument");
  if (!threshold_from_model(a, b, *threshold_bytes))
    return fail(CARAMEL_EINVAL, "need finite a >= 0, b > 0 and a threshold below 2^64");
  return CARAMEL_OK;
}

int caramel_schedule_transfers(const uint64_t* group_bytes, const double* ready, const double* need,
                               uint32_t n_groups, double bp_len, double fp_len, double net_a, double net_b,
                               caramel_slot* slots, caramel_schedule_summary* summary) {
  std::string why;
  try {
    const int rc = schedule_transfers(group_bytes, ready, need, n_groups, bp_len, fp_len, net_a, net_b, slots,
                                      summary, why);
    return rc == CARAMEL_OK ? rc : fail(rc, why.c_str());
  } catch (const std::bad_alloc&) {
    return fail(CARAMEL_ENOMEM, "out of host memory");
  }
}

int caramel_plan_windows(const caramel_plan* plan, const double* ready_time, const double* read_time,
                         uint64_t* group_bytes, double* ready, double* need, uint32_t cap) {
  if (!plan || !ready_time || !read_time) return fail(CARAMEL_EINVAL, "NULL argument");
  const size_t n = plan->host.units.size();
  if (cap < n) return fail(CARAMEL_EINVAL, "cap is smaller than the number of units");
  try {
    std::vector<uint64_t> b(n);
    std::vector<double> r(n), d(n);
    unit_windows(plan->host, ready_time, read_time, b.data(), r.data(), d.data());
    if (group_bytes) std::copy(b.begin(), b.end(), group_bytes);
    if (ready) std::copy(r.begin(), r.end(), ready);
    if (need) std::copy(d.begin(), d.end(), need);
  } catch (const std::bad_alloc&) {
    return fail(CARAMEL_ENOMEM, "out of host memory");
  }
  return CARAMEL_OK;
}

}  // extern "C"

namespace {
int create_plan(const caramel_config* cfg, const uint64_t* tensor_elems, uint32_t n_tensors,
                const double* ready_time, double net_a, double net_b, caramel_plan** out) {
  if (!cfg || !out) return fail(CARAMEL_EINVAL, "NULL argument");
  *out = nullptr;
  caramel_plan* p = new (std::nothrow) caramel_plan;
  if (!p) return fail(CARAMEL_ENOMEM, "out of host memory");
  std::string why;
  int rc;
  try {
    rc = build_host_plan(*cfg, tensor_elems, n_tensors, ready_time, net_a, net_b, p->host, why);
  } catch (const std::bad_alloc&) {
    delete p;
    return fail(CARAMEL_ENOMEM, "out of host memory");
  }
  if (rc != CARAMEL_OK) {
    delete p;
    return fail(rc, "%s", why.c_str());
  }
  *out = p;
  return CARAMEL_OK;
}
}  // namespace

extern "C" {

void caramel_plan_destroy(caramel_plan* p) {
  if (!p) return;
  if (p->bound || p->streams[1] || p->ev_fork) {
    for (int s = 0; s < 2; ++s)
      if (p->streams[s]) (void)hipStreamSynchronize(p->streams[s]);
    drop_events(p);
    release_device(p);
    for (int s = 0; s < 2; ++s) {
      if (p->streams[s]) (void)hipStreamDestroy(p->streams[s]);
      if (p->ev_join[s]) (void)hipEventDestroy(p->ev_join[s]);
    }
    if (p->ev_fork) (void)hipEventDestroy(p->ev_fork);
  }
  delete p;
}

int caramel_plan_counts(const caramel_plan* p, uint32_t* n_units, uint32_t* n_entries, uint64_t* fused_elems) {
  if (!p) return fail(CARAMEL_EINVAL, "plan is NULL");
  if (n_units) *n_units = uint32_t(p->host.units.size());
  if (n_entries) *n_entries = uint32_t(p->host.entries.size());
  if (fused_elems) *fused_elems = p->host.fused_elems;
  return CARAMEL_OK;
}

int caramel_plan_units(const caramel_plan* p, caramel_unit* out, uint32_t cap) {
  if (!p || !out) return fail(CARAMEL_EINVAL, "NULL argument");
  if (cap < p->host.units.size()) return fail(CARAMEL_EINVAL, "capacity %u < %zu units", cap, p->host.units.size());
  std::copy(p->host.units.begin(), p->host.units.end(), out);
  return CARAMEL_OK;
}

int caramel_plan_entries(const caramel_plan* p, caramel_entry* out, uint32_t cap) {
  if (!p || !out) return fail(CARAMEL_EINVAL, "NULL argument");
  if (cap < p->host.entries.size())
    return fail(CARAMEL_EINVAL, "capacity %u < %zu entries", cap, p->host.entries.size());
  std::copy(p->host.entries.begin(), p->host.entries.end(), out);
  return CARAMEL_OK;
}

int caramel_plan_segments(const caramel_plan* p, uint32_t unit, uint64_t* seg_start) {
  if (!p || !seg_start) return fail(CARAMEL_EINVAL, "NULL argument");
  if (unit >= p->host.units.size()) return fail(CARAMEL_EINVAL, "unit %u out of range", unit);
  const uint64_t* s = p->host.segments(unit);
  std::copy(s, s + p->host.cfg.world + 1, seg_start);
  return CARAMEL_OK;
}

int caramel_plan_serialize(const caramel_plan* p, void* buf, size_t* len) {
  if (!p || !len) return fail(CARAMEL_EINVAL, "NULL argument");
  return guarded([&]() -> int {
    const std::vector<uint8_t> img = serialize(p->host);
    if (!buf) {
      *len = img.size();
      return CARAMEL_OK;
    }
    if (*len < img.size()) return fail(CARAMEL_EINVAL, "buffer of %zu bytes, need %zu", *len, img.size());
    std::memcpy(buf, img.data(), img.size());
    *len = img.size();
    return CARAMEL_OK;
  });
}

int caramel_plan_set_option(caramel_plan* p, uint32_t option, uint64_t value) {
  if (!p) return fail(CARAMEL_EINVAL, "plan is NULL");
  auto regroup = [&] {
    for (Binding* b : {&p->bind, &p->fixed}) b->groups_stale[0] = b->groups_stale[1] = true;
  };
  auto is_block = [](uint64_t v) { return v == 256 || v == 512 || v == 1024; };
  switch (option) {
    case CARAMEL_OPT_LAUNCH_MODE:
      if (value > CARAMEL_LAUNCH_AUTO) return fail(CARAMEL_EINVAL, "unknown launch mode");
      p->opt.launch_mode = uint32_t(value);
      regroup();
      return CARAMEL_OK;
    case CARAMEL_OPT_BATCH_PATH:
      if (value > CARAMEL_BATCH_DIRECT) return fail(CARAMEL_EINVAL, "unknown batch path");
      p->opt.batch_path = uint32_t(value);
      return CARAMEL_OK;
    case CARAMEL_OPT_TILE_VECS:
      if (value != 0 && (value < 64 || value > (1u << 20))) return fail(CARAMEL_EINVAL, "tile_vecs must be 0 or in [64, 2^20]");
      p->opt.shape.long_vecs = uint32_t(value);
      p->fixed_valid = false;
      return CARAMEL_OK;
    case CARAMEL_OPT_SMALL_TILE_VECS:
      if (value < 64 || value > (1u << 20)) return fail(CARAMEL_EINVAL, "tile_vecs must be in [64, 2^20]");
      p->opt.shape.small_vecs = uint32_t(value);
      p->fixed_valid = false;
      return CARAMEL_OK;
    case CARAMEL_OPT_SMALL_BLOCK:
      if (!is_block(value)) return fail(CARAMEL_EINVAL, "block must be 256, 512 or 1024");
      p->opt.small_block = uint32_t(value);
      return CARAMEL_OK;
    case CARAMEL_OPT_LONG_LAUNCH_MIN_BYTES:
      p->opt.long_launch_min_bytes = value;
      regroup();
      return CARAMEL_OK;
    case CARAMEL_OPT_STREAM_MAJOR:
      if (value != 0 && value != 2 && value != 4 && value != 8) return fail(CARAMEL_EINVAL, "stream_major must be 0, 2, 4 or 8");
      p->opt.stream_major = uint32_t(value);
      return CARAMEL_OK;
    case CARAMEL_OPT_ALIGN_TILES:
      if (value > 3) return fail(CARAMEL_EINVAL, "align_tiles must be 0..3");
      p->opt.shape.align_tiles = uint32_t(value);
      p->fixed_valid = false;
      return CARAMEL_OK;
    case CARAMEL_OPT_LONG_RUN_BYTES:
      p->opt.shape.long_run_bytes = value;
      p->fixed_valid = false;
      return CARAMEL_OK;
    case CARAMEL_OPT_MAX_GRID:
      if (value > 0x7FFFFFFFu) return fail(CARAMEL_EINVAL, "max_grid too large");
      p->opt.max_grid = uint32_t(value);
      return CARAMEL_OK;
    case CARAMEL_OPT_NONTEMPORAL:
      p->opt.nontemporal = value ? 1 : 0;
      return CARAMEL_OK;
    case CARAMEL_OPT_UNROLL:
      if (value != 0 && value != 1 && value != 2 && value != 4) return fail(CARAMEL_EINVAL, "unroll must be 0, 1, 2 or 4");
      p->opt.unroll = uint32_t(value);
      return CARAMEL_OK;
    case CARAMEL_OPT_LAUNCH_MIN_BYTES:
      p->opt.launch_min_bytes = value;
      regroup();
      return CARAMEL_OK;
    case CARAMEL_OPT_PIPELINE_MIN_BYTES:
      p->opt.pipeline_min_bytes = value;
      regroup();
      return CARAMEL_OK;
    case CARAMEL_OPT_BLOCK:
      if (!is_block(value)) return fail(CARAMEL_EINVAL, "block must be 256, 512 or 1024");
      p->opt.block = uint32_t(value);
      regroup();
      return CARAMEL_OK;
    case CARAMEL_OPT_TAIL_TILES:
      if (value > 0x7FFFFFFFu) return fail(CARAMEL_EINVAL, "tail_tiles too large");
      p->opt.shape.tail_tiles = uint32_t(value);
      p->fixed_valid = false;
      return CARAMEL_OK;
    case CARAMEL_OPT_SPLIT_TILES:
      if (value > 1) return fail(CARAMEL_EINVAL, "split_tiles must be 0 or 1");
      p->opt.split_tiles = value != 0;
      p->fixed_valid = false;
      return CARAMEL_OK;
    case CARAMEL_OPT_MERGE_SMALL_BYTES:
      p->opt.merge_small_bytes = value;
      regroup();
      return CARAMEL_OK;
    default:
      return fail(CARAMEL_EINVAL, "unknown option %u", option);
  }
}

namespace {
int bind_plan(caramel_plan* p, void* const* grads, void* fused_ws);
}

int caramel_bind(caramel_plan* p, void* const* grads, void* fused_ws) {
  return guarded([&] { return bind_plan(p, grads, fused_ws); });
}

}  // extern "C"

namespace {
// Argument checks of a binding; on success `rows` holds the (n_tensors + 1) x W base addresses.
int check_pointers(const HostPlan& h, void* const* grads, void* fused_ws, std::vector<uint64_t>& rows) {
  const uint32_t W = h.cfg.world;
  const size_t n = h.tensor_elems.size();
  const uint64_t es = h.elem_size();
  struct Span {
    uint64_t lo, hi;
  };
  std::vector<Span> spans;
  spans.reserve(W * n + 1);
  for (uint32_t w = 0; w < W; ++w)
    for (size_t t = 0; t < n; ++t) {
      const uint64_t a = reinterpret_cast<uint64_t>(grads[w * n + t]);
      if (a == 0) return fail(CARAMEL_EINVAL, "grads[%u][%zu] is NULL", w, t);
      if (a % h.cfg.align_bytes) return fail(CARAMEL_EINVAL, "grads[%u][%zu] is not aligned to %u bytes", w, t, h.cfg.align_bytes);
      spans.push_back({a, a + h.tensor_elems[t] * es});
    }
  if (fused_ws) {
    const uint64_t a = reinterpret_cast<uint64_t>(fused_ws);
    if (a % h.cfg.align_bytes) return fail(CARAMEL_EINVAL, "fused_ws is not aligned to %u bytes", h.cfg.align_bytes);
    if (h.fused_elems) spans.push_back({a, a + uint64_t(W) * h.fused_elems * es});
  }
  std::sort(spans.begin(), spans.end(), [](const Span& x, const Span& y) { return x.lo < y.lo; });
  for (size_t i = 1; i < spans.size(); ++i)
    if (spans[i].lo < spans[i - 1].hi) return fail(CARAMEL_EINVAL, "gradient / workspace buffers overlap");
  rows.assign((n + 1) * W, 0);
  for (uint32_t w = 0; w < W; ++w) {
    for (size_t t = 0; t < n; ++t) rows[t * W + w] = reinterpret_cast<uint64_t>(grads[w * n + t]);
    rows[n * W + w] = fused_ws ? reinterpret_cast<uint64_t>(fused_ws) + uint64_t(w) * h.fused_elems * es : 0;
  }
  return CARAMEL_OK;
}

void fill_binding(const caramel_plan* p, std::vector<uint64_t>&& rows, Binding& bd) {
  bd.shape = p->opt.shape;
  // Shapes left to the library (option value 0) follow the size of the job, measured on MI355X:
  //  * a replica of less than 32 MiB is done before long tiles pay off (a 1024-lane workgroup
  //    walks its tile one replica after the other): every run is cut into small tiles, whose
  //    workgroups fetch all replicas at once (the MLP configuration: 3.4 against 6.3 us);
  //  * fp32 chains of 2, 4 or 8 workers, for which the kernel can keep eight vectors per lane in
  //    registers, get long tiles of 128 KiB once a replica holds 64 MiB (VGG-16 +2 %); everything
  //    else 64 KiB.
  bd.shape.tail_vecs = p->opt.block;  // one vector per lane: a piece is fetched from all replicas at once
  const caramel_config& c = p->host.cfg;
  //  * tiles may straddle a segment boundary where the kernel for the world size sums the two
  //    parts in their own orders (the kernel for any world size; W = 48, 4 MiB chunks: 63 -> 71 %
  //    of peak); the kernels specialised for 2, 4, 8 and 16 workers get tiles inside one segment.
  bd.shape.split_tiles = p->opt.split_tiles && reduce_handles_split_tiles(c.world);
  uint64_t replica_bytes = 0;
  for (uint64_t e : p->host.tensor_elems) replica_bytes += e * p->host.elem_size();
  //  * halving-doubling with 32 or 64 workers has no kernel that walks the replicas one at a time
  //    (its partial sums do not fit the registers): small tiles throughout (W = 32: 64.9 -> 69.1 %).
  const bool tree_any = c.pattern == CARAMEL_PATTERN_HALVING_DOUBLING && c.world > 16;
  if (bd.shape.long_run_bytes == 0)
    bd.shape.long_run_bytes = (replica_bytes < (32u << 20) || tree_any) ? ~uint64_t(0) : 16u << 10;
  if (bd.shape.long_vecs == 0) {
    const bool wide = c.dtype == CARAMEL_F32 && c.pattern != CARAMEL_PATTERN_HALVING_DOUBLING &&
                      (c.world == 2 || c.world == 4 || c.world == 8) && p->opt.stream_major >= 8 &&
                      p->opt.block == 1024 && replica_bytes >= (64u << 20);
    // the bf16 tree keeps two vectors per lane: tiles of one pass (a second pass of a workgroup
    // waits for the stores of the first; Transformer shapes 65.4 -> 66.5 %)
    const bool narrow = c.dtype == CARAMEL_BF16 && c.pattern == CARAMEL_PATTERN_HALVING_DOUBLING;
    bd.shape.long_vecs = wide ? 8192 : (narrow ? 2048 : 4096);
  }
  bd.rows = std::move(rows);
  build_tiles(p->host, bd.shape, bd.tt, bd.rows.data());
  bd.groups_stale[0] = bd.groups_stale[1] = true;
}

int bind_plan(caramel_plan* p, void* const* grads, void* fused_ws) {
  if (!p || !grads) return fail(CARAMEL_EINVAL, "NULL argument");
  const HostPlan& h = p->host;
  // argument checks first: nothing is touched on the device if they fail
  std::vector<uint64_t> rows;
  if (int rc = check_pointers(h, grads, fused_ws, rows)) return rc;

  // a plan stays on the device it was first bound on: its stream and events live there
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (p->device >= 0 && dev != p->device)
    return fail(CARAMEL_ESTATE, "plan was bound with device %d current, now device %d is", p->device, dev);
  for (int s = 0; s < 2; ++s)
    if (p->streams[s]) HIP_TRY(hipStreamSynchronize(p->streams[s]));
  release_device(p);
  p->device = dev;

  fill_binding(p, std::move(rows), p->bind);
  int rc = upload(p->bind.rows, &p->d_rows);
  if (!rc) rc = upload(p->bind.tt.direct, &p->d_direct);
  if (!rc && fused_ws) rc = upload(p->bind.tt.staged, &p->d_staged);
  if (!rc && fused_ws) rc = upload(p->bind.tt.copy, &p->d_copy);
  if (rc) {
    release_device(p);
    return rc;
  }
  if (h.cfg.num_streams > 1) {
    // each handle under its own check: a plan whose earlier bind failed half-way is completed here
    hipError_t e = hipSuccess;
    if (!p->streams[1]) e = hipStreamCreateWithFlags(&p->streams[1], hipStreamNonBlocking);
    if (e == hipSuccess && !p->ev_join[1]) e = hipEventCreateWithFlags(&p->ev_join[1], kOrderOnly);
    if (e == hipSuccess && !p->ev_fork) e = hipEventCreateWithFlags(&p->ev_fork, kOrderOnly);
    if (e != hipSuccess) {
      release_device(p);  // the tables go too: the plan stays unbound
      return fail(CARAMEL_EHIP, "creating the internal stream and its events: %s", hipGetErrorString(e));
    }
  }
  p->has_ws = fused_ws != nullptr;
  p->bound = true;
  if (tracing()) {
    std::fprintf(stderr, "caramel: bind  %zu units, long tiles of %u vectors, small of %u, runs of %llu bytes or more are long\n",
                 h.units.size(), p->bind.shape.long_vecs, p->bind.shape.small_vecs,
                 (unsigned long long)p->bind.shape.long_run_bytes);
    for (size_t u = 0; u < h.units.size(); ++u) {
      const UnitTiles& ut = p->bind.tt.direct_unit[u];
      std::fprintf(stderr, "caramel: unit %zu %s stream %u %llu bytes per replica: %u long + %u small tiles\n", u,
                   h.units[u].kind == CARAMEL_KIND_BATCH ? "batch" : "chunk", h.units[u].stream,
                   (unsigned long long)(h.units[u].elems * h.elem_size()), ut.tiles[kLong].count, ut.tiles[kSmall].count);
    }
  }
  return CARAMEL_OK;
}
}  // namespace

extern "C" {

int caramel_pack(caramel_plan* p, void* stream) {
  return guarded([&]() -> int {
    if (int rc = need_bound(p, true)) return rc;
    begin_call(p, hipStream_t(stream));
    Range all{0, uint32_t(p->bind.tt.copy.size())};
    return run_copy(p, p->tables(), false, all, hipStream_t(stream));
  });
}

int caramel_unpack(caramel_plan* p, void* stream) {
  return guarded([&]() -> int {
    if (int rc = need_bound(p, true)) return rc;
    begin_call(p, hipStream_t(stream));
    Range all{0, uint32_t(p->bind.tt.copy.size())};
    return run_copy(p, p->tables(), true, all, hipStream_t(stream));
  });
}

int caramel_ring_reduce(caramel_plan* p, void* stream) {
  return guarded([&]() -> int {
    if (int rc = need_bound(p, true)) return rc;
    // without a workspace there are no batch units, and the two tables coincide
    return pipeline(p, hipStream_t(stream), false, !p->has_ws);
  });
}

int caramel_allreduce(caramel_plan* p, void* stream) {
  return guarded([&]() -> int {
    const bool direct = p && (p->opt.batch_path == CARAMEL_BATCH_DIRECT || p->host.fused_elems == 0);
    if (int rc = need_bound(p, !direct)) return rc;
    return pipeline(p, hipStream_t(stream), true, direct);
  });
}

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
unsigned char* g_scratch_ptr[kMaxDevices] = {};  // device address of each GPU's copy of `scratch`
uint64_t g_scratch_holds[kMaxDevices] = {};      // generation of the tables it holds (0: none)
hipStream_t g_scratch_stream[kMaxDevices] = {};  // stream they were uploaded on
uint64_t g_generation = 0;

int allreduce_static(caramel_plan* p, void* const* grads, hipStream_t stream) {
  if (!p || !grads) return fail(CARAMEL_EINVAL, "NULL argument");
  const HostPlan& h = p->host;
  std::vector<uint64_t> rows;
  if (int rc = check_pointers(h, grads, nullptr, rows)) return rc;
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(CARAMEL_ESTATE, "device %d is beyond the %d this entry point serves", dev, kMaxDevices);

  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!p->fixed_valid || rows != p->fixed.rows) {
    fill_binding(p, std::move(rows), p->fixed);
    p->fixed_valid = true;
    p->fixed_generation = ++g_generation;
  }
  const Binding& bd = p->fixed;
  const size_t rows_bytes = (bd.rows.size() * sizeof(uint64_t) + 255) / 256 * 256;
  const size_t tile_bytes = bd.tt.direct.size() * sizeof(ReduceTile);
  if (rows_bytes + tile_bytes > CARAMEL_STATIC_TABLE_BYTES)
    return fail(CARAMEL_EINVAL,
                "this plan needs %zu bytes of descriptor tables (%zu tensors x %u workers, %zu tiles); the "
                "static array holds %u: use caramel_bind + caramel_allreduce",
                rows_bytes + tile_bytes, h.tensor_elems.size(), h.cfg.world, bd.tt.direct.size(),
                unsigned(CARAMEL_STATIC_TABLE_BYTES));

  // this GPU's copy of the array: looked up once, with this device current
  if (!g_scratch_ptr[dev]) {
    void* q = nullptr;
    HIP_TRY(hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)));
    if (!q) return fail(CARAMEL_EHIP, "hipGetSymbolAddress returned no address for the static table array");
    g_scratch_ptr[dev] = static_cast<unsigned char*>(q);
  }
  unsigned char* base = g_scratch_ptr[dev];
  // The array keeps what the last call put there.  Tables are written whole before they are
  // used and nothing is read beyond them, so nothing needs clearing; they are uploaded again
  // unless this GPU's array still holds exactly these, put there through this same stream.
  if (g_scratch_holds[dev] != p->fixed_generation || g_scratch_stream[dev] != stream) {
    g_scratch_holds[dev] = 0;
    HIP_TRY(hipMemcpyAsync(base, bd.rows.data(), bd.rows.size() * sizeof(uint64_t), hipMemcpyHostToDevice, stream));
    if (tile_bytes)
      HIP_TRY(hipMemcpyAsync(base + rows_bytes, bd.tt.direct.data(), tile_bytes, hipMemcpyHostToDevice, stream));
    // the host tables may be rebuilt or freed by a later call: wait until they have been read
    HIP_TRY(hipStreamSynchronize(stream));
    g_scratch_holds[dev] = p->fixed_generation;
    g_scratch_stream[dev] = stream;
  }
  DeviceTables dt;
  dt.rows = reinterpret_cast<const uint64_t*>(base);
  dt.direct = reinterpret_cast<const ReduceTile*>(base + rows_bytes);
  for (const LaunchGroup& g : launch_groups(p, p->fixed, true, false))
    if (int rc = run_reduce(p, p->fixed, dt, true, g, stream, false)) return rc;
  return CARAMEL_OK;
}

}  // namespace

int caramel_allreduce_static(caramel_plan* p, void* const* grads, void* stream) {
  return guarded([&] { return allreduce_static(p, grads, hipStream_t(stream)); });
}

int caramel_allreduce_loop(caramel_plan* p, void* stream, uint32_t n_calls, double* host_us_per_call,
                           double* stream_us_per_call) {
  return guarded([&]() -> int {
    if (!host_us_per_call || !stream_us_per_call || n_calls == 0) return fail(CARAMEL_EINVAL, "NULL argument or no calls");
    const bool direct = p && (p->opt.batch_path == CARAMEL_BATCH_DIRECT || p->host.fused_elems == 0);
    if (int rc = need_bound(p, !direct)) return rc;
    hipStream_t s = hipStream_t(stream);
    hipEvent_t e0 = nullptr, e1 = nullptr;
    HIP_TRY(hipEventCreate(&e0));
    if (hipEventCreate(&e1) != hipSuccess) {
      (void)hipEventDestroy(e0);
      return fail(CARAMEL_EHIP, "hipEventCreate failed");
    }
    int rc = CARAMEL_OK;
    hipError_t he = hipStreamSynchronize(s);
    if (he == hipSuccess) he = hipEventRecord(e0, s);
    const auto t0 = std::chrono::steady_clock::now();
    for (uint32_t i = 0; i < n_calls && !rc && he == hipSuccess; ++i) rc = pipeline(p, s, true, direct);
    const auto t1 = std::chrono::steady_clock::now();
    if (he == hipSuccess) he = hipEventRecord(e1, s);
    if (he == hipSuccess) he = hipEventSynchronize(e1);
    float ms = 0.f;
    if (he == hipSuccess) he = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc) return rc;
    if (he != hipSuccess) return fail(CARAMEL_EHIP, "timing the loop: %s", hipGetErrorString(he));
    *host_us_per_call = std::chrono::duration<double, std::micro>(t1 - t0).count() / n_calls;
    *stream_us_per_call = double(ms) * 1e3 / n_calls;
    return CARAMEL_OK;
  });
}

int caramel_profile(caramel_plan* p, int enable) {
  if (int rc = need_bound(p, false)) return rc;
  for (int s = 0; s < 2; ++s)
    if (p->streams[s]) HIP_TRY(hipStreamSynchronize(p->streams[s]));
  drop_events(p);
  std::memset(p->stats, 0, sizeof p->stats);
  p->profiling = enable < 0 ? 0 : (enable > 2 ? 2 : enable);
  return CARAMEL_OK;
}

namespace {
int read_profile(caramel_plan* p, caramel_kernel_stat* out);
}

int caramel_profile_read(caramel_plan* p, caramel_kernel_stat* out) {
  return guarded([&] { return read_profile(p, out); });
}

}  // extern "C"

namespace {
int read_profile(caramel_plan* p, caramel_kernel_stat* out) {
  if (int rc = need_bound(p, false)) return rc;
  if (!out) return fail(CARAMEL_EINVAL, "out is NULL");
  // every pending stop event has completed once its own synchronize returns
  struct Window {
    float lo, hi;
    bool any;
  };
  size_t bi = 0;
  for (size_t i = 0; i < p->pending.size();) {
    const uint64_t call = p->pending[i].call;
    while (bi < p->call_base.size() && p->call_base[bi].first < call) ++bi;
    hipEvent_t base = (bi < p->call_base.size() && p->call_base[bi].first == call) ? p->call_base[bi].second : nullptr;
    Window win[CARAMEL_K_COUNT] = {};
    for (; i < p->pending.size() && p->pending[i].call == call; ++i) {
      TimedLaunch& t = p->pending[i];
      HIP_TRY(hipEventSynchronize(t.stop));
      float ms = 0.f;
      HIP_TRY(hipEventElapsedTime(&ms, t.start, t.stop));
      if (t.kind == CARAMEL_K_SEQUENCE) p->stats[t.kind].launches += 1;
      p->stats[t.kind].total_ms += ms;
      if (base) {
        float a = 0.f, b = 0.f;
        HIP_TRY(hipEventElapsedTime(&a, base, t.start));
        HIP_TRY(hipEventElapsedTime(&b, base, t.stop));
        Window& w = win[t.kind];
        if (!w.any) w = {a, b, true};
        w.lo = std::min(w.lo, a);
        w.hi = std::max(w.hi, b);
      }
      p->spare.push_back(t.start);
      p->spare.push_back(t.stop);
    }
    for (int k = 0; k < CARAMEL_K_COUNT; ++k)
      if (win[k].any) {
        p->stats[k].span_ms += double(win[k].hi) - double(win[k].lo);
        p->stats[k].calls += 1;
      }
  }
  p->pending.clear();
  for (auto& b : p->call_base) p->spare.push_back(b.second);
  p->call_base.clear();
  std::memcpy(out, p->stats, sizeof p->stats);
  return CARAMEL_OK;
}
}  // namespace

extern "C" {

const char* caramel_last_error(void) { return g_err.c_str(); }

int caramel_version(void) { return 100; }

}  // extern "C"
