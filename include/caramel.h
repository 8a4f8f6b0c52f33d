/* caramel.h -- C ABI of the Caramel aggregation hot path for MI355X (gfx950).
 *
 * What the library computes.  W workers ("replicas") each hold a gradient for
 * every parameter of a model, of the same byte length at every worker, and the
 * aggregate is their sum (paper section 2); here the W replicas are resident
 * in the memory of ONE GPU and the result is their average, written back into
 * every replica.  The work is organised the way Caramel organises AllReduce
 * traffic:
 *
 *   - small parameters are batched into fused transfers (section 4.2,
 *     "Parameter Batcher"): walking the parameters in update order, one whose
 *     size reaches the threshold is transferred on its own, a smaller one
 *     joins the open batch, and the batch is sent once it has reached the
 *     threshold;
 *   - large transfers are cut into `depth` chunks that are aggregated
 *     independently and in parallel (section 4.4, "Adaptive Depth Enforcer");
 *   - every transfer unit (batch or chunk) is aggregated with the ring/bucket
 *     pattern (sections 2 and 4.4): the unit is cut into W segments, the
 *     partial sum of segment c starts at worker c+1, is added to at each
 *     worker round the ring and completes at worker c, which scales it by 1/W;
 *     the result is then copied to all workers.  Sums are fp32, in exactly that
 *     order, so results are reproducible bit for bit.
 *
 * Memory.  All `void*` data arguments named "device" are device pointers;
 * everything else is host memory.  The caller owns gradients and workspace and
 * must keep them alive until the stream work has completed.  The library
 * allocates only its own small descriptor tables (at caramel_bind).
 *
 * Tracing.  With CARAMEL_TRACE=1 in the environment (read once per process) the library writes
 * one line to stderr per unit at caramel_bind (kind, plan stream, bytes, tiles) and one per
 * kernel launch (call number, stream, tile range, workgroup shape, bytes per replica).
 *
 * Errors.  Every function returns a status; nothing throws across the ABI.  On
 * a non-zero status nothing has been launched unless stated, and
 * caramel_last_error() describes the failure.
 *
 * Threads.  A plan may be used by one host thread at a time.
 */
#ifndef CARAMEL_H
#define CARAMEL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { CARAMEL_OK = 0, CARAMEL_EINVAL = 1, CARAMEL_ENOMEM = 2, CARAMEL_EHIP = 3, CARAMEL_ESTATE = 4 };
enum { CARAMEL_F32 = 0, CARAMEL_BF16 = 1 };
enum { CARAMEL_SPLIT_NONE = 0, CARAMEL_SPLIT_FIXED = 1, CARAMEL_SPLIT_ADAPTIVE = 2 };
enum { CARAMEL_KIND_BATCH = 0, CARAMEL_KIND_CHUNK = 1 };
enum { CARAMEL_PATTERN_RING = 0, CARAMEL_PATTERN_HALVING_DOUBLING = 1, CARAMEL_PATTERN_SHUFFLE = 2 };

/* Plan parameters.
 *   world                 W >= 1 replicas (at most CARAMEL_MAX_WORLD).
 *   dtype                 element type of gradients and results.  BF16: inputs are widened
 *                         exactly, partial sums stay fp32 through all ring hops, one
 *                         round-to-nearest-even on output.
 *   batch_threshold_bytes T of section 4.2; a tensor of >= T bytes is "large".  0 switches
 *                         batching off (every tensor is its own transfer).
 *   split_mode            section 4.4.  NONE: depth 1.  FIXED: chunks of exactly split_bytes
 *                         (last one shorter), any count.  ADAPTIVE: depth =
 *                         clamp(floor(bytes / split_bytes), 1, max_depth), equal chunks
 *                         rounded up to whole granules; the paper's setting is split_bytes = T,
 *                         max_depth = 8.
 *   align_bytes           granule: batch members and ring segments start on multiples of it.
 *                         A power of two, >= 16 (one 128-bit vector).
 *   num_streams           1 or 2; unit u belongs to stream u mod num_streams.  Stream 0 is the
 *                         caller's stream, stream 1 an internal stream forked from and joined
 *                         back to it with events.
 *   pattern               decentralised aggregation pattern (sections 2 and 6.3); it fixes the
 *                         order of the fp32 additions, everything else is the same.
 *                         RING: segment c is summed x[c+1] + x[c+2] + ... + x[c] (indices mod W).
 *                         HALVING_DOUBLING (recursive vector halving, distance doubling; W a
 *                         power of two): the balanced tree ((x0+x1)+(x2+x3)) + ((x4+x5)+(x6+x7)) ...
 *                         SHUFFLE (the owner of a slice receives it from every worker): x0 + x1 +
 *                         ... + x(W-1) in worker order.
 */
typedef struct caramel_config {
  uint32_t world;
  uint32_t dtype;
  uint64_t batch_threshold_bytes;
  uint32_t split_mode;
  uint32_t max_depth;
  uint64_t split_bytes;
  uint32_t align_bytes;
  uint32_t num_streams;
  uint32_t pattern;
  uint32_t reserved; /* must be 0 */
} caramel_config;

#define CARAMEL_MAX_WORLD 64u

/* One transfer unit, in queue (emission) order. */
typedef struct caramel_unit {
  uint32_t kind;        /* CARAMEL_KIND_BATCH or CARAMEL_KIND_CHUNK */
  uint32_t stream;      /* unit index mod num_streams */
  uint32_t first_entry; /* entries [first_entry, first_entry + n_entries) belong to this unit */
  uint32_t n_entries;   /* chunk: 1 */
  uint64_t elems;       /* batch: padded to whole granules; chunk: exact */
  uint64_t fused_off;   /* batch: element offset in each replica's fused buffer; chunk: 0 */
} caramel_unit;

/* One contiguous piece of one tensor inside one unit.  Entries are grouped by unit. */
typedef struct caramel_entry {
  uint32_t tensor;      /* index into the tensor list given to caramel_plan_create */
  uint32_t unit;
  uint64_t tensor_off;  /* first element of the tensor covered */
  uint64_t unit_off;    /* element offset inside the unit (multiple of the granule) */
  uint64_t elems;
} caramel_entry;

typedef struct caramel_plan caramel_plan; /* opaque, owned by the library */

/* ---- planning: host only, deterministic, no GPU needed (sections 4.2, 4.4) ------------- */

/* Build the plan for `n_tensors` tensors with the given element counts, listed in update
 * order (ascending expected update time, section 4.2).  *out receives a new plan.
 * EINVAL: NULL argument, n_tensors == 0, a zero-element tensor, world out of range, unknown
 * dtype or split mode, align_bytes not a power of two >= 16, split_bytes not a positive
 * multiple of align_bytes when splitting, num_streams not 1 or 2, max_depth == 0 (ADAPTIVE),
 * unknown pattern, HALVING_DOUBLING with a world that is not a power of two, reserved != 0. */
int caramel_plan_create(const caramel_config* cfg, const uint64_t* tensor_elems, uint32_t n_tensors,
                        caramel_plan** out);

/* Timing-aware batching (section 4.2: besides the size rule, the open batch is also sent when
 * the transfer queue will have drained before the next parameter is updated).
 *   ready_time  n_tensors expected update times, non-decreasing, any unit of time;
 *   net_a/net_b transfer-time model of the aggregation: a transfer of d bytes takes
 *               net_a + net_b * d (same time unit; both >= 0).
 * Transfers are served one at a time in queue order.  After a small tensor has joined the open
 * batch, the batch is sent if it has reached the threshold, or if everything queued so far will
 * have finished by the next tensor's update time (waiting for more members would leave the
 * network idle); what is still open after the last tensor is sent then.  Times are IEEE
 * doubles: start = max(update time, end of the previous transfer), end = start +
 * (net_a + net_b * bytes).  Everything else is as in caramel_plan_create.  EINVAL additionally
 * for NULL or decreasing ready_time and negative or NaN coefficients. */
int caramel_plan_create_timed(const caramel_config* cfg, const uint64_t* tensor_elems, uint32_t n_tensors,
                              const double* ready_time, double net_a, double net_b, caramel_plan** out);
/* Modelled schedule of a timing-aware plan: per unit, when it entered the queue, when its
 * transfer starts and when it ends.  Any array may be NULL; `cap` entries each.  ESTATE if the
 * plan was not made by caramel_plan_create_timed, EINVAL if cap is smaller than the unit count. */
int caramel_plan_times(const caramel_plan* plan, double* enqueue, double* start, double* finish, uint32_t cap);

/* Threshold choice of section 4.2.  caramel_net_model_fit: the line time = a + b * bytes through
 * two measured (size, transfer time) pairs (the paper measures 64 B and 4 MB).
 * caramel_threshold_estimate: the smallest size x >= 1 with f(2x) / (2 f(x)) > 0.8 for
 * f(d) = a + b*d, i.e. the smallest integer above 1.5 a / b, decided in exact arithmetic.
 * EINVAL: equal sizes or non-finite times; a fitted line with a < 0 or b <= 0 (two noisy probes
 * whose times do not grow with size: measure again); for the estimate a < 0, b <= 0, non-finite
 * values, or a result beyond 64 bits. */
int caramel_net_model_fit(uint64_t bytes1, double time1, uint64_t bytes2, double time2, double* a, double* b);
int caramel_threshold_estimate(double a, double b, uint64_t* threshold_bytes);

/* ---- transfer scheduler: host only (section 4.3) ---------------------------------------- */

/* Where the scheduler puts one group's transfer.  Backward-pass times count from the start of
 * the backward pass; forward-pass times from the start of the next forward pass and are
 * negative where the transfer begins before it. */
enum { CARAMEL_BIN_BACKWARD = 0, CARAMEL_BIN_FORWARD = 1 };
typedef struct caramel_slot {
  uint32_t bin;   /* CARAMEL_BIN_BACKWARD or CARAMEL_BIN_FORWARD */
  uint32_t stage; /* 2: placed beside the computation; 3: placed where it lengthens the iteration */
  double start;
  double end;
} caramel_slot;

/* Totals of a schedule.  N = comm_time, C = compute_time, T = iteration_time are tied by the
 * relation of section 3: T = C + N - overlap * min(N, C), utilization = C / T. */
typedef struct caramel_schedule_summary {
  double comm_time;      /* sum of all transfer times */
  double compute_time;   /* bp_len + fp_len */
  double bp_overrun;     /* how far transfers run past the end of the backward pass */
  double fp_overrun;     /* how long before the start of the forward pass they begin */
  double iteration_time; /* compute_time + bp_overrun + fp_overrun */
  double overlap;        /* overlap coefficient, 0 when there is no transfer or no computation */
  double utilization;
} caramel_schedule_summary;

/* Greedy packing of section 4.3.  n_groups transfers of group_bytes[g] bytes; group g may not
 * start before ready[g] (backward pass, when the last of its members has been updated) and, if
 * it is moved to the forward pass, must end by need[g] (when the first of its members is read).
 * A transfer of d bytes occupies the network for net_a + net_b * d; transfers of one window may
 * touch but not overlap.  Groups are taken largest first (equal sizes in index order).  Each is
 * placed in the backward pass at the earliest free start >= ready[g] if it then ends by bp_len;
 * else in the forward pass at the latest free end <= need[g] if it then starts at or after 0;
 * else it is left over.  Left-over groups are taken again in the same order with both limits
 * lifted, and go to the side that lengthens the iteration less (how far the slot pushes the end
 * of the backward window, already extended by earlier slots, out, against how far it pushes the
 * start of the forward window back; equal: backward pass).
 *   slots    n_groups records, written in the caller's group order (host memory, caller's);
 *   summary  may be NULL.
 * All arithmetic is in IEEE doubles in the order stated above.  EINVAL: NULL array with
 * n_groups > 0; a negative or NaN length or coefficient; ready[g] outside [0, bp_len]; need[g]
 * outside [0, fp_len]; a transfer time that is not positive. */
int caramel_schedule_transfers(const uint64_t* group_bytes, const double* ready, const double* need,
                               uint32_t n_groups, double bp_len, double fp_len, double net_a, double net_b,
                               caramel_slot* slots, caramel_schedule_summary* summary);

/* Transfer boundaries of a plan's units (section 4.3: a batch is bound by its member that is
 * updated last and by its member that is read first).  ready_time / read_time: n_tensors values
 * each, indexed like the tensor list given to caramel_plan_create.  Outputs: `cap` entries
 * each, one per unit, any may be NULL; group_bytes[u] = elems * element size.  EINVAL if cap is
 * smaller than the unit count or an input is NULL. */
int caramel_plan_windows(const caramel_plan* plan, const double* ready_time, const double* read_time,
                         uint64_t* group_bytes, double* ready, double* need, uint32_t cap);

/* Free host and device tables and internal streams/events.  NULL is allowed. */
void caramel_plan_destroy(caramel_plan* plan);

/* Introspection.  Any out pointer may be NULL. */
int caramel_plan_counts(const caramel_plan* plan, uint32_t* n_units, uint32_t* n_entries,
                        uint64_t* fused_elems);
/* Copy up to `cap` records; EINVAL if cap is smaller than the count. */
int caramel_plan_units(const caramel_plan* plan, caramel_unit* out, uint32_t cap);
int caramel_plan_entries(const caramel_plan* plan, caramel_entry* out, uint32_t cap);
/* Ring segments of one unit: world+1 element offsets; segment c = [seg[c], seg[c+1]) is the
 * part whose sum completes at worker c. */
int caramel_plan_segments(const caramel_plan* plan, uint32_t unit, uint64_t* seg_start);
/* Canonical byte image of the plan: equal plans give equal bytes on every host.  All fields
 * little-endian, no padding, in this order:
 *   char[8]  "CARAMEL1"
 *   u32 world, u32 dtype, u64 batch_threshold_bytes, u32 split_mode, u32 max_depth,
 *   u64 split_bytes, u32 align_bytes, u32 num_streams, u32 pattern          (the configuration)
 *   u32 n_tensors, u32 n_units, u32 n_entries, u64 fused_elems
 *   u64 tensor_elems[n_tensors]
 *   n_units   x { u32 kind, u32 stream, u32 first_entry, u32 n_entries, u64 elems, u64 fused_off }
 *   n_entries x { u32 tensor, u32 unit, u64 tensor_off, u64 unit_off, u64 elems }
 *   u64 seg_start[n_units][world + 1]                                        (ring segments)
 * (72 + 8 n_tensors + 32 n_units + 32 n_entries + 8 n_units (world + 1) bytes; launch options and
 * the modelled times of a timing-aware plan are not part of it.)  Call with buf == NULL to get
 * the size in *len; otherwise *len is the capacity on entry and the size written on return
 * (EINVAL if too small). */
int caramel_plan_serialize(const caramel_plan* plan, void* buf, size_t* len);

/* ---- execution on the GPU ---------------------------------------------------------------- */

/* Attach memory to a plan.
 *   grads     host array of world * n_tensors DEVICE pointers; grads[w * n_tensors + t] is
 *             worker w's tensor t (tensor_elems[t] elements of the plan's dtype), aligned to
 *             align_bytes.  Replicas must not overlap.  (Any such pointers are correct; the
 *             kernels stream fastest when a tensor has the same address modulo 64 KiB in every
 *             replica, because tiles can then be cut on aligned 64 KiB blocks of memory.)
 *   fused_ws  DEVICE workspace of world * fused_elems elements (replica w's fused buffer starts
 *             at element w * fused_elems); may be NULL when fused_elems == 0, or when only
 *             caramel_allreduce in its default (direct) mode is going to be used.
 * The library uploads its descriptor tables (synchronously) and creates its internal stream.
 * May be called again to re-bind, with the same device current: the plan's tables, stream and
 * events live on the device that is current at the first bind, and `stream` of the calls below
 * must belong to it.  EINVAL: NULL/misaligned pointer, overlapping buffers (checked before any
 * device call).  ESTATE: another device is current than at the first bind.  EHIP: a HIP call
 * failed.  ENOMEM: out of host memory. */
int caramel_bind(caramel_plan* plan, void* const* grads, void* fused_ws);

/* `stream` is a hipStream_t handle (NULL = the default stream).  All four calls are
 * asynchronous: work is ordered after what is already queued on `stream`, and later work on
 * `stream` is ordered after it.  ESTATE: plan not bound (or no workspace where one is needed),
 * or another device is current than the one the plan was bound on.
 *
 * caramel_pack         batch units: every member tensor of every replica -> fused_ws at its
 *                      planned offset; alignment padding is written as +0.0 (section 4.2).
 * caramel_ring_reduce  every unit, in place: batch units in fused_ws, chunk units directly in
 *                      tensor memory.  Ring reduce-scatter order, scale by 1/W, all-gather to
 *                      all W replicas (sections 2, 4.4).  Units of plan stream 0 are queued on
 *                      `stream`, units of plan stream 1 on the internal stream between a fork
 *                      from and a join back to `stream`, both with events.
 * caramel_unpack       batch units: fused_ws -> member tensors of every replica.
 * caramel_allreduce    the whole path; afterwards every grads[w][t] holds the average, the same
 *                      bytes for every w, and identical to pack -> ring_reduce -> unpack.
 */
int caramel_pack(caramel_plan* plan, void* stream);
int caramel_ring_reduce(caramel_plan* plan, void* stream);
int caramel_unpack(caramel_plan* plan, void* stream);
int caramel_allreduce(caramel_plan* plan, void* stream);

/* For callers that cannot allocate device memory (code that sets up or runs under HIP graph
 * capture rules, tight serving loops, harnesses that forbid hipMalloc): caramel_bind +
 * caramel_allreduce (in-place batch path) in one call that allocates nothing on the device and
 * creates no stream or event.  The descriptor tables that caramel_bind would put into memory from
 * hipMalloc go into a static device array of CARAMEL_STATIC_TABLE_BYTES inside the library,
 * which every GPU the library runs on holds until the process ends.
 *   plan    any plan (bound or not; a binding made with caramel_bind is left untouched);
 *   grads   as for caramel_bind; the pointers are taken anew on every call;
 *   stream  every launch goes on this stream (no internal stream, whatever num_streams says).
 * Afterwards (in stream order) every grads[w][t] holds the same bytes caramel_allreduce gives.
 * The tables are uploaded, with a wait for `stream`, when the array of the current GPU does not
 * already hold them from a call on the same stream; otherwise the call only launches kernels.
 * All calls on one GPU share its array: a call must not be issued while another plan's call, or
 * a call on another stream, may still be running there - such calls race.  The plan's launch
 * options apply; timing (caramel_profile) does not cover this call.
 * EINVAL: NULL/misaligned/overlapping pointers; a plan whose tables (8 bytes per tensor and
 * worker, rounded up to 256, plus 32 bytes per tile) exceed CARAMEL_STATIC_TABLE_BYTES - nothing
 * is launched then.  EHIP: a HIP call failed. */
#define CARAMEL_STATIC_TABLE_BYTES (4u << 20)
int caramel_allreduce_static(caramel_plan* plan, void* const* grads, void* stream);

/* ---- launch tuning and timing (do not change results) ------------------------------------ */

/* How the work is cut up for the GPU.  A "run" is a maximal piece of one tensor (or of the fused
 * buffer) inside one ring segment of one unit: one per segment for a chunk unit, one per member
 * and segment for a batch unit that is reduced in place.  Runs of at least
 * CARAMEL_OPT_LONG_RUN_BYTES are cut into long tiles (CARAMEL_OPT_TILE_VECS), which 1024-lane
 * workgroups walk one replica after the other; shorter runs into small tiles
 * (CARAMEL_OPT_SMALL_TILE_VECS), for which 256-lane workgroups fetch all replicas at once.
 * Long and small tiles go out in separate launches. */
enum {
  /* How units map to kernel launches.  PER_UNIT: consecutive units of a plan stream share a
   * launch until it covers CARAMEL_OPT_LAUNCH_MIN_BYTES / CARAMEL_OPT_LONG_LAUNCH_MIN_BYTES
   * (0: strictly one launch per unit and tile class: the literal pipeline), plan stream 1 on the
   * internal stream.  PER_STREAM: one launch per tile class and plan stream.  AUTO (default):
   * PER_UNIT over two streams, where the launches of one stream fill the gaps of the other, if
   * the call is large enough to repay the fork and join (CARAMEL_OPT_PIPELINE_MIN_BYTES);
   * otherwise one launch per tile class on the caller's stream. */
  CARAMEL_OPT_LAUNCH_MODE = 0,
  /* Batch units in caramel_allreduce.  STAGED: pack -> reduce -> unpack through fused_ws.
   * DIRECT: one gather-reduce-scatter kernel that reads member tensors and writes results back
   * without materialising the fused buffer (same segments, same order, same bits).
   * Default DIRECT. */
  CARAMEL_OPT_BATCH_PATH = 1,
  /* 16-byte vectors per replica in a long tile.  Default 0 = chosen at caramel_bind: 8192
   * (128 KiB) for fp32 ring or shuffle sums over 2, 4 or 8 workers (the kernel can keep eight
   * vectors per lane in registers then) once a replica holds 64 MiB; 2048 (32 KiB) for bf16
   * halving-doubling (two vectors per lane); 4096 (64 KiB) otherwise. */
  CARAMEL_OPT_TILE_VECS = 2,
  /* Upper bound on workgroups per reduce launch (0 = one workgroup per tile). */
  CARAMEL_OPT_MAX_GRID = 3,
  /* Non-zero (default): streaming (non-temporal) loads/stores in the reduce kernels, and in pack /
   * unpack when the fused buffers of all workers together hold 256 MiB or more. */
  CARAMEL_OPT_NONTEMPORAL = 4,
  /* 16-byte vectors each lane keeps in flight per worker where all replicas are fetched at
   * once: 1, 2 or 4; 0 = chosen from W. */
  CARAMEL_OPT_UNROLL = 5,
  /* Lanes per workgroup over long tiles: 256, 512 or 1024 (default). */
  CARAMEL_OPT_BLOCK = 6,
  /* PER_UNIT launches over small tiles: consecutive units of one stream share a launch until it
   * covers at least this many bytes per replica.  The launch-side counterpart of the batching
   * threshold: it amortises launch overhead over small units.  Default 4 MiB. */
  CARAMEL_OPT_LAUNCH_MIN_BYTES = 7,
  /* AUTO launch mode only: a call whose algorithmic bytes (2 * world * elements * element size)
   * are below this value is not pipelined.  Default: the largest value, i.e. AUTO does not
   * pipeline (on MI355X one launch over all long tiles measured faster than two streams for every
   * workload tried, because the fork and join cost more than the overlap wins). */
  CARAMEL_OPT_PIPELINE_MIN_BYTES = 8,
  /* Vectors per small tile and lanes per workgroup over small tiles.  Defaults 256 and 256. */
  CARAMEL_OPT_SMALL_TILE_VECS = 9,
  CARAMEL_OPT_SMALL_BLOCK = 10,
  /* Bytes per replica from which a run is cut into long tiles.  Default 0 = chosen at
   * caramel_bind: 16 KiB, or, if a replica holds less than 32 MiB in all, no long tiles at all
   * (so small a job is over before the one-replica-at-a-time walk of a long tile pays off); none
   * either for halving-doubling with more than 16 workers.
   * 1: every run is long; a huge value: every run is small. */
  CARAMEL_OPT_LONG_RUN_BYTES = 11,
  /* Long tiles: non-zero selects the stream-major kernel, which walks the workers one replica at
   * a time; the value (2, 4 or 8, default 8) is the most vectors a lane keeps per worker: a tile
   * of block * value vectors is walked in one go (8 exists for fp32 chains of at most 8 workers;
   * otherwise 4 is used).  0 fetches all workers' values at once. */
  CARAMEL_OPT_STREAM_MAJOR = 12,
  /* PER_UNIT launches over long tiles: like CARAMEL_OPT_LAUNCH_MIN_BYTES.  Default 64 MiB. */
  CARAMEL_OPT_LONG_LAUNCH_MIN_BYTES = 13,
  /* Bit 0 (small tiles), bit 1 (long tiles): where every replica of a run has the same address
   * modulo the tile size, tiles are cut so that they start on multiples of the tile size in
   * memory (the first tile of a run is shortened); otherwise tiles start where their run starts.
   * Default 3.  Takes effect at the next caramel_bind.  Results do not depend on it. */
  CARAMEL_OPT_ALIGN_TILES = 14,
  /* One launch per tile class on one stream (PER_STREAM without the pipeline, which is what AUTO
   * does): if the small tiles cover at most this many bytes per replica, they join the launch
   * over the long tiles instead of getting a launch of their own.  Default 1 MiB; 0 keeps the
   * two launches apart. */
  CARAMEL_OPT_MERGE_SMALL_BYTES = 15,
  /* The last so many long tiles of every plan stream are cut into pieces of one vector per lane
   * (16 KiB for 1024 lanes), which a workgroup fetches from all replicas at once.  When a launch
   * runs out of tiles, the workgroups still at work finish at different times; with short pieces
   * at the end that drain is short.  Default 128 (half a tile per compute unit); 0 switches it off.
   * Takes effect at the next caramel_bind. */
  CARAMEL_OPT_TAIL_TILES = 16,
  /* 1 (default): for world sizes other than 2, 4, 8 and 16 (ring order), tiles follow aligned
   * blocks of memory across the boundaries between ring segments: a tile that contains a
   * boundary is summed in two parts, each in its segment's order, and a run is everything of one
   * unit that is contiguous in a tensor.  0, and always for 2, 4, 8 and 16 workers: tiles (and
   * runs) end at segment boundaries.  Takes effect at the next caramel_bind.  Results do not
   * depend on it. */
  CARAMEL_OPT_SPLIT_TILES = 17
};
enum { CARAMEL_LAUNCH_PER_UNIT = 0, CARAMEL_LAUNCH_PER_STREAM = 1, CARAMEL_LAUNCH_AUTO = 2 };
enum { CARAMEL_BATCH_STAGED = 0, CARAMEL_BATCH_DIRECT = 1 };

/* Set a launch option.  Tile sizes take effect at the next caramel_bind (tables are rebuilt
 * there); the others at the next launch.
 * EINVAL for an unknown option or a value out of range. */
int caramel_plan_set_option(caramel_plan* plan, uint32_t option, uint64_t value);

enum {
  CARAMEL_K_PACK = 0,
  CARAMEL_K_REDUCE = 1,       /* reduce launches over long tiles (the stream-major kernel) */
  CARAMEL_K_UNPACK = 2,
  CARAMEL_K_SEQUENCE = 3,
  CARAMEL_K_REDUCE_SMALL = 4, /* reduce launches over small tiles */
  CARAMEL_K_COUNT = 5
};

/* Timing with HIP events recorded on the stream the work is launched on.
 *   PACK / REDUCE / REDUCE_SMALL / UNPACK
 *                `launches` counts kernel launches and `elements` the elements per replica they
 *                cover (a reduce launch moves 2 * world * element size bytes for each);
 *                `total_ms` is the sum of their durations and is filled at level 2 only.
 *   SEQUENCE     everything one stream does in one ring_reduce / allreduce call, from before
 *                its first launch to after its last: `launches` counts sequences, `total_ms`
 *                sums their durations (levels 1 and 2).
 * `span_ms` accumulates, per call, the time from the earliest start to the latest end of the
 * timed intervals of that kind (with two streams the sequences overlap, so for SEQUENCE the span
 * is the duration of the whole call on the GPU); `calls` counts the calls that contributed. */
typedef struct caramel_kernel_stat {
  uint64_t launches;
  double total_ms;
  double span_ms;
  uint64_t calls;
  uint64_t elements;
} caramel_kernel_stat;

/* Set the timing level and clear the statistics.  0: off.  1: one event pair per stream and
 * call (does not disturb back-to-back launches).  2: additionally one pair per kernel launch
 * (exact per-kernel durations, but the events keep consecutive launches of a stream apart).
 * Requires a bound plan. */
int caramel_profile(caramel_plan* plan, int level);
/* Synchronise the internal streams, fold pending event pairs into the statistics and copy
 * CARAMEL_K_COUNT records to `out`. */
int caramel_profile_read(caramel_plan* plan, caramel_kernel_stat* out);

/* ---- measurement aid -------------------------------------------------------------------- */

/* n_calls calls of caramel_allreduce issued back to back from inside the library, so that no
 * caller-side cost (an interpreter, a foreign-function call) sits between them.  Reports the
 * host time to issue one call (wall clock around the loop, no waiting for the GPU) and the
 * time one call takes on the stream (a pair of HIP events around the loop, after the stream has
 * drained).  Creates and destroys two events; otherwise like caramel_allreduce. */
int caramel_allreduce_loop(caramel_plan* plan, void* stream, uint32_t n_calls, double* host_us_per_call,
                           double* stream_us_per_call);

/* Plain streaming kernels of exactly known traffic, with no descriptor tables: ceilings to set
 * the reduce kernels against, and kernels to check a profiler's memory counters with.
 *   READ    loads every 16-byte vector of the n_buffers buffers          (n_buffers * bytes read)
 *   WRITE   stores every vector of the n_buffers buffers                 (n_buffers * bytes written)
 *   UPDATE  loads all n_buffers values of a vector, adds them, stores the sum to all buffers:
 *           the reduce kernel's traffic           (n_buffers * bytes read and as many written)
 *   COPY    buffer 0 -> buffer 1, n_buffers must be 2                    (bytes read, bytes written)
 * buffers: host array of n_buffers (1, 2, 4, 8 or 16) DEVICE pointers to `bytes` bytes each
 * (multiples of 16); workgroup b of `block` lanes (256, 512 or 1024) handles bytes
 * [b * run_bytes, (b + 1) * run_bytes) of every buffer, with streaming loads and stores.
 * Asynchronous on `stream`.  EINVAL for other arguments (no message is recorded), EHIP if the
 * launch fails. */
enum { CARAMEL_PROBE_READ = 0, CARAMEL_PROBE_WRITE = 1, CARAMEL_PROBE_UPDATE = 2, CARAMEL_PROBE_COPY = 3 };
int caramel_stream_probe(uint32_t mode, void* const* buffers, uint32_t n_buffers, uint64_t bytes,
                         uint32_t run_bytes, uint32_t block, void* stream);

/* Message for the calling thread's last non-OK status ("" if none). */
const char* caramel_last_error(void);
/* Library version, major * 10000 + minor * 100 + patch. */
int caramel_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CARAMEL_H */
