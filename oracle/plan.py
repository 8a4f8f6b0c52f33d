"""CPU oracle, part 1: the transfer plan (batching, splitting, ring segments).

TEST INFRASTRUCTURE.  This package is the slow, plain reference the GPU library
is checked against.  Only tests, the smoke check and the benchmark's CPU
baseline may import it; the library never does, and the two share no code.

What is computed (all integer work, hence compared bit-exactly):

* Parameter batcher (paper section 4.2): parameters are visited in ascending
  order of update time.  One whose byte size reaches the threshold is sent on
  its own; a smaller one joins the currently open batch, and the batch is sent
  once its size has reached the threshold.  What is still open at the end is
  sent as the last batch.  Without timing information this size-only rule is
  the whole batcher (the paper's "the network is busy" case).
* Depth / chunking (section 4.4): a large transfer is cut into `depth` pieces
  that are aggregated independently and in parallel.  Three modes: no split,
  literal fixed-size chunks, and the adaptive rule (depth grows with the ratio
  size / threshold from 1 up to a cap of 8).
* Ring segments (section 2, ring/bucket pattern; section 4.4, multi-stage
  transfer with aggregation at each worker): a transfer unit is divided into W
  contiguous segments, one owned by each worker.  The paper does not say how;
  here segments are balanced over 16-byte granules so no 128-bit vector
  straddles two segments.

* Timing-aware batching (section 4.2, second half of the batching rule): when the
  caller also gives every parameter's expected update time and a linear model of
  the transfer time, transfers are served one at a time in queue order, and the
  open batch is additionally sent as soon as everything queued so far will have
  finished before the next parameter is updated (the network would otherwise idle).
* Threshold choice (section 4.2): with transfer time f(d) fitted as a + b*d from
  two measurements, the threshold is the smallest size x with f(2x) / (2 f(x)) > 0.8.

Readings of points the paper leaves open: equality with the threshold counts as
large; a large parameter does not flush the open batch; members of a batch
start on granule boundaries.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence

F32, BF16 = 0, 1
SPLIT_NONE, SPLIT_FIXED, SPLIT_ADAPTIVE = 0, 1, 2
KIND_BATCH, KIND_CHUNK = 0, 1
PATTERN_RING, PATTERN_HALVING_DOUBLING, PATTERN_SHUFFLE = 0, 1, 2


@dataclass(frozen=True)
class Config:
    world: int
    dtype: int = F32
    batch_threshold_bytes: int = 0
    split_mode: int = SPLIT_NONE
    max_depth: int = 8
    split_bytes: int = 0
    align_bytes: int = 16
    num_streams: int = 2
    pattern: int = PATTERN_RING

    @property
    def elem_size(self) -> int:
        return 4 if self.dtype == F32 else 2

    @property
    def granule(self) -> int:
        """Elements per alignment granule."""
        return self.align_bytes // self.elem_size


@dataclass
class Entry:
    tensor: int       # index into the caller's tensor list (update order)
    tensor_off: int   # first element of the tensor covered by this entry
    unit: int         # transfer unit the entry belongs to
    unit_off: int     # element offset inside the unit
    elems: int


@dataclass
class Unit:
    kind: int         # KIND_BATCH or KIND_CHUNK
    first_entry: int
    n_entries: int
    elems: int        # batch: padded to whole granules; chunk: exact
    fused_off: int    # batch: element offset in a replica's fused buffer; chunk: 0
    stream: int
    seg_start: List[int] = field(default_factory=list)   # W+1 element offsets


@dataclass
class Plan:
    cfg: Config
    n_tensors: int
    units: List[Unit]
    entries: List[Entry]
    fused_elems: int
    # timing-aware plans only: per unit, when it entered the queue, started and finished
    enqueue_time: List[float] = field(default_factory=list)
    start_time: List[float] = field(default_factory=list)
    finish_time: List[float] = field(default_factory=list)


def _align_up(x: int, a: int) -> int:
    return (x + a - 1) // a * a


def chunk_sizes(cfg: Config, elems: int) -> List[int]:
    """Section 4.4: element counts of the pieces one large transfer is cut into."""
    s = cfg.elem_size
    nbytes = elems * s
    if cfg.split_mode == SPLIT_NONE or nbytes <= cfg.split_bytes:
        return [elems]
    if cfg.split_mode == SPLIT_FIXED:
        piece = cfg.split_bytes // s
    else:
        depth = min(max(nbytes // cfg.split_bytes, 1), cfg.max_depth)
        piece = _align_up(-(-elems // depth), cfg.granule)
    out = []
    left = elems
    while left > 0:
        take = min(piece, left)
        out.append(take)
        left -= take
    return out


def ring_segments(cfg: Config, unit_elems: int) -> List[int]:
    """W+1 element offsets; segment c = [seg[c], seg[c+1]) is owned by worker c."""
    g, w = cfg.granule, cfg.world
    q = -(-unit_elems // g)
    base, rem = divmod(q, w)
    out = []
    for c in range(w + 1):
        gran = c * base + min(c, rem)
        out.append(min(gran * g, unit_elems))
    return out


def validate(cfg: Config, elems: Sequence[int]) -> None:
    if cfg.world < 1:
        raise ValueError("world must be >= 1")
    if cfg.dtype not in (F32, BF16):
        raise ValueError("dtype")
    a = cfg.align_bytes
    if a <= 0 or a & (a - 1) or a % cfg.elem_size:
        raise ValueError("align_bytes must be a power of two and a multiple of the element size")
    if cfg.num_streams not in (1, 2):
        raise ValueError("num_streams")
    if cfg.split_mode not in (SPLIT_NONE, SPLIT_FIXED, SPLIT_ADAPTIVE):
        raise ValueError("split_mode")
    if cfg.split_mode != SPLIT_NONE:
        if cfg.split_bytes <= 0 or cfg.split_bytes % a:
            raise ValueError("split_bytes must be a positive multiple of align_bytes")
    if cfg.split_mode == SPLIT_ADAPTIVE and cfg.max_depth < 1:
        raise ValueError("max_depth")
    if cfg.pattern not in (PATTERN_RING, PATTERN_HALVING_DOUBLING, PATTERN_SHUFFLE):
        raise ValueError("pattern")
    if cfg.pattern == PATTERN_HALVING_DOUBLING and cfg.world & (cfg.world - 1):
        raise ValueError("halving-doubling needs a power-of-two world")
    if len(elems) == 0:
        raise ValueError("no tensors")
    if any(e <= 0 for e in elems):
        raise ValueError("zero-element tensor")


def build_plan(cfg: Config, elems: Sequence[int], ready_time: Sequence[float] = None,
               net_a: float = 0.0, net_b: float = 0.0) -> Plan:
    """Walk the tensors in update order and emit transfer units in queue order.

    With `ready_time` (non-decreasing update times, one per tensor) the network is modelled too:
    a transfer of d bytes takes net_a + net_b * d, transfers are served one after the other in
    queue order, and the open batch is also sent when the queue will have drained before the
    next tensor's update time.  Times are IEEE doubles, evaluated exactly in the order written
    here."""
    validate(cfg, elems)
    timed = ready_time is not None
    if timed:
        if len(ready_time) != len(elems):
            raise ValueError("ready_time must have one entry per tensor")
        if any(not (ready_time[i] <= ready_time[i + 1]) for i in range(len(elems) - 1)):
            raise ValueError("ready_time must be non-decreasing")
        if not (net_a >= 0.0 and net_b >= 0.0):
            raise ValueError("network model coefficients must be non-negative")
    s, g, t_bytes = cfg.elem_size, cfg.granule, cfg.batch_threshold_bytes
    units: List[Unit] = []
    entries: List[Entry] = []
    fused_elems = 0
    open_batch: List[Entry] = []     # members of the active batch (unit id filled at close)
    open_elems = 0
    free_at = 0.0                    # when the network has finished everything queued so far
    enq: List[float] = []
    start: List[float] = []
    fin: List[float] = []

    def emit(kind: int, members: List[Entry], n: int, now: float) -> None:
        nonlocal fused_elems, free_at
        u = len(units)
        for m in members:
            m.unit = u
        fused_off = 0
        if kind == KIND_BATCH:
            fused_off = fused_elems
            fused_elems += n
        units.append(Unit(kind, len(entries), len(members), n, fused_off,
                          u % cfg.num_streams, ring_segments(cfg, n)))
        entries.extend(members)
        if timed:
            begin = max(now, free_at)
            free_at = begin + (net_a + net_b * float(n * s))
            enq.append(now)
            start.append(begin)
            fin.append(free_at)

    for t, n in enumerate(elems):
        now = float(ready_time[t]) if timed else 0.0
        if t_bytes == 0 or n * s >= t_bytes:
            off = 0
            for piece in chunk_sizes(cfg, n):
                emit(KIND_CHUNK, [Entry(t, off, -1, 0, piece)], piece, now)
                off += piece
            continue
        at = _align_up(open_elems, g)
        open_batch.append(Entry(t, 0, -1, at, n))
        open_elems = at + n
        full = _align_up(open_elems, g) * s >= t_bytes
        idle_ahead = timed and t + 1 < len(elems) and free_at <= float(ready_time[t + 1])
        if full or idle_ahead:
            emit(KIND_BATCH, open_batch, _align_up(open_elems, g), now)
            open_batch, open_elems = [], 0
    if open_batch:
        emit(KIND_BATCH, open_batch, _align_up(open_elems, g), float(ready_time[-1]) if timed else 0.0)
    return Plan(cfg, len(elems), units, entries, fused_elems, enq, start, fin)


# ---------------------------------------------------------------- threshold choice (section 4.2)
def fit_linear(bytes1: int, time1: float, bytes2: int, time2: float):
    """The line through two (size, transfer time) measurements: time = a + b * size."""
    from fractions import Fraction
    if bytes1 == bytes2:
        raise ValueError("the two sizes must differ")
    b = (Fraction(time2) - Fraction(time1)) / (bytes2 - bytes1)
    a = Fraction(time1) - b * bytes1
    return a, b


def threshold_from_model(a, b) -> int:
    """Smallest integer size x >= 1 with f(2x) / (2 f(x)) > 0.8 for f(d) = a + b*d, by exact
    rational arithmetic.  (a + 2bx) / (2a + 2bx) > 4/5  <=>  2bx > 3a  <=>  x > 3a / (2b).)"""
    from fractions import Fraction
    a, b = Fraction(a), Fraction(b)
    if a < 0 or b <= 0:
        raise ValueError("need a >= 0 and b > 0")
    x = (3 * a) // (2 * b) + 1
    return max(int(x), 1)
