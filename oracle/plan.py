"""CPU oracle, part 1: the transfer plan (batching, splitting, ring segments).

TEST INFRASTRUCTURE.  This package is the slow, plain reference the GPU library
is checked against.  Only tests, the smoke check and the benchmark's CPU
baseline may import it; the library never does, and the two share no code.

What is computed (all integer work, hence compared bit-exactly):

* Parameter batcher (paper section 4.2): parameters are visited in ascending
  order of update time.  One whose byte size reaches the threshold is sent on
  its own; a smaller one joins the currently open batch, and the batch is sent
  once its size has reached the threshold.  What is still open at the end is
  sent as the last batch.  The size-only rule corresponds to the paper's "the
  network is busy" case; the clause that also flushes a batch when the queue
  has drained needs a timing model and is not part of this plan.
* Depth / chunking (section 4.4): a large transfer is cut into `depth` pieces
  that are aggregated independently and in parallel.  Three modes: no split,
  literal fixed-size chunks, and the adaptive rule (depth grows with the ratio
  size / threshold from 1 up to a cap of 8).
* Ring segments (section 2, ring/bucket pattern; section 4.4, multi-stage
  transfer with aggregation at each worker): a transfer unit is divided into W
  contiguous segments, one owned by each worker.  The paper does not say how;
  here segments are balanced over 16-byte granules so no 128-bit vector
  straddles two segments.

Readings of points the paper leaves open (equality with the threshold counts as
large; a large parameter does not flush the open batch; members of a batch
start on granule boundaries) are the ones listed in the design notes.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence

F32, BF16 = 0, 1
SPLIT_NONE, SPLIT_FIXED, SPLIT_ADAPTIVE = 0, 1, 2
KIND_BATCH, KIND_CHUNK = 0, 1


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
    if len(elems) == 0:
        raise ValueError("no tensors")
    if any(e <= 0 for e in elems):
        raise ValueError("zero-element tensor")


def build_plan(cfg: Config, elems: Sequence[int]) -> Plan:
    """Walk the tensors in update order and emit transfer units in queue order."""
    validate(cfg, elems)
    s, g, t_bytes = cfg.elem_size, cfg.granule, cfg.batch_threshold_bytes
    units: List[Unit] = []
    entries: List[Entry] = []
    fused_elems = 0
    open_batch: List[Entry] = []     # members of the active batch (unit id filled at close)
    open_elems = 0

    def emit(kind: int, members: List[Entry], n: int) -> None:
        nonlocal fused_elems
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

    for t, n in enumerate(elems):
        if t_bytes == 0 or n * s >= t_bytes:
            off = 0
            for piece in chunk_sizes(cfg, n):
                emit(KIND_CHUNK, [Entry(t, off, -1, 0, piece)], piece)
                off += piece
            continue
        at = _align_up(open_elems, g)
        open_batch.append(Entry(t, 0, -1, at, n))
        open_elems = at + n
        if _align_up(open_elems, g) * s >= t_bytes:
            emit(KIND_BATCH, open_batch, _align_up(open_elems, g))
            open_batch, open_elems = [], 0
    if open_batch:
        emit(KIND_BATCH, open_batch, _align_up(open_elems, g))
    return Plan(cfg, len(elems), units, entries, fused_elems)
