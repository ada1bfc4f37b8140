"""Device buffers placed over HBM.

On MI355X a streaming step that touches many arrays at once sustains about 0.65 of peak HBM
bandwidth when those arrays all lie inside one third (96 GiB) of the device's physical memory -
where a fresh process's consecutive allocations land - and 0.78-0.79 when half of them lie in one
third and half in another (measured; which arrays does not matter as long as every group that is
streamed together is split).  Nobody outside the driver sees physical addresses.  A large
allocation is pieced together from whatever is free, emptiest third first: made first, its bytes
[0, 96 GiB) lie in one third and [96, 192 GiB) in the next; made after 100 GiB of other
allocations, the second boundary was seen at 160 GiB and, for a smaller arena, at 128 GiB.

What can be done is to MEASURE.  A mixing pass over sixteen 64 MiB sources and outputs runs at
0.78-0.80 of peak when half of its buffers sit in one third and half in another, and at 0.61-0.73
when all sit in the same third, repeatable to 1 %: timing that pass over pairs of 1 GiB chunks of
an arena tells which chunks share a third.

``SpreadArena`` makes ONE allocation (by default: free memory minus ``keep_free_bytes``) and, before
anything is stored in it (``calibrate=True``, about half a second): finds the stretches of it that
lie in different thirds; deals the buffers over the two of them with the most room
(``dadam_deal_offsets``: alternately, buffers 0, 2, 4, ... in one and 1, 3, 5, ... in the other, so
that any run of consecutive buffers - all sources, all outputs, one kind of state - is split
evenly; or every 3rd ... 8th buffer in a second stretch that is too small for half of them); and
confirms the choice with one more pass across the two regions and one inside each.  ``policy``,
``advice`` and ``describe()`` say what was done and what the probe measured.  If the probe finds
nothing usable, or with ``calibrate=False``, the library's rule for an allocation that covers the
device applies (``dadam_place_offsets``), which falls back to equal distances when the arena does
not cover the device.  The space between the buffers stays untouched
and can be handed out as views for anything else.
Memory management only - nothing of the method is computed here.
"""

from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

import torch

from . import binding as B

UNIT = 2 << 20
GIB = 1 << 30
HBM_PEAK = 8.0e12

# the timing probe: sixteen sources and sixteen outputs of 64 MiB, half of each in one 1 GiB chunk
PROBE_ROWS = 16
PROBE_ELEMS = 16 << 20
PROBE_CHUNK = 2 * (PROBE_ROWS // 2) * PROBE_ELEMS * 4          # bytes of one chunk: 8 sources + 8 outputs
PROBE_STEP = 4 * GIB


def _round_up(n: int, unit: int = UNIT) -> int:
    return -(-int(n) // unit) * unit


class ThirdsProbe:
    """Times the library's mixing pass over two 1 GiB chunks of a device allocation."""

    def __init__(self, storage: torch.Tensor, base_offset: int):
        from . import workloads as WL
        self.storage, self.base = storage, base_offset
        self.launches = 0
        dev = storage.device
        self.state = [torch.empty(PROBE_ELEMS, dtype=torch.float32, device=dev) for _ in range(2 * PROBE_ROWS)]
        self.h = B.dadam_init(PROBE_ROWS, PROBE_ROWS, PROBE_ELEMS, [0], [PROBE_ELEMS], device=dev.index or 0)
        B.dadam_set_topology(self.h, 0, *WL.ring(PROBE_ROWS))

    def _view(self, off: int) -> torch.Tensor:
        nb = PROBE_ELEMS * 4
        return self.storage[self.base + off:self.base + off + nb].view(torch.float32)

    def rate(self, off_a: int, off_b: int, reps: int = 6) -> float:
        """Fraction of the HBM peak the pass sustains with half of its buffers at off_a and half at off_b."""
        nb, half = PROBE_ELEMS * 4, PROBE_ROWS // 2
        return self.rate_of_layout([off_a + k * nb for k in range(half)] + [off_b + k * nb for k in range(half)] +
                                   [off_a + (half + k) * nb for k in range(half)] + [off_b + (half + k) * nb for k in range(half)], reps)

    def rate_of_layout(self, offsets: Sequence[int], reps: int = 6) -> float:
        """The same for any placement of the pass's buffers: offsets of its 16 sources, then of its 16 outputs."""
        xs = [self._view(o) for o in offsets[:PROBE_ROWS]]
        xd = [self._view(o) for o in offsets[PROBE_ROWS:]]
        nb = PROBE_ELEMS * 4
        B.dadam_bind(self.h, xs, xd, self.state[:PROBE_ROWS], self.state[PROBE_ROWS:], None)
        st = B.current_stream()
        for _ in range(2):
            B.dadam_mix(self.h, 0, 0, st)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            B.dadam_mix(self.h, 0, 0, st)
        e1.record()
        torch.cuda.synchronize()
        self.launches += 2 + reps
        seconds = e0.elapsed_time(e1) / reps / 1e3
        return 2 * PROBE_ROWS * nb / seconds / HBM_PEAK

    def close(self):
        torch.cuda.synchronize()
        B.dadam_destroy(self.h)
        self.h, self.state = None, None


def stretches_in_different_thirds(span_bytes: int, rate, attempts: int = 2) -> List[Tuple[int, int, int]]:
    """Stretches (third id, lo, hi) of an arena of span_bytes, found by timing: ``rate(off_a, off_b)`` is the
    fraction of peak a streaming pass sustains over the chunks at those offsets.  Chunks every PROBE_STEP bytes
    are compared with a reference chunk; those that run fast with it (>= 0.95 of the fastest pairing, which
    itself must reach 0.75 of peak; measured: 0.78-0.80 across thirds, 0.61-0.73 inside one) lie in another
    third.  A second reference taken from those separates the other two thirds.  The same third may come
    back later in the arena (the driver pieces a large allocation together from what is free), but an answer
    with more than six stretches is noise: the timing is repeated, and an empty list returned if that does
    not help.  Pure bookkeeping around the timings (tested on the CPU with a model of the memory)."""
    offs = list(range(0, span_bytes - PROBE_CHUNK + 1, PROBE_STEP))
    if len(offs) < 3:
        return []

    def same_third_as(ref_index: int) -> List[bool]:
        rates = [None if k == ref_index else rate(offs[ref_index], offs[k]) for k in range(len(offs))]
        best = max(r for r in rates if r is not None)
        if best < 0.75:                 # no pairing reaches the two-thirds level: everything shares the reference's third
            return [True] * len(offs)
        return [r is None or r < 0.95 * best for r in rates]

    for _attempt in range(attempts):
        third = [-1] * len(offs)
        for k, s in enumerate(same_third_as(0)):
            if s:
                third[k] = 0
        rest = [k for k in range(len(offs)) if third[k] < 0]
        if rest:
            with_b = same_third_as(rest[min(2, len(rest) - 1)])     # not the first: that chunk may lie across a boundary
            for k in rest:
                third[k] = 1 if with_b[k] else 2
        for k in range(1, len(offs) - 1):      # one chunk at odds with two neighbours that agree: a timing outlier
            if third[k - 1] == third[k + 1] != third[k]:
                third[k] = third[k - 1]
        runs, k = [], 0
        while k < len(offs):
            j = k
            while j + 1 < len(offs) and third[j + 1] == third[k]:
                j += 1
            # a run covers its first chunk's start to its last chunk's end: every byte in between lies in chunks
            # that were classified alike on both sides
            runs.append((third[k], offs[k], offs[j] + PROBE_CHUNK))
            k = j + 1
        if len(runs) <= 6:
            return runs
    return []


def region_candidates(runs: Sequence[Tuple[int, int, int]], nbytes: Sequence[int]):
    """Ways to deal the buffers over two stretches of different thirds: a list of ((lo0, hi0), (lo1, hi1), every)
    for dadam_deal_offsets, at most one per `every` (2: alternately; 3, 4, 6, 8: every 3rd ... 8th buffer goes
    to the smaller stretch), each over the two stretches with the most room that hold their shares.  A region
    is cut down to max(64 GiB, 1.2 x what it holds), at the end of its stretch nearest the other one."""
    out = []
    for every in (2, 3, 4, 6, 8):
        minor = sum(_round_up(n) for k, n in enumerate(nbytes) if k % every == every - 1)
        major = sum(_round_up(n) for n in nbytes) - minor
        best = None
        for a in runs:                  # a holds the larger share
            for b in runs:
                if a[0] == b[0] or a[2] - a[1] < major or b[2] - b[1] < minor:
                    continue
                size = min(a[2] - a[1], 96 * GIB) + min(b[2] - b[1], 96 * GIB)
                if best is None or size > best[0]:
                    best = (size, a, b)
        if best is None:
            continue
        _, a, b = best
        wa = min(a[2] - a[1], max(64 * GIB, _round_up(major * 6 // 5)))
        wb = min(b[2] - b[1], max(64 * GIB, _round_up(minor * 6 // 5)))
        if a[1] < b[1]:
            out.append(((a[2] - wa, a[2]), (b[1], b[1] + wb), every))
        else:
            out.append(((a[1], a[1] + wa), (b[2] - wb, b[2]), every))
    return out


def two_regions_from_stretches(runs: Sequence[Tuple[int, int, int]], nbytes: Sequence[int]):
    """The first of region_candidates (the most even deal that fits), or None."""
    found = region_candidates(runs, nbytes)
    return found[0] if found else None


class SpreadArena:
    def __init__(self, nbytes: Sequence[int], device, span_bytes: Optional[int] = None, keep_free_bytes: int = 12 << 30,
                 two_regions: bool = True, calibrate: bool = True, offsets: Optional[Sequence[int]] = None):
        """nbytes: sizes of the buffers, in the order they are laid out.  span_bytes: size of the
        arena; default is the free device memory minus ``keep_free_bytes``, never less than the packed
        size.  two_regions=False: equal distances over the whole arena.  calibrate=False: no timing,
        the library's rule for a whole-device arena.  offsets: an explicit placement (one offset per
        buffer, multiples of 2 MiB)."""
        self.device = torch.device(device)
        self.nbytes = [int(n) for n in nbytes]
        packed = sum(_round_up(n) for n in self.nbytes)
        free, total = torch.cuda.mem_get_info(self.device)
        self.in_use_before = total - free
        if span_bytes is None:
            span_bytes = max(packed, free - keep_free_bytes)
        span_bytes = max(int(span_bytes), packed)
        while True:
            try:
                self.storage = torch.empty(span_bytes + UNIT, dtype=torch.uint8, device=self.device)
                break
            except torch.OutOfMemoryError:
                # free memory is not always one contiguous range: settle for a smaller span
                if span_bytes == packed:
                    raise
                span_bytes = max(packed, span_bytes - (8 << 30))
        self.base_offset = (-self.storage.data_ptr()) % UNIT            # start on a 2 MiB boundary
        self.span_bytes = span_bytes
        self.advice = 0
        self.probe_launches = 0                   # mixing passes launched by the timing probe (profiles set them apart)
        self.probe_note = ""                      # what the probe could not tell, if anything
        self.probe_rates = ""                     # what its pass sustained under each candidate placement
        self.stretches: List[Tuple[int, int, int]] = []
        placed = None
        if offsets is not None:
            self.policy, placed = "given offsets", [int(o) for o in offsets]
            self.regions_used = [(min(placed), max(o + n for o, n in zip(placed, self.nbytes)))]
        elif two_regions and calibrate and len(self.nbytes) >= 2 and span_bytes >= 2 * PROBE_STEP + PROBE_CHUNK:
            try:
                probe = ThirdsProbe(self.storage, self.base_offset)
            except torch.OutOfMemoryError:
                probe = None                      # no room for the probe's 2 GiB of state: fall through to the rule
            if probe is not None:
                try:
                    placed = self._place_by_timing(probe, span_bytes, total)
                finally:
                    self.probe_launches = probe.launches
                    probe.close()
        if placed is None and two_regions:
            placed, self.regions_used, self.advice = B.dadam_place_offsets(self.nbytes, span_bytes, total)
            self.policy = {B.DADAM_PLACE_TWO_REGIONS: "two regions across the first boundary (whole-device rule)",
                           B.DADAM_PLACE_ARENA_ELSEWHERE: "equal distances (no two thirds found, arena does not cover the device)",
                           B.DADAM_PLACE_TOO_LARGE: "equal distances (buffers too large for two regions)"}.get(self.advice, "equal distances")
        elif placed is None:
            self.policy, placed = "equal distances", B.dadam_spread_offsets(self.nbytes, span_bytes)
            self.regions_used = [(0, span_bytes)]
        self.offsets = placed
        taken = sorted(zip(self.offsets, self.nbytes))
        for k, (o, n) in enumerate(taken):
            assert o % UNIT == 0 and self.base_offset + o + n <= self.storage.numel(), (k, o, n)
            if k:
                assert o >= taken[k - 1][0] + taken[k - 1][1], "buffers overlap"

    def _place_by_timing(self, probe: "ThirdsProbe", span_bytes: int, total: int):
        """Finds the stretches of the arena that lie in different thirds and deals the buffers over the two
        with the most room, as evenly as they allow; the choice is kept only if one more pass across the two
        regions runs at the two-thirds level and a pass inside each does not.  Returns the offsets, or None
        (then ``probe_note`` says why and the caller falls back to the library's rule).

        (Timing the probe's own pass with its buffers laid out like each candidate placement - dealt, by the
        rule, at equal distances - and taking the fastest was tried and does not work: 32 buffers of one pass
        are no model of 100 arrays streamed at once; it preferred equal distances at 0.80 on the probe where
        the step then ran at 0.60-0.66.  Against equal distances an uneven deal won every matched comparison:
        0.75 / 0.73 / 0.70 against 0.60 / 0.64 / 0.62 with 160 / 200 / 180 GiB allocated first.)"""
        self.stretches = stretches_in_different_thirds(span_bytes // UNIT * UNIT, probe.rate)
        if not self.stretches:
            self.probe_note = "timing probe: no consistent picture of the thirds"
            return None
        found = two_regions_from_stretches(self.stretches, self.nbytes)
        if found is None:
            self.probe_note = "timing probe: no two stretches in different thirds hold the buffers"
            return None
        (lo0, hi0), (lo1, hi1), every = found
        ends = [(lo, max(lo, (hi - PROBE_CHUNK) // UNIT * UNIT)) for lo, hi in ((lo0, hi0), (lo1, hi1))]
        across = probe.rate(ends[0][0] if lo0 < lo1 else ends[0][1], ends[1][1] if lo0 < lo1 else ends[1][0])
        inside = [probe.rate(lo, hi) for lo, hi in ends if hi - lo >= PROBE_CHUNK]
        self.probe_rates = f"probe pass: {across:.3f} of peak across the regions, " + ", ".join(f"{r:.3f}" for r in inside) + " inside"
        if across < 0.75 or any(r >= 0.95 * across for r in inside):
            self.probe_note = "timing probe: regions not confirmed"
            return None
        self.regions_used, self.advice = [found[0], found[1]], B.DADAM_PLACE_TWO_REGIONS
        self.policy = "two regions found by timing" + ("" if every == 2 else f" (every {every}th buffer in the second)")
        return B.dadam_deal_offsets(self.nbytes, found[0], found[1], every)

    def describe(self) -> str:
        gib = lambda v: f"{v / GIB:.1f}"
        regs = " + ".join(f"[{gib(lo)}, {gib(hi)})" for lo, hi in self.regions_used)
        found = ""
        if self.stretches:
            found = "; thirds seen at " + ", ".join(f"[{gib(lo)}, {gib(hi)})" for _t, lo, hi in self.stretches)
        if self.probe_note:
            found += f"; {self.probe_note}"
        if self.probe_rates:
            found += f"; {self.probe_rates}"
        return (f"{self.policy}: {regs} GiB of a {gib(self.span_bytes)} GiB allocation made with "
                f"{gib(self.in_use_before)} GiB in use{found}")

    def view(self, k: int, dtype: torch.dtype) -> torch.Tensor:
        o = self.base_offset + self.offsets[k]
        t = self.storage[o:o + self.nbytes[k]].view(dtype)
        assert t.numel() * t.element_size() == self.nbytes[k]
        return t

    def views(self, dtypes: Sequence[torch.dtype]) -> List[torch.Tensor]:
        return [self.view(k, dt) for k, dt in enumerate(dtypes)]
