"""Device buffers placed over HBM.

On MI355X a streaming step that touches many arrays at once sustains about 0.65 of peak HBM
bandwidth when those arrays all lie inside one third (96 GiB) of the device's physical memory -
where a fresh process's consecutive allocations land - and 0.78-0.79 when half of them lie in one
third and half in another (measured; which arrays does not matter as long as every group that is
streamed together is split).  Nobody outside the driver sees physical addresses, and where the
driver puts one allocation relative to another is not predictable; what holds is that ONE
allocation of nearly the whole device covers the physical memory in order.  ``SpreadArena`` makes
that allocation (free memory minus ``keep_free_bytes``) and carves the buffers out of two regions
either side of the boundary between the first two thirds by the library's advice
(``dadam_place_offsets``): buffers 0, 2, 4, ... below, 1, 3, 5, ... above, so that any run of
consecutive buffers - all sources, all outputs, one kind of state - is split evenly.  The space
between the buffers stays untouched and can be handed out as views for anything else.

When the arena cannot cover the device (memory already in use, or a span given by the caller) the
buffers are spread at equal distances over whatever arena there is, and ``advice`` says so.
Memory management only - nothing of the method is computed here.
"""

from __future__ import annotations

from typing import List, Optional, Sequence

import torch

from . import binding as B

UNIT = 2 << 20
GIB = 1 << 30


def _round_up(n: int, unit: int = UNIT) -> int:
    return -(-int(n) // unit) * unit


class SpreadArena:
    def __init__(self, nbytes: Sequence[int], device, span_bytes: Optional[int] = None, keep_free_bytes: int = 12 << 30,
                 two_regions: bool = True, offsets: Optional[Sequence[int]] = None):
        """nbytes: sizes of the buffers, in the order they are laid out.  span_bytes: size of the
        arena; default is the free device memory minus ``keep_free_bytes``, never less than the packed
        size.  two_regions=False: equal distances over the whole arena.  offsets: an explicit
        placement (one offset per buffer, multiples of 2 MiB)."""
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
        if offsets is not None:
            self.policy, self.offsets = "given offsets", [int(o) for o in offsets]
            self.regions_used = [(min(self.offsets), max(o + n for o, n in zip(self.offsets, self.nbytes)))]
        elif two_regions:
            self.offsets, self.regions_used, self.advice = B.dadam_place_offsets(self.nbytes, span_bytes, total)
            self.policy = {B.DADAM_PLACE_TWO_REGIONS: "two regions across the first boundary",
                           B.DADAM_PLACE_ARENA_ELSEWHERE: "equal distances (the arena does not cover the device)",
                           B.DADAM_PLACE_TOO_LARGE: "equal distances (buffers too large for two regions)"}.get(self.advice, "equal distances")
        else:
            self.policy, self.offsets = "equal distances", B.dadam_spread_offsets(self.nbytes, span_bytes)
            self.regions_used = [(0, span_bytes)]
        taken = sorted(zip(self.offsets, self.nbytes))
        for k, (o, n) in enumerate(taken):
            assert o % UNIT == 0 and self.base_offset + o + n <= self.storage.numel(), (k, o, n)
            if k:
                assert o >= taken[k - 1][0] + taken[k - 1][1], "buffers overlap"

    def describe(self) -> str:
        gib = lambda v: f"{v / GIB:.1f}"
        regs = " + ".join(f"[{gib(lo)}, {gib(hi)})" for lo, hi in self.regions_used)
        return (f"{self.policy}: {regs} GiB of a {gib(self.span_bytes)} GiB allocation made with "
                f"{gib(self.in_use_before)} GiB in use")

    def view(self, k: int, dtype: torch.dtype) -> torch.Tensor:
        o = self.base_offset + self.offsets[k]
        t = self.storage[o:o + self.nbytes[k]].view(dtype)
        assert t.numel() * t.element_size() == self.nbytes[k]
        return t

    def views(self, dtypes: Sequence[torch.dtype]) -> List[torch.Tensor]:
        return [self.view(k, dt) for k, dt in enumerate(dtypes)]
