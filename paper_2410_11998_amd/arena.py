"""Device buffers placed over HBM.

On MI355X a streaming step that touches many arrays at once sustains about 0.65 of peak HBM
bandwidth when those arrays all lie inside one third (96 GiB) of the device's physical memory -
where a fresh process's consecutive allocations land - and 0.77-0.79 when half of them lie in one
third and half in another (measured; which arrays does not matter as long as every group that is
streamed together is split).  ``SpreadArena`` makes one allocation that covers nearly the whole
device, so that offsets inside it are physical positions up to what was allocated before it, and
carves the buffers out of two regions, one below and one above the boundary between the first two
thirds, dealing them alternately: buffers 0, 2, 4, ... below, 1, 3, 5, ... above, spread evenly
inside each region (``dadam_spread_offsets``).  Any run of consecutive buffers - all sources, all
outputs, one kind of state - is then split evenly.  The space between buffers stays untouched and can
be used for anything else.  When the arena cannot cover the device, or the buffers do not fit the
two regions, they are spread evenly over the whole arena instead.
Memory management only - nothing of the method is computed here.
"""

from __future__ import annotations

from typing import List, Optional, Sequence

import torch

from . import binding as B


class SpreadArena:
    def __init__(self, nbytes: Sequence[int], device, span_bytes: Optional[int] = None, keep_free_bytes: int = 12 << 30,
                 window: Optional[Sequence[int]] = None, regions: Optional[Sequence[Sequence[int]]] = None,
                 default_regions: bool = True, offsets: Optional[Sequence[int]] = None):
        """nbytes: sizes of the buffers, in the order they are laid out.  span_bytes: size of the
        arena; default is the free device memory minus ``keep_free_bytes``, but never less than the
        packed size.  window = (lo, hi) in bytes: spread the buffers over that part of the arena only.
        regions = [(lo, hi), ...]: deal the buffers round-robin over these parts.  With neither, the two
        regions described above are used when they apply (default_regions=False: never).
        offsets: an explicit placement (one offset per buffer, multiples of 2 MiB, inside the arena)."""
        self.device = torch.device(device)
        unit = 2 << 20
        packed = sum(-(-int(n) // unit) * unit for n in nbytes)
        win_lo = 0
        if window is not None:
            win_lo, win_hi = int(window[0]), int(window[1])
            assert win_lo % unit == 0 and win_hi - win_lo >= packed, "window too small or not 2 MiB aligned"
        if span_bytes is None:
            free, _total = torch.cuda.mem_get_info(self.device)
            span_bytes = max(packed, free - keep_free_bytes)
        span_bytes = max(int(span_bytes), packed)
        while True:
            try:
                self.storage = torch.empty(span_bytes + unit, dtype=torch.uint8, device=self.device)
                break
            except torch.OutOfMemoryError:
                # free memory is not always one contiguous range: settle for a smaller span
                if span_bytes == packed or window is not None:
                    raise
                span_bytes = max(packed, span_bytes - (8 << 30))
        self.base_offset = (-self.storage.data_ptr()) % unit            # start on a 2 MiB boundary
        self.span_bytes = span_bytes
        self.policy = "regions" if regions is not None else "window" if window is not None else "whole arena"
        placed = None
        if offsets is not None:
            self.policy, placed = "given offsets", [int(o) for o in offsets]
            regions = [(min(placed), max(o + int(n) for o, n in zip(placed, nbytes)))]
        elif regions is None and window is None and default_regions:
            placed, used = B.dadam_place_offsets(nbytes, span_bytes, torch.cuda.mem_get_info(self.device)[1])
            if len(used) == 2:
                self.policy, regions = "two thirds", used
            else:
                placed = None
        self.regions_used = ([(int(lo), int(hi)) for lo, hi in regions] if regions is not None
                             else [(win_lo, win_hi)] if window is not None else [(0, span_bytes)])
        if regions is not None:
            for lo, hi in regions:
                assert int(lo) % unit == 0 and int(lo) < int(hi) <= span_bytes, "region beyond the arena or not 2 MiB aligned"
            self.offsets = placed if placed is not None else deal_offsets(nbytes, regions)
        elif window is not None:
            assert win_hi <= span_bytes, "window beyond the arena"
            self.offsets = [win_lo + o for o in B.dadam_spread_offsets(nbytes, win_hi - win_lo)]
        else:
            self.offsets = B.dadam_spread_offsets(nbytes, span_bytes)
        self.nbytes = [int(n) for n in nbytes]
        taken = sorted(zip(self.offsets, self.nbytes))
        for k, (o, n) in enumerate(taken):
            assert o % unit == 0 and self.base_offset + o + n <= self.storage.numel(), (k, o, n)
            if k:
                assert o >= taken[k - 1][0] + taken[k - 1][1], "buffers overlap"

    @staticmethod
    def nbytes_rounded(nbytes, unit):
        return [-(-int(n) // unit) * unit for n in nbytes]

    def view(self, k: int, dtype: torch.dtype) -> torch.Tensor:
        o = self.base_offset + self.offsets[k]
        t = self.storage[o:o + self.nbytes[k]].view(dtype)
        assert t.numel() * t.element_size() == self.nbytes[k]
        return t

    def views(self, dtypes: Sequence[torch.dtype]) -> List[torch.Tensor]:
        return [self.view(k, dt) for k, dt in enumerate(dtypes)]


GIB = 1 << 30


def deal_offsets(nbytes: Sequence[int], regions: Sequence[Sequence[int]]) -> List[int]:
    """Offsets of the buffers when they are dealt round-robin over the regions (lo, hi) and spread evenly
    inside each: buffer k goes to region k mod len(regions)."""
    offsets = [0] * len(nbytes)
    for r, (lo, hi) in enumerate(regions):
        idx = list(range(r, len(nbytes), len(regions)))
        if idx:
            for k, o in zip(idx, B.dadam_spread_offsets([nbytes[k] for k in idx], int(hi) - int(lo))):
                offsets[k] = int(lo) + o
    return offsets


def two_thirds_regions(rounded_nbytes: Sequence[int], span_bytes: int, total: int):
    """The two regions either side of the boundary between the first and the second third of the
    device memory (total bytes) that the library's placement advice (dadam_place_offsets) uses, or
    None when it falls back to the whole arena: the arena does not cover the device closely enough
    for its offsets to be physical positions, or the buffers do not fit."""
    _offsets, regions = B.dadam_place_offsets(rounded_nbytes, span_bytes, total)
    return regions if len(regions) == 2 else None
