"""Device buffers carved from one large allocation, placed by the library.

On MI355X a streaming step that touches many arrays at once sustains about 0.65 of peak HBM
bandwidth when those arrays all lie inside one third (96 GiB) of the device's physical memory -
where a fresh process's consecutive allocations land - and 0.78-0.79 when half of them lie in one
third and half in another.  The library finds the thirds inside an allocation by timing its own
mixing pass over pairs of chunks and deals the buffers over two stretches that lie in different
thirds (``dadam_place_by_timing`` in include/dadam.h, which also says what is measured and why).

``SpreadArena`` is the PyTorch side of that: it makes ONE allocation (by default: free memory
minus ``keep_free_bytes``), hands it to the library before anything is stored in it, and gives out
views at the offsets that come back.  ``policy``, ``advice``, ``report`` and ``describe()`` say what
the library did.  With ``calibrate=False`` nothing is timed and the library's rule for an allocation
that covers the device applies (``dadam_place_offsets``), which falls back to equal distances when
the arena does not cover the device.  The space between the buffers stays untouched and can be
handed out as views for anything else.  Memory management only - nothing of the method is computed
here.
"""

from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

import torch

from . import binding as B

UNIT = 2 << 20
GIB = 1 << 30

_POLICY_TEXT = {B.DADAM_POLICY_TIMED_REGIONS: "two regions found by timing",
                B.DADAM_POLICY_RULE_REGIONS: "two regions across the first boundary (whole-device rule)",
                B.DADAM_POLICY_EQUAL_DISTANCES: "equal distances"}
_NOTE_TEXT = {B.DADAM_NOTE_NO_PROBE: "no timing probe (arena too small, or no 2 GiB to spare)",
              B.DADAM_NOTE_NO_PICTURE: "timing probe: no consistent picture of the thirds",
              B.DADAM_NOTE_NO_ROOM: "timing probe: no two stretches in different thirds hold the buffers",
              B.DADAM_NOTE_NOT_CONFIRMED: "timing probe: regions not confirmed"}
_ADVICE_TEXT = {B.DADAM_PLACE_ARENA_ELSEWHERE: " (arena does not cover the device)",
                B.DADAM_PLACE_TOO_LARGE: " (buffers too large for two regions)"}


def _round_up(n: int, unit: int = UNIT) -> int:
    return -(-int(n) // unit) * unit


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
        self.report = None                        # dadam_placement of a timed placement
        self.probe_launches = 0                   # mixing passes launched by the timing probe (profiles set them apart)
        self.stretches: List[Tuple[int, int, int]] = []
        if offsets is not None:
            self.policy, placed = "given offsets", [int(o) for o in offsets]
            self.regions_used = [(min(placed), max(o + n for o, n in zip(placed, self.nbytes)))]
        elif two_regions and calibrate:
            torch.cuda.synchronize(self.device)
            placed, rep = B.dadam_place_by_timing(self.storage.data_ptr() + self.base_offset, span_bytes,
                                                  self.device.index or 0, self.nbytes, total)
            self.report, self.advice, self.probe_launches = rep, int(rep.advice), int(rep.probe_launches)
            self.stretches = [(int(s.third), int(s.lo), int(s.hi)) for s in rep.stretches[:rep.n_stretches]]
            self.policy = _POLICY_TEXT[rep.policy] + _ADVICE_TEXT.get(int(rep.advice), "")
            if rep.policy == B.DADAM_POLICY_TIMED_REGIONS and rep.every != 2:
                self.policy += f" (every {rep.every}th buffer in the second)"
            regs = [int(r) for r in rep.regions]
            self.regions_used = [(regs[0], regs[1])] + ([(regs[2], regs[3])] if regs[3] else [])
        elif two_regions:
            placed, self.regions_used, self.advice = B.dadam_place_offsets(self.nbytes, span_bytes, total)
            self.policy = (_POLICY_TEXT[B.DADAM_POLICY_RULE_REGIONS] if self.advice == B.DADAM_PLACE_TWO_REGIONS
                           else "equal distances" + _ADVICE_TEXT.get(self.advice, ""))
        else:
            self.policy, placed = "equal distances", B.dadam_spread_offsets(self.nbytes, span_bytes)
            self.regions_used = [(0, span_bytes)]
        self.offsets = placed
        taken = sorted(zip(self.offsets, self.nbytes))
        for k, (o, n) in enumerate(taken):
            assert o % UNIT == 0 and self.base_offset + o + n <= self.storage.numel(), (k, o, n)
            if k:
                assert o >= taken[k - 1][0] + taken[k - 1][1], "buffers overlap"

    def describe(self) -> str:
        gib = lambda v: f"{v / GIB:.1f}"
        regs = " + ".join(f"[{gib(lo)}, {gib(hi)})" for lo, hi in self.regions_used)
        found = ""
        if self.stretches:
            found = "; thirds seen at " + ", ".join(f"[{gib(lo)}, {gib(hi)})" for _t, lo, hi in self.stretches)
        rep = self.report
        if rep is not None and rep.note:
            found += "; " + _NOTE_TEXT.get(int(rep.note), f"note {rep.note}")
        if rep is not None and rep.rate_across > 0:
            found += (f"; probe pass: {rep.rate_across:.3f} of peak across the regions, "
                      + ", ".join(f"{r:.3f}" for r in rep.rate_inside if r > 0) + " inside")
        return (f"{self.policy}: {regs} GiB of a {gib(self.span_bytes)} GiB allocation made with "
                f"{gib(self.in_use_before)} GiB in use{found}")

    def view(self, k: int, dtype: torch.dtype) -> torch.Tensor:
        o = self.base_offset + self.offsets[k]
        t = self.storage[o:o + self.nbytes[k]].view(dtype)
        assert t.numel() * t.element_size() == self.nbytes[k]
        return t

    def views(self, dtypes: Sequence[torch.dtype]) -> List[torch.Tensor]:
        return [self.view(k, dt) for k, dt in enumerate(dtypes)]
