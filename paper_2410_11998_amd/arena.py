"""Device buffers spread over HBM.

On MI355X a streaming step that touches ~100 arrays at once sustains about 0.65 of peak HBM
bandwidth when those arrays all lie inside one 96 GiB third of the device's physical memory (where
a fresh process's consecutive allocations land) and 0.75-0.77 when they straddle the boundaries
between thirds (measured).  ``SpreadArena`` makes one allocation and carves the buffers out of it at the
offsets ``dadam_spread_offsets`` computes; the space between buffers stays untouched and can be used
for anything else.  Memory management only - nothing of the method is computed here.
"""

from __future__ import annotations

from typing import List, Optional, Sequence

import torch

from . import binding as B


class SpreadArena:
    def __init__(self, nbytes: Sequence[int], device, span_bytes: Optional[int] = None, keep_free_bytes: int = 12 << 30):
        """nbytes: sizes of the buffers, in the order they are laid out.  span_bytes: size of the
        arena; default is the free device memory minus ``keep_free_bytes``, but never less than the
        packed size."""
        self.device = torch.device(device)
        unit = 2 << 20
        packed = sum(-(-int(n) // unit) * unit for n in nbytes)
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
                if span_bytes == packed:
                    raise
                span_bytes = max(packed, span_bytes - (8 << 30))
        self.base_offset = (-self.storage.data_ptr()) % unit            # start on a 2 MiB boundary
        self.span_bytes = span_bytes
        self.offsets = B.dadam_spread_offsets(nbytes, span_bytes)
        self.nbytes = [int(n) for n in nbytes]
        for k, (o, n) in enumerate(zip(self.offsets, self.nbytes)):
            assert o % unit == 0 and self.base_offset + o + n <= self.storage.numel(), (k, o, n)
            if k:
                assert o >= self.offsets[k - 1] + self.nbytes[k - 1]

    def view(self, k: int, dtype: torch.dtype) -> torch.Tensor:
        o = self.base_offset + self.offsets[k]
        t = self.storage[o:o + self.nbytes[k]].view(dtype)
        assert t.numel() * t.element_size() == self.nbytes[k]
        return t

    def views(self, dtypes: Sequence[torch.dtype]) -> List[torch.Tensor]:
        return [self.view(k, dt) for k, dt in enumerate(dtypes)]
