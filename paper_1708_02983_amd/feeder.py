"""Host-to-device minibatch feed that overlaps the copy of the next round's data with the current round.

This is the data path of Algorithm 3 (Sync EASGD2/3, Section 6.1): the host picks b samples per worker, copies
them to the device asynchronously, and Sync EASGD3 overlaps that copy and the forward/backward pass with the
rest of the round.  Here all P workers share one device, so one copy per round brings the minibatches of all
workers; two device buffers alternate, a copy stream of default priority fills one while the round reads the
other, and two events per buffer order the streams (filled -> may be read, read -> may be refilled).

Plumbing only: no arithmetic of the method happens here.  Host tensors must be pinned (allocate them with
``pin_memory=True``), otherwise the copy is not asynchronous.
"""
from __future__ import annotations

from typing import Optional, Tuple

import torch


class BatchFeeder:
    def __init__(self, P: int, b: int, d_in: int, device="cuda", slots: int = 2):
        if slots < 2:
            raise ValueError("need at least two buffers to overlap a copy with a round")
        self.slots = slots
        self.X = [torch.empty(P, b, d_in, dtype=torch.float32, device=device) for _ in range(slots)]
        self.y = [torch.empty(P, b, dtype=torch.int32, device=device) for _ in range(slots)]
        self.copy_stream = torch.cuda.Stream(device=device)          # default priority
        self._filled = [torch.cuda.Event() for _ in range(slots)]
        self._free = [torch.cuda.Event() for _ in range(slots)]
        self._used = [False] * slots

    def submit(self, slot: int, host_X: torch.Tensor, host_y: torch.Tensor) -> None:
        """Start copying one round's minibatches into buffer `slot` (returns at once)."""
        if not (host_X.is_pinned() and host_y.is_pinned()):
            raise ValueError("host batches must be pinned (pin_memory=True) for an asynchronous copy")
        if host_X.shape != self.X[slot].shape or host_y.shape != self.y[slot].shape:
            raise ValueError("host batch shape does not match the device buffers")
        with torch.cuda.stream(self.copy_stream):
            if self._used[slot]:
                self.copy_stream.wait_event(self._free[slot])        # the round that read it has finished
            self.X[slot].copy_(host_X, non_blocking=True)
            self.y[slot].copy_(host_y, non_blocking=True)
            self._filled[slot].record(self.copy_stream)

    def acquire(self, slot: int, stream: Optional[torch.cuda.Stream] = None) -> Tuple[torch.Tensor, torch.Tensor]:
        """Device tensors of buffer `slot`; work queued on `stream` after this call sees the copied data."""
        (stream or torch.cuda.current_stream()).wait_event(self._filled[slot])
        return self.X[slot], self.y[slot]

    def release(self, slot: int, stream: Optional[torch.cuda.Stream] = None) -> None:
        """Call after the round that reads buffer `slot` has been queued on `stream`."""
        self._free[slot].record(stream or torch.cuda.current_stream())
        self._used[slot] = True
