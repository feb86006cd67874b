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
    def __init__(self, P: int, b: int, d_in: int, device="cuda", slots: int = 2, rounds_per_copy: int = 1):
        """rounds_per_copy = g > 1: a buffer holds the minibatches of g consecutive rounds (X[g][P][b][d_in],
        y[g][P][b]) and one copy, one wait and one release serve g rounds.  Ordering two streams costs the reading
        stream about 13 us per wait/release pair on MI355X whatever the copy's size, which a short round notices."""
        if slots < 2:
            raise ValueError("need at least two buffers to overlap a copy with a round")
        if rounds_per_copy < 1:
            raise ValueError("rounds_per_copy must be >= 1")
        self.slots = slots
        # samples and labels of a buffer sit back to back in one allocation, so that a host batch laid out the same
        # way (host_batch()) arrives in ONE copy: a second, small copy per round goes through a copy kernel on the
        # copy stream's queue, and the round's own launches then share the chip with another queue every round
        g = rounds_per_copy
        self._xs = (P, b, d_in) if g == 1 else (g, P, b, d_in)
        self._ys = (P, b) if g == 1 else (g, P, b)
        self._x_bytes = g * P * b * d_in * 4
        self._y_bytes = g * P * b * 4
        self._blob = [torch.empty(self._x_bytes + self._y_bytes, dtype=torch.uint8, device=device) for _ in range(slots)]
        self.X = [blob[:self._x_bytes].view(torch.float32).view(self._xs) for blob in self._blob]
        self.y = [blob[self._x_bytes:].view(torch.int32).view(self._ys) for blob in self._blob]
        self.copy_stream = torch.cuda.Stream(device=device)          # default priority
        self._filled = [torch.cuda.Event() for _ in range(slots)]
        self._free = [torch.cuda.Event() for _ in range(slots)]
        self._used = [False] * slots

    def host_batch(self) -> Tuple[torch.Tensor, torch.Tensor]:
        """Pinned host tensors (X fp32, y int32, shaped like the device buffers) laid out back to back like them:
        fill them and pass them to submit(), which then needs a single copy."""
        blob = torch.empty(self._x_bytes + self._y_bytes, dtype=torch.uint8).pin_memory()
        return blob[:self._x_bytes].view(torch.float32).view(self._xs), blob[self._x_bytes:].view(torch.int32).view(self._ys)

    def submit(self, slot: int, host_X: torch.Tensor, host_y: torch.Tensor) -> None:
        """Start copying the minibatches of one round (of rounds_per_copy rounds) into buffer `slot` (returns at once)."""
        if not (host_X.is_pinned() and host_y.is_pinned()):
            raise ValueError("host batches must be pinned (pin_memory=True) for an asynchronous copy")
        if host_X.shape != self.X[slot].shape or host_y.shape != self.y[slot].shape:
            raise ValueError("host batch shape does not match the device buffers")
        with torch.cuda.stream(self.copy_stream):
            if self._used[slot]:
                self.copy_stream.wait_event(self._free[slot])        # the round that read it has finished
            if host_y.data_ptr() == host_X.data_ptr() + self._x_bytes and host_X.is_contiguous() and host_y.is_contiguous():
                whole = torch.as_strided(host_X.view(torch.uint8).view(-1), (self._blob[slot].numel(),), (1,))
                self._blob[slot].copy_(whole, non_blocking=True)         # a batch from host_batch(): one copy
            else:
                self.X[slot].copy_(host_X, non_blocking=True)
                self.y[slot].copy_(host_y, non_blocking=True)
            self._filled[slot].record(self.copy_stream)

    def acquire(self, slot: int, stream: Optional[torch.cuda.Stream] = None) -> Tuple[torch.Tensor, torch.Tensor]:
        """Device tensors of buffer `slot`; work queued on `stream` after this call sees the copied data."""
        (stream or torch.cuda.current_stream()).wait_event(self._filled[slot])
        return self.X[slot], self.y[slot]

    def release(self, slot: int, stream: Optional[torch.cuda.Stream] = None) -> None:
        """Call after the round (the last of the rounds) that reads buffer `slot` has been queued on `stream`."""
        self._free[slot].record(stream or torch.cuda.current_stream())
        self._used[slot] = True
