"""One device allocation for all large buffers, and a measured choice of where the outer state goes.

Why.  On an MI355X the streaming kernels' speed depends on where their buffers lie in physical
memory, at a scale of tens of GiB (the outer step alone: 27.0 to 29.9 ms over placements that differ
only by a shift).  With one allocation per buffer the placement differs from process to process;
buffers carved from a single allocation made first thing in a process land in the same place every
time, and the same layout then reproduces to 0.1 %.  The arena is that single allocation, and
`place_outer_state` picks, by timing the outer step on a few candidate shifts before any data is
written, the shift at which theta_outer / theta_local / momentum are carved.

This is memory plumbing around the library: nothing here touches the values.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple

import torch

from . import binding as B

GiB = 1 << 30
ALIGN = 4096


class Arena:
    """One uint8 allocation; carve() hands out aligned, non-overlapping views of it."""

    def __init__(self, device, nbytes: Optional[int] = None, leave_free: int = 6 * GiB):
        free, _ = torch.cuda.mem_get_info(device)
        if nbytes is None:
            nbytes = (free - leave_free) // GiB * GiB
        if nbytes <= 0:
            raise RuntimeError("no device memory left for an arena")
        self.buf = torch.empty(nbytes, dtype=torch.uint8, device=device)
        self.nbytes = nbytes
        self.pos = 0

    def carve(self, numel: int, dtype, at: Optional[int] = None) -> torch.Tensor:
        """A [numel] view of the given dtype, at the next free aligned offset (or at `at`, which
        moves the arena's position there)."""
        if at is not None:
            self.pos = at
        start = (self.pos + ALIGN - 1) // ALIGN * ALIGN
        nbytes = numel * torch.empty((), dtype=dtype).element_size()
        if start + nbytes > self.nbytes:
            raise RuntimeError(f"arena exhausted: need {start + nbytes} of {self.nbytes} bytes")
        self.pos = start + nbytes
        return self.buf[start:start + nbytes].view(dtype)


def place_outer_state(arena: Arena, N: int, seg_offsets: Sequence[int], shifts_gib: Sequence[int],
                      tail_bytes: int, log=None) -> int:
    """Times outer_nesterov_step (coded form) with theta at shift s, theta_local at s + 4N and
    momentum at s + 8N bytes of the arena, the byte arrays behind them, for every candidate shift, and
    returns the fastest shift in bytes.  The memory is used as it is (timing does not depend on the
    values); the caller fills its buffers afterwards.  tail_bytes = what must still fit behind the
    three fp32 arrays."""
    dev = arena.buf.device
    T = len(seg_offsets) - 1
    lut = torch.zeros((T, 256), dtype=torch.float32, device=dev)
    ws = B.new_workspace(T, dev)
    best: Tuple[float, int] = (float("inf"), 0)
    for s_gib in shifts_gib:
        shift = s_gib * GiB
        if shift + 12 * N + tail_bytes + 8 * ALIGN > arena.nbytes:
            continue
        theta = arena.carve(N, torch.float32, at=shift)
        arena.carve(N, torch.float32)                       # theta_local's place
        mom = arena.carve(N, torch.float32)
        arena.carve(tail_bytes - N, torch.uint8)            # the other byte arrays' place
        codes = arena.carve(N, torch.uint8)                 # the reduced codes come last
        times = []
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            B.outer_step(theta, mom, 0.0, 0.0, delta_codes=codes, delta_lut=lut, seg_offsets=seg_offsets,
                         workspace=ws)
            e1.record()
            torch.cuda.synchronize(dev)
            times.append(e0.elapsed_time(e1))
        ms = min(times[1:])
        if log:
            log(f"[arena] outer step with the state at +{s_gib} GiB: {ms:.2f} ms")
        if ms < best[0]:
            best = (ms, shift)
    arena.pos = 0
    return best[1]
