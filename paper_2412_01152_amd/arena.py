"""One device allocation for all large buffers, and a measured choice of where the outer state goes.

Why.  On an MI355X the streaming kernels' speed depends on where their buffers lie in physical
memory, at a scale of tens of GiB (with 4 GiB arrays the outer step runs at 5.4 TB/s when momentum
lies within 64 GiB of theta_outer and at 6.3 TB/s from 96 GiB on).  With one allocation per buffer the placement differs from process to process;
buffers carved from a single allocation made first thing in a process land in the same place every
time, and the same layout then reproduces to 0.1 %.  The arena is that single allocation, and
`place_outer_state` picks, by timing the two placement-sensitive kernels on a few candidate shifts
before any data is written, the shift at which theta_outer / theta_local / momentum are carved.

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


def role_bases(arena: Arena) -> Dict[str, int]:
    """Where small buffers go so that no kernel writes near what it reads: three groups 100 GiB
    apart, at +4, +104 and +204 GiB (beyond the 96 GiB at which the measured dependence on distance
    levels off), or a third of the arena apart when the arena is smaller than that needs.
      "read"   what stage 1, stage 2 and the outer step only read from: theta (also updated in place),
               theta_local, the peers' codes
      "state"  momentum and the codes stage 1 writes
      "out"    the codes stage 2 writes (and the outer step reads)
    Offsets in bytes into the arena; carve with carve(..., at=base) for the first buffer of a group.
    The rule itself is the library's (diloco_placement); this only names the three results."""
    read, state, out = B.placement(arena.nbytes)
    return {"read": read, "state": state, "out": out}


def place_outer_state(arena: Arena, N: int, seg_offsets: Sequence[int], shifts_gib: Sequence[int],
                      tail_bytes: int, log=None) -> int:
    """Times, for every candidate shift s, the two kernels whose speed depends on where the state lies
    and not on its values - the statistics pass of diloco_pseudograd_quantize (reads theta_outer and
    theta_local) and outer_nesterov_step (updates theta_outer and momentum in place) - with theta at
    s, theta_local at s + 4N and momentum at s + 8N bytes of the arena and the byte arrays behind
    them, and returns the shift with the smallest sum, in bytes.  The memory is used as it is; the
    caller fills its buffers afterwards.  tail_bytes = what must still fit behind the three fp32
    arrays."""
    dev = arena.buf.device
    T = len(seg_offsets) - 1
    lut = torch.zeros((T, 256), dtype=torch.float32, device=dev)
    lut_out = torch.empty((T, 256), dtype=torch.float32, device=dev)
    qp = B.new_qparams(T, dev)
    ws = B.new_workspace(T, dev)
    events = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    for e in events:
        e.record()
    best: Tuple[float, int] = (float("inf"), 0)
    for s_gib in shifts_gib:
        shift = s_gib * GiB
        if shift + 12 * N + tail_bytes + 8 * ALIGN > arena.nbytes:
            continue
        theta = arena.carve(N, torch.float32, at=shift)
        local = arena.carve(N, torch.float32)
        mom = arena.carve(N, torch.float32)
        arena.carve(tail_bytes - 2 * N, torch.uint8)        # the peers' codes
        codes1 = arena.carve(N, torch.uint8)                # stage 1 writes here
        codes2 = arena.carve(N, torch.uint8)                # the outer step reads these
        t_stats, t_outer = [], []
        for _ in range(2):
            B.profile_passes([e.cuda_event for e in events])
            B.pseudograd_quantize(theta, local, seg_offsets, codes_out=codes1, lut_out=lut_out, qparams_out=qp,
                                  workspace=ws)
            torch.cuda.synchronize(dev)
            t_stats.append(events[0].elapsed_time(events[1]))
            B.outer_step(theta, mom, 0.0, 0.0, delta_codes=codes2, delta_lut=lut, seg_offsets=seg_offsets,
                         workspace=ws)
            torch.cuda.synchronize(dev)
            t_outer.append(events[0].elapsed_time(events[1]))
        B.profile_passes(None)
        ms = min(t_stats) + min(t_outer)
        if log:
            log(f"[arena] state at +{s_gib} GiB: statistics pass {min(t_stats):.2f} ms + outer step {min(t_outer):.2f} ms")
        if ms < best[0]:
            best = (ms, shift)
    arena.pos = 0
    return best[1]
