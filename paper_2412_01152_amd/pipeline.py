"""Chunk-pipelined reduce: the transfer of ring chunk c+1 overlaps the reduction of chunk c.

Section 2.2 of the paper hides the quantise / dequantise work of its ring all-reduce behind the
communication by running them asynchronously.  On one GPU the incoming transfer is stood in for by
a host-to-device copy from pinned memory on a copy stream; `int8_reduce_chunk` runs on the compute
stream and waits only for the event that marks its own chunk's arrival.  This module is stream and
event plumbing around the library call; the arithmetic is all in the library.
"""
from __future__ import annotations

from typing import Callable, List, Optional, Sequence

import torch

from . import binding as B


kLine = 128     # elements; the kernels peel a call's head so that element (offset % 128 == 0) starts a memory line


def new_staging(max_chunk: int, W: int, device):
    """Two alternating sets of W code buffers [max_chunk + 127] and W codebooks [1, 256]."""
    codes = [[torch.empty(max_chunk + kLine - 1, dtype=torch.uint8, device=device) for _ in range(W)]
             for _ in range(2)]
    luts = [[torch.empty((1, 256), dtype=torch.float32, device=device) for _ in range(W)] for _ in range(2)]
    return codes, luts


def reduce_chunks_pipelined(chunk_offsets: Sequence[int], W: int, divisor: int,
                            arrive: Callable[[int, List[torch.Tensor], List[torch.Tensor]], None],
                            local_fp32: torch.Tensor, codes_out: torch.Tensor, lut_out: torch.Tensor,
                            copy_stream: Optional[torch.cuda.Stream] = None,
                            overlap: bool = True, staging=None, timing_out: Optional[list] = None):
    """Reduce a flat buffer chunk by chunk.

    chunk_offsets  C+1 ascending element offsets; chunk c is its own quantisation group
    arrive(c, code_bufs, lut_bufs)
                   enqueues, on the *current* stream, whatever brings chunk c's W coded
                   contributions into the given device buffers (code_bufs[p] is [chunk size] bytes,
                   lut_bufs[p] is [1, 256] fp32)
    local_fp32     [N] fp32: the owner's un-quantised data; receives the averaged sum in place
    codes_out      [N] bytes, lut_out [C, 256] fp32: the requantised chunks
    overlap        False runs copy and compute strictly one after the other (for comparison)
    staging        optional result of new_staging(), reused across calls
    timing_out     optional list; receives one (start, end) pair of timing events per reduce call

    Two sets of staging buffers alternate, so chunk c+1 may arrive while chunk c is reduced; the
    buffers of chunk c are reused for chunk c+2 only after its reduction has finished.  A chunk is
    staged at the same offset modulo 128 elements as it has in the flat buffer, so that the code
    streams, the fp32 stream and the output codes all reach a 128-byte line boundary at the same
    element and the library's head peel aligns every stream of the call at once.
    Returns the list of per-chunk qparams tensors.
    """
    dev = local_fp32.device
    C = len(chunk_offsets) - 1
    max_chunk = max(chunk_offsets[c + 1] - chunk_offsets[c] for c in range(C))
    compute = torch.cuda.current_stream(dev)
    copy = copy_stream if copy_stream is not None else torch.cuda.Stream(dev)     # default priority
    stage_codes, stage_luts = staging if staging is not None else new_staging(max_chunk, W, dev)
    assert all(len(s) == W and s[0].numel() >= max_chunk + kLine - 1 for s in stage_codes)

    def views(c):
        a, b = chunk_offsets[c], chunk_offsets[c + 1]
        ph = a % kLine
        return [buf[ph:ph + b - a] for buf in stage_codes[c & 1]]
    arrived = [torch.cuda.Event() for _ in range(C)]
    reduced = [torch.cuda.Event() for _ in range(C)]
    ws = B.new_workspace(1, dev)
    qps = []

    def start_arrival(c):
        with torch.cuda.stream(copy):
            if c >= 2:
                copy.wait_event(reduced[c - 2])          # the staging set is free again
            arrive(c, views(c), stage_luts[c & 1])
            arrived[c].record(copy)

    copy.wait_stream(compute)
    start_arrival(0)
    for c in range(C):
        if overlap and c + 1 < C:
            start_arrival(c + 1)
        a, b = chunk_offsets[c], chunk_offsets[c + 1]
        compute.wait_event(arrived[c])
        qp = B.new_qparams(1, dev)
        if timing_out is not None:
            t0 = torch.cuda.Event(enable_timing=True)
            t0.record(compute)
        B.reduce_chunk(views(c), stage_luts[c & 1], [0, b - a], divisor,
                       local_fp32=local_fp32[a:b], acc_out=local_fp32[a:b], codes_out=codes_out[a:b],
                       lut_out=lut_out[c:c + 1], qparams_out=qp, workspace=ws, stream=compute)
        reduced[c].record(compute)
        if timing_out is not None:
            t1 = torch.cuda.Event(enable_timing=True)
            t1.record(compute)
            timing_out.append((t0, t1))
        qps.append(qp)
        if not overlap and c + 1 < C:
            copy.wait_event(reduced[c])
            start_arrival(c + 1)
    return qps
