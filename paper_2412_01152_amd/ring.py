"""The ring reduce as Section 2.2 literally describes it, next to the one-shot W-way reduce.

In a ring reduce-scatter a chunk visits the W workers in turn: every worker dequantises what it
received, adds its own fp32 data, requantises and forwards; the paper notes that the additions must
happen on dequantised fp32 values and that only the transmitted terms are quantised.  Each hop is one
`int8_reduce_chunk` call with one coded contribution plus the fp32 local addend, so a value passes
through W quantisations on its way round (W - 1 hops and the final averaged result).  The one-shot
form hands all W coded contributions to a single call: every contribution is quantised once and the
result once.  Both are sequences of library calls; nothing here touches the data itself.
"""
from __future__ import annotations

from typing import List, Sequence

import torch

from . import binding as B


def quantise_fp32(d: torch.Tensor, seg_offsets: Sequence[int], workspace=None):
    """Q(d) for an fp32 tensor: the reduce call with no coded contribution and divisor 1."""
    return B.reduce_chunk([], [], seg_offsets, 1, local_fp32=d, workspace=workspace)


def dequantise(codes: torch.Tensor, lut: torch.Tensor, seg_offsets: Sequence[int], out=None, workspace=None):
    """lut[codes] as fp32: the reduce call with one coded contribution, divisor 1, storing the sum."""
    out = torch.empty(codes.numel(), dtype=torch.float32, device=codes.device) if out is None else out
    B.reduce_chunk([codes], [lut], seg_offsets, 1, acc_out=out, workspace=workspace)
    return out


def ring_reduce(d: List[torch.Tensor], seg_offsets: Sequence[int], workspace=None):
    """The chunk's trip round the ring: d[0] is quantised by its owner, workers 1 .. W-1 each add
    their own fp32 pseudo-gradient to the dequantised incoming chunk and requantise; the last one
    divides by W before requantising.  Returns (codes, lut, qparams) of the averaged chunk."""
    W = len(d)
    ws = B.new_workspace(len(seg_offsets) - 1, d[0].device) if workspace is None else workspace
    if W == 1:
        return quantise_fp32(d[0], seg_offsets, ws)
    codes, lut, qp = quantise_fp32(d[0], seg_offsets, ws)
    for s in range(1, W):
        nxt_codes = torch.empty_like(codes)
        nxt_lut = torch.empty_like(lut)
        _, _, qp = B.reduce_chunk([codes], [lut], seg_offsets, W if s == W - 1 else 1, local_fp32=d[s],
                                  codes_out=nxt_codes, lut_out=nxt_lut, workspace=ws)
        codes, lut = nxt_codes, nxt_lut
    return codes, lut, qp


def one_shot_reduce(d: List[torch.Tensor], seg_offsets: Sequence[int], workspace=None):
    """Every worker quantises its own pseudo-gradient once; one call reduces the W coded
    contributions and requantises the average."""
    W = len(d)
    ws = B.new_workspace(len(seg_offsets) - 1, d[0].device) if workspace is None else workspace
    coded = [quantise_fp32(x, seg_offsets, ws) for x in d]
    return B.reduce_chunk([c[0] for c in coded], [c[1] for c in coded], seg_offsets, W, workspace=ws)
