"""Chunk-pipelined reduce (transfer of chunk c+1 overlapping the reduction of chunk c) against the
oracle's per-chunk reduce, and against the same calls issued strictly in order.

The coded contributions start in pinned host memory, or in a second resident copy in device memory; each
chunk is brought in by asynchronous copies on a second stream while the previous chunk is being reduced.
"""
import sys

import numpy as np
import pytest
import torch

from paper_2412_01152_amd import synth
from parity_utils import check_acc, check_codes, check_luts, check_qparams, t2n

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def B():
    from paper_2412_01152_amd import binding
    binding.load()
    assert torch.cuda.is_available(), "these tests need the GPU"
    return binding


@pytest.mark.parametrize("arrival", ["host to device", "device to device"])
@pytest.mark.parametrize("overlap", [True, False])
def test_pipelined_chunks_match_oracle(B, oracle_mod, overlap, arrival):
    from paper_2412_01152_amd.pipeline import reduce_chunks_pipelined
    W, C = 3, 5
    N = 1_500_007                                    # odd chunk size: chunks start off the 128-byte grid
    chunk_sizes = synth.ring_chunk_sizes(N, C)
    coff = synth.offsets_from_sizes(chunk_sizes)
    say(f"[pipeline] overlap={overlap} arrival={arrival} N={N} chunks={chunk_sizes} W={W}")
    theta, locals_, _ = synth.make_inputs([N], W + 1, kind="mixture", device="cpu")
    # every peer quantises each ring chunk as its own group (oracle, on the CPU)
    st = [oracle_mod.pseudograd_quantize(theta.numpy(), locals_[p].numpy(), coff) for p in range(W)]
    own = (theta - locals_[W]).numpy().copy()        # the owner's fp32 pseudo-gradient
    host_codes = [torch.from_numpy(s[0]).pin_memory() for s in st]
    host_luts = [torch.from_numpy(s[1]).pin_memory() for s in st]
    if arrival == "device to device":                # a second resident copy: the stand-in for a fast link
        host_codes = [h.to(DEV) for h in host_codes]
        host_luts = [h.to(DEV) for h in host_luts]

    def arrive(c, code_bufs, lut_bufs):
        a, b = coff[c], coff[c + 1]
        for p in range(W):
            code_bufs[p].copy_(host_codes[p][a:b], non_blocking=True)
            lut_bufs[p].copy_(host_luts[p][c:c + 1], non_blocking=True)

    local = torch.from_numpy(own).to(DEV)
    codes_out = torch.empty(N, dtype=torch.uint8, device=DEV)
    lut_out = torch.empty((C, 256), dtype=torch.float32, device=DEV)
    qps = reduce_chunks_pipelined(coff, W, W + 1, arrive, local, codes_out, lut_out, overlap=overlap)
    torch.cuda.synchronize()

    g_codes, g_luts, g_acc = t2n(codes_out), t2n(lut_out), t2n(local)
    for c in range(C):
        a, b = coff[c], coff[c + 1]
        o_acc, o_codes, o_luts, o_qp = oracle_mod.reduce([s[0][a:b] for s in st], [s[1][c:c + 1] for s in st],
                                                         [0, b - a], W + 1, local_fp32=own[a:b])
        check_qparams(B.qparams_to_numpy(qps[c]), o_qp)
        check_codes(g_codes[a:b], o_codes, o_acc, [0, b - a], o_qp)
        check_luts(g_luts[c:c + 1], o_luts, o_codes, [0, b - a], o_qp)
        mag = np.abs(own[a:b]).astype(np.float64)
        for s in st:
            mag += np.abs(s[1][c][s[0][a:b]])
        assert check_acc(g_acc[a:b], o_acc, np.maximum(np.abs(o_acc), mag / (W + 1))) == 0
