"""int8_reduce_chunk_static (the entry point that takes no workspace and allocates nothing) against
int8_reduce_chunk on the same inputs, through the C ABI (needs an MI355X).

Two calls in a row share the library's one static scratch array: the second, smaller call must not see
anything the first one left there.  Compared to the bar of every other parity test: the stored fp32
accumulation bit for bit (a fixed sequence of fp32 operations), mean / standard deviation to 1e-9 of the
standard deviation, codes byte-equal wherever the fp32 range came out bit-equal (else within the 1e-6
flip budget), codebooks within 1e-6 * max(|entry|, bucket width).
"""
import sys

import numpy as np
import pytest
import torch

from paper_2412_01152_amd import synth
from parity_utils import check_codes, check_luts, check_qparams, t2n

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


def _compare(B, peer_codes, peer_luts, off, divisor, local, label):
    n, T, W = off[-1], len(off) - 1, len(peer_codes)
    say(f"[static] {label}: n={n} T={T} W={W} local={'yes' if local is not None else 'no'}")
    # the existing entry point, with a caller's workspace
    acc_ref = torch.empty(n, dtype=torch.float32, device=DEV)
    c_ref, l_ref, q_ref = B.reduce_chunk(peer_codes, peer_luts, off, divisor, local_fp32=local, acc_out=acc_ref)
    torch.cuda.synchronize()
    # the static-scratch entry point: every buffer exists before the call
    acc = torch.empty(n, dtype=torch.float32, device=DEV)
    codes = torch.empty(n, dtype=torch.uint8, device=DEV)
    lut = torch.empty((T, 256), dtype=torch.float32, device=DEV)
    qp = B.new_qparams(T, DEV)
    torch.cuda.synchronize()
    free_before, _ = torch.cuda.mem_get_info()
    B.reduce_chunk_static(peer_codes, peer_luts, off, divisor, codes, lut, qp, local_fp32=local, acc_out=acc)
    torch.cuda.synchronize()
    free_after, _ = torch.cuda.mem_get_info()
    assert torch.equal(acc, acc_ref)
    g, r = B.qparams_to_numpy(qp), B.qparams_to_numpy(q_ref)
    exact = check_qparams(g, r)
    x = t2n(acc_ref)
    flips = check_codes(t2n(codes), t2n(c_ref), x, off, r)
    check_luts(t2n(lut), t2n(l_ref), t2n(c_ref), off, r)
    if exact == sum(1 for s in range(T) if off[s + 1] > off[s]):
        assert flips == 0
    say(f"[static] {label}: {exact}/{T} ranges bit-equal, flips={flips}, free HBM {free_before} -> {free_after}")
    return free_after


def test_static_scratch_matches_the_workspace_entry_point(B):
    W = 4
    sizes = [700_001, 4096, 0, 1_200_000, 3, 65_536 + 5, 1_000_000]
    off = synth.offsets_from_sizes(sizes)
    n, T = off[-1], len(sizes)
    peer_codes = [synth.fill_coded_contribution(torch.empty(n, dtype=torch.uint8, device=DEV), p) for p in range(W)]
    peer_luts = [synth.synthetic_codebooks(T, p, device=DEV) for p in range(W)]
    local = synth.fill_delta(torch.empty(n, dtype=torch.float32, device=DEV), W)
    free1 = _compare(B, peer_codes, peer_luts, off, W + 1, local, "first call")
    # second call, smaller and with fewer segments and peers, on views of the same buffers; no local addend
    sizes2 = [300_000, 17, 450_001]
    off2 = synth.offsets_from_sizes(sizes2)
    n2, T2 = off2[-1], len(sizes2)
    free2 = _compare(B, [c[5:5 + n2] for c in peer_codes[:3]], [l[:T2].contiguous() for l in peer_luts[:3]], off2, 3,
                     None, "second, smaller call")
    # once more the first shape: what the smaller call left in the scratch does not leak either
    _compare(B, peer_codes, peer_luts, off, W + 1, local, "third call, first shape again")
    assert free2 >= free1 - (64 << 20)                       # nothing of a chunk's size was allocated in between


def test_static_scratch_limit_is_refused(B):
    T = B.STATIC_MAX_SEGMENTS + 1
    off = list(range(0, 8 * (T + 1), 8))
    n = off[-1]
    codes = torch.zeros(n, dtype=torch.uint8, device=DEV)
    lut = torch.zeros((T, 256), dtype=torch.float32, device=DEV)
    with pytest.raises(B.DilocoError) as e:
        B.reduce_chunk_static([codes], [lut], off, 1, codes.clone(), lut.clone(), B.new_qparams(T, DEV))
    assert e.value.code == -6
    # exactly the limit is accepted
    off = off[:-1]
    n, T = off[-1], T - 1
    out_c, out_l, out_q = torch.empty(n, dtype=torch.uint8, device=DEV), lut[:T].clone(), B.new_qparams(T, DEV)
    B.reduce_chunk_static([codes[:n]], [lut[:T].contiguous()], off, 1, out_c, out_l, out_q)
    torch.cuda.synchronize()
    assert np.all(B.qparams_to_numpy(out_q)["status"] == B.STATUS_DEGENERATE)   # all-zero codebooks: constant tensors
