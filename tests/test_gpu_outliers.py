"""Outliers at the places the statistics pass samples its pivot from (needs an MI355X).

Section 2.2's quantiser takes the mean and standard deviation of the whole tensor and is meant to
tolerate outliers (they are clipped).  The library sums (x - c) and (x - c)^2 about a pivot c taken
from the segment itself, so a pivot that IS an outlier would cost precision in the variance.  These
tests put outliers of 3, 7 and 100 (the bulk has a standard deviation of 1e-3) on the first element
of large segments - one of them starting in the middle of a chunk of work - and on a last element,
for both quantising calls in all their forms, and require the fp32 range (lo, 1 / width) to be
bit-equal to the oracle's and not a single code to differ.
"""
import sys

import numpy as np
import pytest
import torch

from paper_2412_01152_amd import synth
from parity_utils import bf16_bits, check_codes, check_luts, check_qparams, t2n

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
SIZES = [5000, 1 << 24, (1 << 24) + 3]          # segment 1 starts mid-chunk, segment 2 at an odd offset


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def B():
    from paper_2412_01152_amd import binding
    binding.load()
    assert torch.cuda.is_available(), "these tests need the GPU"
    return binding


def _plant(values, off, outlier):
    """+outlier on the first element of every segment, -outlier on the last element of segment 1."""
    for s in range(len(off) - 1):
        values[off[s]] = outlier
    values[off[2] - 1] = -outlier


@pytest.mark.parametrize("outlier", [3.0, 7.0, 100.0])
@pytest.mark.parametrize("local_dtype", [torch.float32, torch.bfloat16])
def test_stage1_outlier_on_the_first_element(B, oracle_mod, outlier, local_dtype):
    theta, locals_, off = synth.make_inputs(SIZES, 1, kind="normal", device=DEV, local_dtype=local_dtype)
    local = locals_[0]
    for s in range(len(SIZES)):
        local[off[s]] = (theta[off[s]] - outlier).to(local_dtype)          # d = theta - local = +outlier
    local[off[2] - 1] = (theta[off[2] - 1] + outlier).to(local_dtype)
    say(f"[outlier] stage 1, {outlier} at segment starts, theta_local {local_dtype}")
    codes, luts, qp = B.pseudograd_quantize(theta, local, off)
    torch.cuda.synchronize()
    if local_dtype == torch.bfloat16:
        o_codes, o_luts, o_qp, o_d = oracle_mod.pseudograd_quantize(t2n(theta), bf16_bits(local), off,
                                                                    local_is_bf16=True)
    else:
        o_codes, o_luts, o_qp, o_d = oracle_mod.pseudograd_quantize(t2n(theta), t2n(local), off)
    assert abs(float(o_d[off[1]]) - outlier) < 0.05 * outlier                 # the outlier is where it should be
    exact = check_qparams(B.qparams_to_numpy(qp), o_qp, require_exact=1.0)
    flips = check_codes(t2n(codes), o_codes, o_d, off, o_qp)
    check_luts(t2n(luts), o_luts, o_codes, off, o_qp)
    assert flips == 0 and exact == len(SIZES)


def _stage2_both_forms(B, oracle_mod, off, codes, luts, divisor, local):
    """Recompute form, then the materialise form (in place over the local addend when there is one)."""
    n = off[-1]
    o_acc, o_c2, o_l2, o_q2 = oracle_mod.reduce(codes, luts, off, divisor, local_fp32=local)
    pc = [torch.from_numpy(c).to(DEV) for c in codes]
    pl = [torch.from_numpy(l).to(DEV) for l in luts]
    for materialise in (False, True):
        local_t = torch.from_numpy(local).to(DEV) if local is not None else None
        acc_t = None
        if materialise:
            acc_t = local_t if local_t is not None else torch.empty(n, dtype=torch.float32, device=DEV)
        c2, l2, q2 = B.reduce_chunk(pc, pl, off, divisor, local_fp32=local_t, acc_out=acc_t)
        torch.cuda.synchronize()
        exact = check_qparams(B.qparams_to_numpy(q2), o_q2, require_exact=1.0)
        flips = check_codes(t2n(c2), o_c2, o_acc, off, o_q2)
        check_luts(t2n(l2), o_l2, o_c2, off, o_q2)
        assert flips == 0 and exact == len(off) - 1
        if materialise:
            assert np.array_equal(t2n(acc_t), o_acc)
    return o_acc


@pytest.mark.parametrize("outlier", [3.0, 7.0, 100.0])
def test_stage2_outlier_in_the_local_addend(B, oracle_mod, outlier):
    """Three coded contributions plus the owner's fp32 data, whose first elements are outliers."""
    W = 3
    theta, locals_, off = synth.make_inputs(SIZES, W + 1, kind="normal", device="cpu")
    st = [oracle_mod.pseudograd_quantize(theta.numpy(), l.numpy(), off) for l in locals_[:W]]
    local = oracle_mod.pseudograd(theta.numpy(), locals_[W].numpy())
    _plant(local, off, np.float32(outlier * (W + 1)))                          # the average carries `outlier`
    say(f"[outlier] stage 2, W={W} coded + local addend with {outlier * (W + 1)} at segment starts")
    o_acc = _stage2_both_forms(B, oracle_mod, off, [s[0] for s in st], [s[1] for s in st], W + 1, local)
    assert abs(float(o_acc[off[1]]) - outlier) < 0.05 * outlier


@pytest.mark.parametrize("outlier", [3.0, 7.0, 100.0])
def test_stage2_outlier_decoded_from_a_code(B, oracle_mod, outlier):
    """Two coded contributions; the first one's top bucket holds a single element, the segment's first,
    and its codebook entry is the outlier (what stage 1 produces for a lone clipped value)."""
    W = 2
    theta, locals_, off = synth.make_inputs(SIZES, W, kind="normal", device="cpu")
    st = [oracle_mod.pseudograd_quantize(theta.numpy(), l.numpy(), off) for l in locals_]
    codes0, luts0 = st[0][0].copy(), st[0][1].copy()
    codes0[codes0 == 255] = 254
    for s in range(len(SIZES)):
        codes0[off[s]] = 255
        luts0[s][255] = np.float32(outlier * W)
    say(f"[outlier] stage 2, W={W} coded, first element decodes to {outlier * W}")
    o_acc = _stage2_both_forms(B, oracle_mod, off, [codes0, st[1][0]], [luts0, st[1][1]], W, None)
    assert abs(float(o_acc[off[1]]) - outlier) < 0.05 * outlier
