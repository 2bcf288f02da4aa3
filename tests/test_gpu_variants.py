"""The quantiser with another clipping width or the midpoint codebook (the *_variant calls) against
the oracle with the same two arguments, and the paper's values against the plain calls, bit for bit."""
import sys

import numpy as np
import pytest
import torch

from paper_2412_01152_amd import synth
from parity_utils import check_acc, check_codes, check_qparams, t2n

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
SIZES = [100_000, 4096, 3, 77_777, 0, 40_001]


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def B():
    from paper_2412_01152_amd import binding
    binding.load()
    assert torch.cuda.is_available(), "these tests need the GPU"
    return binding


def _check_luts_variant(g_luts, o_luts, o_codes, off, o_qp, range_sigmas):
    """Populated buckets within 1e-6 of max(|lut|, bucket width); unpopulated ones hold the midpoint."""
    so = np.asarray(off, dtype=np.int64)
    for s in range(o_luts.shape[0]):
        a, b = so[s], so[s + 1]
        if a == b:
            assert np.all(g_luts[s] == 0.0)
            continue
        w = 2.0 * range_sigmas * float(o_qp[s]["std"]) / 256.0
        pop = np.bincount(o_codes[a:b], minlength=256) > 0
        scale = np.maximum(np.abs(o_luts[s].astype(np.float64)), w)
        err = np.abs(g_luts[s].astype(np.float64) - o_luts[s]) / np.maximum(scale, 1e-300)
        assert np.all(err[pop] <= 1e-6), f"segment {s}: lut rel err {err[pop].max():.2e}"
        assert np.all(err[~pop] <= 1e-5)


@pytest.mark.parametrize("range_sigmas,codebook", [(4.0, "mean"), (8.0, "mean"), (2.5, "mean"), (6.0, "midpoint"),
                                                   (4.0, "midpoint")])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_stage1_variant(B, oracle_mod, range_sigmas, codebook, dtype):
    say(f"[variant] stage 1 c={range_sigmas} codebook={codebook} {dtype}")
    theta, locals_, off = synth.make_inputs(SIZES, 1, kind="mixture", device=DEV, local_dtype=dtype)
    cb = B.CODEBOOK_MIDPOINT if codebook == "midpoint" else B.CODEBOOK_MEAN
    codes, luts, qp = B.pseudograd_quantize(theta, locals_[0], off, variant=(range_sigmas, cb))
    torch.cuda.synchronize()
    if dtype == torch.bfloat16:
        local_np = np.ascontiguousarray(locals_[0].cpu().view(torch.int16).numpy().view(np.uint16))
    else:
        local_np = t2n(locals_[0])
    o_codes, o_luts, o_qp, o_d = oracle_mod.pseudograd_quantize(t2n(theta), local_np, off, local_is_bf16=dtype == torch.bfloat16,
                                                                range_sigmas=range_sigmas, codebook=codebook)
    check_qparams(B.qparams_to_numpy(qp), o_qp)
    check_codes(t2n(codes), o_codes, o_d, off, o_qp)
    _check_luts_variant(t2n(luts), o_luts, o_codes, off, o_qp, range_sigmas)


@pytest.mark.parametrize("range_sigmas,codebook", [(4.0, "mean"), (8.0, "midpoint")])
@pytest.mark.parametrize("W,with_acc", [(3, False), (5, True)])
def test_stage2_variant(B, oracle_mod, range_sigmas, codebook, W, with_acc):
    say(f"[variant] stage 2 c={range_sigmas} codebook={codebook} W={W} acc={with_acc}")
    theta, locals_, off = synth.make_inputs(SIZES, W + 1, kind="mixture", device="cpu")
    st = [oracle_mod.pseudograd_quantize(theta.numpy(), locals_[p].numpy(), off, range_sigmas=range_sigmas,
                                         codebook=codebook) for p in range(W)]
    own = (theta - locals_[W]).numpy().copy()
    cb = B.CODEBOOK_MIDPOINT if codebook == "midpoint" else B.CODEBOOK_MEAN
    acc_t = torch.empty(off[-1], dtype=torch.float32, device=DEV) if with_acc else None
    codes, luts, qp = B.reduce_chunk([torch.from_numpy(s[0]).to(DEV) for s in st],
                                     [torch.from_numpy(s[1]).to(DEV) for s in st], off, W + 1,
                                     local_fp32=torch.from_numpy(own).to(DEV), acc_out=acc_t,
                                     variant=(range_sigmas, cb))
    torch.cuda.synchronize()
    o_acc, o_codes, o_luts, o_qp = oracle_mod.reduce([s[0] for s in st], [s[1] for s in st], off, W + 1,
                                                     local_fp32=own, range_sigmas=range_sigmas, codebook=codebook)
    check_qparams(B.qparams_to_numpy(qp), o_qp)
    check_codes(t2n(codes), o_codes, o_acc, off, o_qp)
    _check_luts_variant(t2n(luts), o_luts, o_codes, off, o_qp, range_sigmas)
    if with_acc:
        so = np.asarray(off)
        mag = np.abs(own).astype(np.float64)
        for s_ in st:
            for k in range(len(off) - 1):
                mag[so[k]:so[k + 1]] += np.abs(s_[1][k][s_[0][so[k]:so[k + 1]]])
        assert check_acc(t2n(acc_t), o_acc, np.maximum(np.abs(o_acc), mag / (W + 1))) == 0


def test_paper_values_equal_the_plain_calls(B):
    theta, locals_, off = synth.make_inputs(SIZES, 3, kind="mixture", device=DEV)
    plain = [B.pseudograd_quantize(theta, l, off) for l in locals_]
    var = [B.pseudograd_quantize(theta, l, off, variant=(6.0, B.CODEBOOK_MEAN)) for l in locals_]
    torch.cuda.synchronize()
    def same_scales(qa, qb):                     # fp64 sums come from atomics: the last bits may differ
        qa, qb = B.qparams_to_numpy(qa), B.qparams_to_numpy(qb)
        for f in ("lo", "inv_w", "n", "status"):
            assert np.array_equal(qa[f], qb[f])
        assert np.allclose(qa["std"], qb["std"], rtol=1e-12, atol=0)

    for a, b in zip(plain, var):
        assert torch.equal(a[0], b[0])
        same_scales(a[2], b[2])
        assert torch.allclose(a[1], b[1], rtol=1e-6, atol=0)
    r0 = B.reduce_chunk([p[0] for p in plain], [p[1] for p in plain], off, 3)
    r1 = B.reduce_chunk([p[0] for p in plain], [p[1] for p in plain], off, 3, variant=(6.0, B.CODEBOOK_MEAN))
    torch.cuda.synchronize()
    assert torch.equal(r0[0], r1[0])
    same_scales(r0[2], r1[2])
    assert torch.allclose(r0[1], r1[1], rtol=1e-6, atol=0)
