"""Pins of the CPU oracle against things other than itself (no GPU).

Each test ties one part of oracle/diloco_oracle.c to what the paper or the mathematics fixes:
error bounds of the 8-bit code (Section 2.2, quantisation list), exact special cases, closed
forms, an exact-rational brute force, and library routines used as black boxes.
"""
import math
from decimal import Decimal, getcontext
from fractions import Fraction

import numpy as np
import pytest
import torch

from paper_2412_01152_amd import synth


def _gauss(n, std=1e-3, mean=0.0, seed=0):
    rng = np.random.default_rng(seed)
    return (rng.normal(mean, std, n)).astype(np.float32)


def _mixture(n, seed=0):
    rng = np.random.default_rng(seed)
    pick = rng.random(n) < 0.9
    return np.where(pick, rng.normal(0, 1e-3, n), rng.laplace(0, 5e-3, n)).astype(np.float32)


# ---------------------------------------------------------------------------------------------
# statistics and range (Section 2.2 items 1-3)
# ---------------------------------------------------------------------------------------------

def test_stats_match_library_mean_std(oracle_mod):
    x = _mixture(200_003, seed=1) + np.float32(3e-4)
    _, _, qp = oracle_mod.quantize(x)
    x64 = x.astype(np.float64)
    assert qp["n"] == x.size
    assert abs(qp["mean"] - np.mean(x64)) <= 1e-12 * np.std(x64)
    assert abs(qp["std"] - np.std(x64, ddof=1)) <= 1e-12 * np.std(x64)
    # sample form, not population form: the two differ by far more than the tolerance here
    assert abs(qp["std"] - np.std(x64, ddof=0)) > 1e-9 * np.std(x64)


def test_range_is_mean_pm_6_sigma_in_256_buckets(oracle_mod):
    """Constants read from tests/golden/paper_constants.txt (6 sigma, 256 buckets)."""
    consts = _golden_constants()
    x = _gauss(50_000, std=2e-3, mean=1e-3, seed=2)
    _, _, qp = oracle_mod.quantize(x)
    mu, sd = np.mean(x.astype(np.float64)), np.std(x.astype(np.float64), ddof=1)
    k_sig, n_b = consts["range_sigmas"], consts["buckets"]
    assert qp["lo"] == np.float32(mu - k_sig * sd)
    w = 2 * k_sig * sd / n_b
    assert qp["inv_w"] == pytest.approx(1.0 / w, rel=2e-7)
    # the top edge lo + 256 w is mu + 6 sigma
    assert float(qp["lo"]) + n_b / float(qp["inv_w"]) == pytest.approx(mu + k_sig * sd, rel=1e-6)


def _golden_constants():
    import os
    out = {}
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_constants.txt")
    for line in open(path):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            out[k.strip()] = float(v)
    return out


# ---------------------------------------------------------------------------------------------
# P1 / P2 / P6: error bound, sum invariance, monotone codebook
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("maker,seed", [(_gauss, 3), (_mixture, 4)])
def test_roundtrip_error_bound(oracle_mod, maker, seed):
    x = maker(300_000, seed=seed)
    codes, lut, qp = oracle_mod.quantize(x)
    w = 12.0 * qp["std"] / 256.0
    xh = oracle_mod.dequantize(codes, lut)
    inside = (codes > 0) & (codes < 255)
    err = np.abs(x.astype(np.float64) - xh.astype(np.float64))
    # a value and the mean of its bucket lie in the same bucket of width w
    assert err[inside].max() < w * (1 + 1e-5)
    # high-resolution uniform quantiser: rms error about w / sqrt(12), never above w / 2
    rms = math.sqrt(np.mean(err[inside] ** 2))
    assert rms < 0.5 * w
    assert rms == pytest.approx(w / math.sqrt(12.0), rel=0.05)
    # every in-range value sits inside the bucket its code names
    t = (x.astype(np.float64) - (qp["mean"] - 6 * qp["std"])) / w
    assert np.all(np.abs(np.floor(t[inside]) - codes[inside]) <= 1)
    assert np.mean(np.floor(t[inside]) != codes[inside]) < 1e-4      # only fp32 edge effects


def test_sum_invariance_per_bucket_and_total(oracle_mod):
    x = _mixture(400_000, seed=5)
    codes, lut, _ = oracle_mod.quantize(x)
    x64 = x.astype(np.float64)
    for k in np.unique(codes):
        sel = codes == k
        s = x64[sel].sum()
        assert sel.sum() * float(lut[k]) == pytest.approx(s, rel=2e-7, abs=1e-12)
    xh = oracle_mod.dequantize(codes, lut).astype(np.float64)
    scale = np.abs(x64).sum()
    assert abs(xh.sum() - x64.sum()) <= 2 ** -23 * scale
    # clipped values are part of the end buckets' means: with them the invariant holds at the ends
    assert (codes == 0).sum() > 0 and (codes == 255).sum() > 0


def test_codebook_monotone_and_inside_buckets(oracle_mod):
    x = _gauss(500_000, seed=6)
    codes, lut, qp = oracle_mod.quantize(x)
    w = 12.0 * qp["std"] / 256.0
    lo = qp["mean"] - 6 * qp["std"]
    pop = np.unique(codes)
    assert np.all(np.diff(lut[pop]) > 0)
    for k in pop:
        if 1 <= k <= 254:
            assert lo + k * w - 1e-5 * w <= lut[k] <= lo + (k + 1) * w + 1e-5 * w
    # empty buckets carry their midpoint
    empty = np.setdiff1d(np.arange(256), pop)
    for k in empty:
        assert lut[k] == pytest.approx(lo + (k + 0.5) * w, rel=1e-6)


# ---------------------------------------------------------------------------------------------
# P3 / P4 / P5 / P9: exact special cases
# ---------------------------------------------------------------------------------------------

def _levels_tensor(n_levels=16, reps=1000, a=1e-3, seed=7):
    levels = (np.arange(n_levels) - (n_levels - 1) / 2.0) * (0.133 * a)
    x = np.repeat(levels.astype(np.float32), reps)
    np.random.default_rng(seed).shuffle(x)
    return np.ascontiguousarray(x)


def test_representable_values_reconstruct_exactly(oracle_mod):
    x = _levels_tensor()
    codes, lut, _ = oracle_mod.quantize(x)
    assert len(np.unique(codes)) == 16
    xh = oracle_mod.dequantize(codes, lut)
    assert np.array_equal(xh, x)
    # idempotence: quantising the decoded tensor decodes to the same values again
    codes2, lut2, _ = oracle_mod.quantize(xh)
    assert np.array_equal(oracle_mod.dequantize(codes2, lut2), x)


def test_power_of_two_equivariance(oracle_mod):
    x = _mixture(100_000, seed=8)
    codes, lut, qp = oracle_mod.quantize(x)
    for j in (-7, 5):
        s = np.float32(2.0 ** j)
        codes2, lut2, qp2 = oracle_mod.quantize(x * s)
        assert np.array_equal(codes2, codes)
        assert np.array_equal(lut2, lut * s)
        assert qp2["lo"] == qp["lo"] * s


@pytest.mark.parametrize("value", [0.0, 0.0123, -3.5e-4])
def test_constant_tensor_is_degenerate_and_exact(oracle_mod, value):
    """The all-zero pseudo-gradient of a node that joins without blocking (Section 2.4.2)."""
    x = np.full(5000, value, dtype=np.float32)
    codes, lut, qp = oracle_mod.quantize(x)
    assert qp["status"] & oracle_mod.STATUS_DEGENERATE
    assert qp["std"] == 0.0 and qp["inv_w"] == 0.0
    assert np.all(codes == 0)
    assert lut[0] == np.float32(value)
    assert np.array_equal(oracle_mod.dequantize(codes, lut), x)
    assert np.all(np.isfinite(lut))


def test_single_element_and_empty(oracle_mod):
    codes, lut, qp = oracle_mod.quantize(np.array([0.25], dtype=np.float32))
    assert codes[0] == 0 and lut[0] == 0.25 and qp["std"] == 0.0
    codes, lut, qp = oracle_mod.quantize(np.zeros(0, dtype=np.float32))
    assert qp["status"] == oracle_mod.STATUS_EMPTY and np.all(lut == 0)


def test_outlier_clips_into_end_bucket(oracle_mod):
    x = _gauss(100_000, seed=9)
    x[17] = 1.0       # a thousand sigma
    x[99] = -2.0
    codes, lut, qp = oracle_mod.quantize(x)
    assert codes[17] == 255 and codes[99] == 0
    # the outliers are part of the end buckets' averages
    assert lut[255] == pytest.approx(x[codes == 255].astype(np.float64).mean(), rel=1e-6)
    assert lut[0] == pytest.approx(x[codes == 0].astype(np.float64).mean(), rel=1e-6)


# ---------------------------------------------------------------------------------------------
# P7: brute force in exact rational arithmetic on tiny tensors
# ---------------------------------------------------------------------------------------------

def _exact_quantize(x, range_sigmas=6, midpoint=False):
    """Section 2.2 in exact arithmetic: returns codes, exact codebook entries of the populated buckets
    (bucket means, or bucket midpoints for the midpoint variant), distance to the nearest edge."""
    getcontext().prec = 60
    xs = [Fraction(float(v)) for v in x]
    n = len(xs)
    mu = sum(xs) / n
    var = sum((v - mu) ** 2 for v in xs) / (n - 1)
    sigma = Decimal(var.numerator) / Decimal(var.denominator)
    sigma = sigma.sqrt()
    sigma = Fraction(sigma)
    lo = mu - range_sigmas * sigma
    w = 2 * range_sigmas * sigma / 256
    codes, dist = [], []
    for v in xs:
        t = (v - lo) / w
        k = math.floor(t)
        dist.append(min(t - k, k + 1 - t))
        codes.append(min(255, max(0, k)))
    means = {}
    for k in set(codes):
        vals = [v for v, c in zip(xs, codes) if c == k]
        means[k] = lo + (k + Fraction(1, 2)) * w if midpoint else sum(vals) / len(vals)
    return codes, means, dist, mu, sigma


@pytest.mark.parametrize("seed", range(8))
def test_brute_force_exact_rational(oracle_mod, seed):
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(5, 64))
    while True:
        x = (rng.normal(0, 1e-3, n) + rng.normal(0, 2e-3)).astype(np.float32)
        if seed % 2:
            x[rng.integers(0, n)] *= 40.0        # force clipping
        codes_e, means_e, dist, mu, sigma = _exact_quantize(x)
        if min(dist) > Fraction(1, 1000):        # stay clear of bucket edges
            break
    codes, lut, qp = oracle_mod.quantize(x)
    assert list(codes) == codes_e
    assert qp["mean"] == pytest.approx(float(mu), rel=1e-13, abs=1e-18)
    assert qp["std"] == pytest.approx(float(sigma), rel=1e-13)
    for k, m in means_e.items():
        ref = np.float32(float(m))
        assert abs(float(lut[k]) - float(ref)) <= np.spacing(np.abs(ref))


@pytest.mark.parametrize("range_sigmas,codebook", [(4, "mean"), (8, "mean"), (3, "mean"), (6, "midpoint"),
                                                   (4, "midpoint")])
@pytest.mark.parametrize("seed", range(3))
def test_brute_force_variants(oracle_mod, seed, range_sigmas, codebook):
    """The quantiser's two knobs (clipping width, codebook of bucket midpoints) against exact arithmetic."""
    rng = np.random.default_rng(300 + seed)
    n = int(rng.integers(8, 64))
    while True:
        x = (rng.normal(0, 1e-3, n) + rng.normal(0, 2e-3)).astype(np.float32)
        codes_e, lut_e, dist, mu, sigma = _exact_quantize(x, range_sigmas, codebook == "midpoint")
        if min(dist) > Fraction(1, 1000):
            break
    codes, lut, qp = oracle_mod.quantize(x, range_sigmas=range_sigmas, codebook=codebook)
    assert list(codes) == codes_e
    for k, m in lut_e.items():
        ref = np.float32(float(m))
        assert abs(float(lut[k]) - float(ref)) <= np.spacing(np.abs(ref))


def test_variant_defaults_are_the_papers(oracle_mod):
    x = _mixture(50_000, seed=21)
    a = oracle_mod.quantize(x)
    b = oracle_mod.quantize(x, range_sigmas=6.0, codebook="mean")
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1]) and a[2] == b[2]


def test_midpoint_codebook_keeps_codes_but_not_the_sum(oracle_mod):
    """The codebook does not influence the codes; bucket means preserve the tensor's sum, midpoints of
    a skewed tensor do not (the reason Section 2.2 gives for the codebook of averages)."""
    rng = np.random.default_rng(22)
    x = rng.exponential(1e-3, 200_000).astype(np.float32)
    c_mean, l_mean, qp = oracle_mod.quantize(x)
    c_mid, l_mid, _ = oracle_mod.quantize(x, codebook="midpoint")
    assert np.array_equal(c_mean, c_mid)
    w = 12 * qp["std"] / 256
    lo = qp["mean"] - 6 * qp["std"]
    assert np.allclose(l_mid, lo + (np.arange(256) + 0.5) * w, rtol=1e-6, atol=0)
    total = x.astype(np.float64).sum()
    assert abs(l_mean[c_mean].astype(np.float64).sum() - total) <= 1e-6 * abs(total)
    assert abs(l_mid[c_mid].astype(np.float64).sum() - total) > 1e-4 * abs(total)
    inside = (c_mid > 0) & (c_mid < 255)
    assert np.all(np.abs(x[inside] - l_mid[c_mid[inside]]) <= 0.5 * w * (1 + 1e-4))


# ---------------------------------------------------------------------------------------------
# P8: Gaussian closed form
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("c", [4.0, 8.0])
def test_gaussian_closed_form_other_clip_widths(oracle_mod, c):
    """Occupancy and error for a range of +-c sigma: inner buckets follow the normal CDF with step
    2c/256, the end buckets also hold the clipped tails (2 Phi(-c) of the values in total)."""
    n = 1 << 22
    s = 1e-3
    x = _gauss(n, std=s, seed=11)
    codes, lut, qp = oracle_mod.quantize(x, range_sigmas=c)
    phi = lambda z: 0.5 * (1 + math.erf(z / math.sqrt(2)))
    counts = np.bincount(codes, minlength=256)
    step = 2 * c / 256.0
    for k in range(256):
        a = -math.inf if k == 0 else (k - 128) * step
        b = math.inf if k == 255 else (k - 127) * step
        p = phi(b) - phi(a) if k not in (0, 255) else (phi(b) if k == 0 else 1 - phi(a))
        se = math.sqrt(n * p * (1 - p))
        assert abs(counts[k] - n * p) <= 5 * se + 2, k
    xh = oracle_mod.dequantize(codes, lut)
    inside = np.abs(x) < (c - step) * s
    rms = math.sqrt(np.mean((x[inside].astype(np.float64) - xh[inside]) ** 2))
    assert rms / s == pytest.approx(step / math.sqrt(12), rel=0.03)


def test_gaussian_bucket_occupancy_and_rms(oracle_mod):
    n = 1 << 22
    s = 1e-3
    x = _gauss(n, std=s, seed=10)
    codes, lut, qp = oracle_mod.quantize(x)
    phi = lambda z: 0.5 * (1 + math.erf(z / math.sqrt(2)))
    counts = np.bincount(codes, minlength=256)
    step = 12.0 / 256.0                       # bucket width in units of sigma
    for k in range(1, 255):
        p = phi((k - 127) * step) - phi((k - 128) * step)
        exp = n * p
        se = math.sqrt(n * p * (1 - p))
        assert abs(counts[k] - exp) <= 5 * se + 2
    xh = oracle_mod.dequantize(codes, lut)
    rms = math.sqrt(np.mean((x.astype(np.float64) - xh) ** 2))
    assert rms / s == pytest.approx(step / math.sqrt(12), rel=0.02)
    # beyond six sigma: about 2 * Phi(-6) = 2e-9 of the values, i.e. none or a handful here
    assert counts[0] + counts[255] < 200


# ---------------------------------------------------------------------------------------------
# pseudo-gradient (Algorithm 1)
# ---------------------------------------------------------------------------------------------

def test_pseudograd_is_fp32_difference(oracle_mod):
    theta, locals_, _ = synth.make_inputs([70_001], 1)
    to, tl = theta.numpy(), locals_[0].numpy()
    d = oracle_mod.pseudograd(to, tl)
    assert np.array_equal(d, to - tl)                       # numpy's own fp32 subtraction
    assert abs(np.std(d) - 2.43e-3) < 2e-4                  # mixture: sqrt(.9*1e-6 + .1*2*25e-6)


def test_pseudograd_bf16_upcast_is_exact(oracle_mod):
    theta, locals_, _ = synth.make_inputs([50_000], 1, local_dtype=torch.bfloat16)
    tl_bits = locals_[0].view(torch.int16).numpy().view(np.uint16)
    d = oracle_mod.pseudograd(theta.numpy(), np.ascontiguousarray(tl_bits), local_is_bf16=True)
    ref = (theta - locals_[0].float()).numpy()              # torch's own widening
    assert np.array_equal(d, ref)


def test_segments_are_independent_groups(oracle_mod):
    sizes = [1000, 1, 0, 4097, 333]
    off = synth.offsets_from_sizes(sizes)
    x = _mixture(sum(sizes), seed=11)
    x[off[3]:off[4]] *= 50          # a very different scale in one segment
    codes, luts, qps = oracle_mod.quantize_segments(x, off)
    for s in range(len(sizes)):
        c1, l1, q1 = oracle_mod.quantize(np.ascontiguousarray(x[off[s]:off[s + 1]]))
        assert np.array_equal(codes[off[s]:off[s + 1]], c1)
        assert np.array_equal(luts[s], l1)
        assert qps[s]["lo"] == q1["lo"] and qps[s]["n"] == sizes[s]
    assert qps[2]["status"] == oracle_mod.STATUS_EMPTY


# ---------------------------------------------------------------------------------------------
# P10 / P11 / P12: reduction (Section 2.2, fp32 accumulation)
# ---------------------------------------------------------------------------------------------

def test_reduce_w1_is_decoding_and_keeps_the_sum(oracle_mod):
    x = _mixture(120_000, seed=12)
    off = [0, 50_000, 120_000]
    codes, luts, _ = oracle_mod.quantize_segments(x, off)
    acc, c2, l2, q2 = oracle_mod.reduce([codes], [luts], off, divisor=1)
    dec = np.concatenate([luts[s][codes[off[s]:off[s + 1]]] for s in range(2)])
    assert np.array_equal(acc, dec)
    for s in range(2):
        seg = slice(off[s], off[s + 1])
        assert acc[seg].astype(np.float64).sum() == pytest.approx(
            x[seg].astype(np.float64).sum(), abs=2 ** -22 * np.abs(x[seg]).sum())
    # requantising a 256-level tensor keeps every level apart or merges neighbours, never moves
    # a value by more than one new bucket
    w2 = 12 * q2["std"][0] / 256
    dec2 = l2[0][c2[:off[1]]]
    inside = (c2[:off[1]] > 0) & (c2[:off[1]] < 255)
    assert np.abs(dec2 - acc[:off[1]])[inside].max() < w2 * (1 + 1e-5)


def test_reduce_two_identical_peers_divisor_two(oracle_mod):
    x = _gauss(40_000, seed=13)
    codes, lut, _ = oracle_mod.quantize(x)
    acc, *_ = oracle_mod.reduce([codes, codes], [lut[None], lut[None]], [0, x.size], divisor=2)
    assert np.array_equal(acc, lut[codes])


def test_reduce_is_fp32_sum_of_decoded_values_not_code_arithmetic(oracle_mod):
    a = _gauss(60_000, std=1e-3, seed=14)
    b = _gauss(60_000, std=3e-3, seed=15)
    ca, la, _ = oracle_mod.quantize(a)
    cb, lb, _ = oracle_mod.quantize(b)
    off = [0, a.size]
    acc, cr, lr_, _ = oracle_mod.reduce([ca, cb], [la[None], lb[None]], off, divisor=1)
    assert np.array_equal(acc, la[ca] + lb[cb])             # numpy fp32 gather + add
    # Q(a) + Q(b) != Q(a + b): neither the codes nor the decoded values agree
    cs, ls, _ = oracle_mod.quantize(a + b)
    assert np.mean(acc != ls[cs]) > 0.5
    naive = np.clip(ca.astype(np.int32) + cb.astype(np.int32) - 128, 0, 255)
    assert np.mean(naive != cs) > 0.5
    # the requantised output is Q of the fp32 sum
    c2, l2, _ = oracle_mod.quantize(acc)
    assert np.array_equal(cr, c2) and np.array_equal(lr_[0], l2)


def test_reduce_average_and_local_addend(oracle_mod):
    W = 5
    xs = [_mixture(30_000, seed=20 + p) for p in range(W)]
    local = _mixture(30_000, seed=40)
    qs = [oracle_mod.quantize(x) for x in xs]
    off = [0, 30_000]
    acc, *_ = oracle_mod.reduce([q[0] for q in qs], [q[1][None] for q in qs], off, divisor=W + 1,
                                local_fp32=local)
    ref = local.copy()
    for c, l, _ in qs:
        ref = ref + l[c]
    ref = ref / np.float32(W + 1)
    assert np.array_equal(acc, ref)
    exact = (local.astype(np.float64) + sum(x.astype(np.float64) for x in xs)) / (W + 1)
    wmax = max(12 * q[2]["std"] / 256 for q in qs)
    inside = np.all([(q[0] > 0) & (q[0] < 255) for q in qs], axis=0)
    assert np.abs(acc - exact)[inside].max() < wmax * W / (W + 1) + 1e-9


# ---------------------------------------------------------------------------------------------
# P13 / P14 / P15: outer Nesterov step (Algorithm 1; lr 0.7, momentum 0.9 from the config table)
# ---------------------------------------------------------------------------------------------

def test_nesterov_closed_form(oracle_mod):
    consts = _golden_constants()
    lr, beta = consts["outer_lr"], consts["outer_momentum"]
    n, steps = 1000, 6
    rng = np.random.default_rng(30)
    theta0 = rng.normal(0, 0.02, n).astype(np.float32)
    g = rng.normal(0, 1e-3, n).astype(np.float32)
    theta, m = theta0.copy(), np.zeros(n, dtype=np.float32)
    b, l = float(np.float32(beta)), float(np.float32(lr))
    for t in range(1, steps + 1):
        oracle_mod.outer_step(theta, m, lr, beta, delta_fp32=g)
        m_ref = g.astype(np.float64) * (1 - b ** t) / (1 - b)
        coef = sum(1 + b * (1 - b ** j) / (1 - b) for j in range(1, t + 1))
        th_ref = theta0.astype(np.float64) - l * g.astype(np.float64) * coef
        assert np.allclose(m, m_ref, rtol=1e-6, atol=1e-12)
        assert np.allclose(theta, th_ref, rtol=1e-6, atol=1e-9)
        if t == 1:      # first step from a zero buffer: theta - lr (1 + beta) g = theta - 1.33 g
            assert np.allclose(theta, theta0 - 1.33 * g.astype(np.float64), rtol=1e-6, atol=1e-9)


def test_nesterov_matches_library_sgd(oracle_mod):
    n = 4096
    rng = np.random.default_rng(31)
    theta0 = rng.normal(0, 0.02, n).astype(np.float32)
    theta, m = theta0.copy(), np.zeros(n, dtype=np.float32)
    p = torch.nn.Parameter(torch.from_numpy(theta0.copy()))
    opt = torch.optim.SGD([p], lr=0.7, momentum=0.9, nesterov=True, dampening=0.0)
    for step in range(5):
        g = rng.normal(0, 1e-3, n).astype(np.float32)
        oracle_mod.outer_step(theta, m, 0.7, 0.9, delta_fp32=g)
        p.grad = torch.from_numpy(g.copy())
        opt.step()
        assert np.allclose(theta, p.detach().numpy(), rtol=1e-6, atol=1e-8)
        # the library rounds every step to fp32; near-cancelling sums are compared on the summands' scale
        assert np.allclose(m, opt.state[p]["momentum_buffer"].numpy(), rtol=1e-6, atol=2e-9)


def test_plain_averaging_special_case(oracle_mod):
    """beta = 0, lr = 1, un-quantised delta: Algorithm 1 is parameter averaging (local SGD)."""
    theta, locals_, _ = synth.make_inputs([20_000], 4)
    to = theta.numpy().copy()
    ls = [l.numpy() for l in locals_]
    delta = np.zeros_like(to, dtype=np.float64)
    for l in ls:
        delta += oracle_mod.pseudograd(to, l).astype(np.float64)
    delta = (delta / 4).astype(np.float32)
    m = np.zeros_like(to)
    oracle_mod.outer_step(to, m, 1.0, 0.0, delta_fp32=delta)
    avg = np.mean(np.stack(ls).astype(np.float64), axis=0)
    assert np.allclose(to, avg, rtol=1e-6, atol=1e-8)


def test_outer_step_coded_delta_and_handback(oracle_mod):
    n = 30_000
    off = [0, 10_000, 30_000]
    g = _mixture(n, seed=32)
    codes, luts, _ = oracle_mod.quantize_segments(g, off)
    dec = np.concatenate([luts[s][codes[off[s]:off[s + 1]]] for s in range(2)])
    rng = np.random.default_rng(33)
    theta = rng.normal(0, 0.02, n).astype(np.float32)
    m = rng.normal(0, 1e-3, n).astype(np.float32)
    t1, m1 = theta.copy(), m.copy()
    t2, m2 = theta.copy(), m.copy()
    out_bf16 = oracle_mod.outer_step(t1, m1, 0.7, 0.9, delta_codes=codes, delta_luts=luts,
                                     seg_offsets=off, local_out_dtype="bf16")
    out_f32 = oracle_mod.outer_step(t2, m2, 0.7, 0.9, delta_fp32=dec, local_out_dtype="fp32")
    assert np.array_equal(t1, t2) and np.array_equal(m1, m2)      # coded form = decoded fp32 form
    assert np.array_equal(out_f32, t2)
    ref_bits = torch.from_numpy(t1).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(out_bf16, ref_bits)                      # library's round-to-nearest-even


# ---------------------------------------------------------------------------------------------
# P16: one full quantised outer synchronisation stays within the composed error bound
# ---------------------------------------------------------------------------------------------

def test_end_to_end_drift_bound(oracle_mod):
    W = 4
    theta, locals_, off = synth.make_inputs([60_000, 5_000], W)
    to = theta.numpy()
    stage1 = [oracle_mod.pseudograd_quantize(to, l.numpy(), off) for l in locals_]
    acc, c2, l2, q2 = oracle_mod.reduce([s[0] for s in stage1], [s[1] for s in stage1], off, W)
    th_q, m_q = to.copy(), np.zeros_like(to)
    oracle_mod.outer_step(th_q, m_q, 0.7, 0.9, delta_codes=c2, delta_luts=l2, seg_offsets=off)
    exact_delta = np.mean(np.stack([s[3] for s in stage1]).astype(np.float64), axis=0)
    th_exact = to.astype(np.float64) - 0.7 * 1.9 * exact_delta
    for s in range(2):
        seg = slice(off[s], off[s + 1])
        w1 = max(12 * st[2]["std"][s] / 256 for st in stage1)
        w2 = 12 * q2["std"][s] / 256
        inside = np.all([(st[0][seg] > 0) & (st[0][seg] < 255) for st in stage1], axis=0)
        inside &= (c2[seg] > 0) & (c2[seg] < 255)
        bound = 0.7 * 1.9 * (w1 + w2) * (1 + 1e-4) + 1e-8
        assert np.abs(th_q[seg] - th_exact[seg])[inside].max() <= bound
        assert inside.mean() > 0.9


def test_payload_is_a_quarter(oracle_mod):
    """One byte per element plus a 1 KiB codebook per tensor: the 4x payload reduction."""
    consts = _golden_constants()
    n = 1 << 20
    x = _gauss(n, seed=34)
    codes, lut, _ = oracle_mod.quantize(x)
    ratio = x.nbytes / (codes.nbytes + lut.nbytes)
    assert ratio == pytest.approx(consts["payload_reduction"], rel=2e-3)
