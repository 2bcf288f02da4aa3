"""Comparison helpers for the GPU-vs-oracle parity tests (tolerances of the benchmark contract).

Codes: byte-equal, except that at most 1e-6 of the elements may differ by exactly one bucket and
only where the oracle's bucket coordinate sits within 1e-3 of a bucket edge.
Scales: lo / inv_w within 1e-6 relative and bit-equal in at least 99 % of the segments (checked where
there are 100 or more); mean (relative to std) and std within 1e-9.
Codebook (populated buckets): |diff| <= 1e-6 * max(|lut|, bucket width).
fp32 accumulations: |diff| <= 1e-6 * max(|a|, sum of |addends| / divisor).
Outer parameters and momentum: |diff| <= 1e-5 * max(|old|, |new|, lr * |g + beta m'|).
"""
import numpy as np


def t2n(t):
    return t.detach().cpu().numpy()


def bf16_bits(t):
    import torch
    return np.ascontiguousarray(t.detach().cpu().view(torch.int16).numpy().view(np.uint16))


def check_qparams(gpu_qp, orc_qp, require_exact=None):
    """Returns the number of segments whose fp32 (lo, inv_w) are bit-equal to the oracle's.  With 100 or
    more segments at least 99 % of them must be (require_exact overrides the fraction: 1.0 = all)."""
    assert gpu_qp.shape == orc_qp.shape
    exact = 0
    populated = 0
    for s in range(orc_qp.size):
        g, o = gpu_qp[s], orc_qp[s]
        assert g["n"] == o["n"], f"segment {s}: n {g['n']} vs {o['n']}"
        assert g["status"] == o["status"], f"segment {s}: status {g['status']} vs {o['status']}"
        sd = max(float(o["std"]), 1e-300)
        if o["n"] == 0:
            continue
        populated += 1
        assert abs(g["mean"] - o["mean"]) <= 1e-9 * sd, f"segment {s}: mean {g['mean']} vs {o['mean']}"
        assert abs(g["std"] - o["std"]) <= 1e-9 * sd, f"segment {s}: std {g['std']} vs {o['std']}"
        assert abs(float(g["lo"]) - float(o["lo"])) <= 1e-6 * abs(float(o["lo"])) + 1e-300, f"segment {s}: lo"
        assert abs(float(g["inv_w"]) - float(o["inv_w"])) <= 1e-6 * abs(float(o["inv_w"])), f"segment {s}: inv_w"
        exact += int(g["lo"] == o["lo"] and g["inv_w"] == o["inv_w"])
    if require_exact is None and populated >= 100:
        require_exact = 0.99
    if require_exact is not None:
        assert exact >= require_exact * populated, f"only {exact} of {populated} segments have bit-equal lo / inv_w"
    return exact


def check_codes(gpu_codes, orc_codes, x, seg_offsets, orc_qp, budget=1e-6):
    """x: the fp32 values the oracle quantised.  Returns the number of one-bucket flips."""
    assert gpu_codes.shape == orc_codes.shape
    diff = np.flatnonzero(gpu_codes != orc_codes)
    if diff.size == 0:
        return 0
    n = gpu_codes.size
    assert diff.size <= max(1.0, budget * n), f"{diff.size} of {n} codes differ (budget {budget * n:.2f})"
    so = np.asarray(seg_offsets, dtype=np.int64)
    seg = np.searchsorted(so, diff, side="right") - 1
    # skip empty segments that share an offset
    for i, s in zip(diff, seg):
        while so[s + 1] <= i:
            s += 1
        d = int(gpu_codes[i]) - int(orc_codes[i])
        assert abs(d) == 1, f"element {i}: codes {gpu_codes[i]} vs {orc_codes[i]}"
        lo, inv_w = np.float32(orc_qp[s]["lo"]), np.float32(orc_qp[s]["inv_w"])
        t = np.float32(np.float32(x[i] - lo) * inv_w)
        assert abs(float(t) - round(float(t))) < 1e-3, f"element {i}: flip away from an edge (t={t})"
    return int(diff.size)


def check_luts(gpu_luts, orc_luts, orc_codes, seg_offsets, orc_qp, tol=1e-6):
    gpu_luts = gpu_luts.reshape(-1, 256)
    orc_luts = orc_luts.reshape(-1, 256)
    so = np.asarray(seg_offsets, dtype=np.int64)
    worst = 0.0
    for s in range(orc_luts.shape[0]):
        a, b = so[s], so[s + 1]
        if b == a:
            assert np.all(gpu_luts[s] == 0.0)
            continue
        counts = np.bincount(orc_codes[a:b], minlength=256)
        pop = counts > 0
        w = 12.0 * float(orc_qp[s]["std"]) / 256.0
        scale = np.maximum(np.abs(orc_luts[s].astype(np.float64)), w)
        err = np.abs(gpu_luts[s].astype(np.float64) - orc_luts[s].astype(np.float64)) / np.maximum(scale, 1e-300)
        worst = max(worst, float(err[pop].max()))
        assert np.all(err[pop] <= tol), f"segment {s}: lut rel err {err[pop].max():.3e} at bucket {np.argmax(err * pop)}"
        # unpopulated buckets hold the bucket midpoint on both sides (never referenced by a code)
        if (~pop).any() and w > 0:
            assert np.all(np.abs(gpu_luts[s][~pop].astype(np.float64) - orc_luts[s][~pop]) <= 1e-5 * scale[~pop])
    return worst


def check_acc(gpu_acc, orc_acc, bound_scale):
    """bound_scale: max(|a|, sum |addends| / divisor) per element."""
    err = np.abs(gpu_acc.astype(np.float64) - orc_acc.astype(np.float64))
    lim = 1e-6 * np.maximum(bound_scale, 1e-300)
    bad = err > lim
    assert not bad.any(), f"{bad.sum()} accumulations off, worst {np.max(err / np.maximum(lim, 1e-300)):.2f}x"
    return int(np.count_nonzero(gpu_acc != orc_acc))


def check_outer(gpu_new, orc_new, old, step_scale, what, tol=1e-5):
    scale = np.maximum(np.maximum(np.abs(old), np.abs(orc_new)), step_scale).astype(np.float64)
    err = np.abs(gpu_new.astype(np.float64) - orc_new.astype(np.float64))
    bad = err > tol * np.maximum(scale, 1e-300)
    assert not bad.any(), f"{what}: {bad.sum()} off, worst rel {np.max(err / np.maximum(scale, 1e-300)):.3e}"
    return float(np.max(err / np.maximum(scale, 1e-300)))
