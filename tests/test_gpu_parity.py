"""GPU-vs-oracle parity, element by element, through the C ABI (needs an MI355X).

Every test generates seeded synthetic inputs once, hands the same bits to the CPU oracle and to the
library, and compares with the tolerances in parity_utils.  Stage-isolated tests feed each GPU
stage the oracle's outputs of the previous stage, so a single edge flip upstream cannot cascade;
the chained test runs GPU stage into GPU stage.
"""
import sys

import numpy as np
import pytest
import torch

from paper_2412_01152_amd import synth
from parity_utils import (bf16_bits, check_acc, check_codes, check_luts, check_outer, check_qparams,
                          t2n)

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


def _oracle_stage1(oracle_mod, theta, local, off):
    if local.dtype == torch.bfloat16:
        return oracle_mod.pseudograd_quantize(t2n(theta), bf16_bits(local), off, local_is_bf16=True)
    return oracle_mod.pseudograd_quantize(t2n(theta), t2n(local), off)


def _check_stage1(B, oracle_mod, theta, local, off, label):
    say(f"[stage1] {label}: N={theta.numel()} T={len(off) - 1} dtype={local.dtype}")
    codes, luts, qp = B.pseudograd_quantize(theta, local, off)
    torch.cuda.synchronize()
    o_codes, o_luts, o_qp, o_d = _oracle_stage1(oracle_mod, theta, local, off)
    g_qp = B.qparams_to_numpy(qp)
    exact = check_qparams(g_qp, o_qp)
    flips = check_codes(t2n(codes), o_codes, o_d, off, o_qp)
    worst = check_luts(t2n(luts), o_luts, o_codes, off, o_qp)
    say(f"[stage1] {label}: flips={flips} exact-scale segments={exact}/{len(off) - 1} worst lut rel={worst:.2e}")
    return codes, luts, qp


# ---------------------------------------------------------------------------------------------
# stage 1
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("local_dtype", [torch.float32, torch.bfloat16])
def test_stage1_config0(B, oracle_mod, local_dtype):
    theta, locals_, off = synth.make_inputs(synth.config_segment_sizes(0), 1, device=DEV,
                                            local_dtype=local_dtype)
    _check_stage1(B, oracle_mod, theta, locals_[0], off, "config0")


@pytest.mark.parametrize("kind", ["mixture", "student_t3"])
def test_stage1_ragged_segments(B, oracle_mod, kind):
    sizes = synth.ragged_sizes(3_000_000)
    theta, locals_, off = synth.make_inputs(sizes, 1, kind=kind, device=DEV)
    _check_stage1(B, oracle_mod, theta, locals_[0], off, f"ragged/{kind}")


@pytest.mark.parametrize("shift", [1, 2, 3])
def test_stage1_misaligned_pointers(B, oracle_mod, shift):
    """Element-aligned only: fp32 pointers off by 4*shift bytes, codes off by `shift` bytes."""
    sizes = [5000, 70_001, 12_345, 262_144 + 3]
    n = sum(sizes)
    theta_full, locals_, _ = synth.make_inputs([n + 8], 1, device=DEV)
    theta = theta_full[shift:shift + n]
    local = locals_[0][shift:shift + n]
    off = synth.offsets_from_sizes(sizes)
    codes_buf = torch.zeros(n + 16, dtype=torch.uint8, device=DEV)
    codes_view = codes_buf[shift:shift + n]
    codes, luts, qp = B.pseudograd_quantize(theta, local, off, codes_out=codes_view)
    torch.cuda.synchronize()
    o_codes, o_luts, o_qp, o_d = oracle_mod.pseudograd_quantize(
        np.ascontiguousarray(t2n(theta)), np.ascontiguousarray(t2n(local)), off)
    check_qparams(B.qparams_to_numpy(qp), o_qp)
    check_codes(t2n(codes), o_codes, o_d, off, o_qp)
    check_luts(t2n(luts), o_luts, o_codes, off, o_qp)
    # nothing written outside the view
    assert int(codes_buf[:shift].sum()) == 0 and int(codes_buf[shift + n:].sum()) == 0


def test_stage1_bf16_misaligned(B, oracle_mod):
    sizes = [4099, 100_000]
    n = sum(sizes)
    theta_full, locals_, _ = synth.make_inputs([n + 8], 1, device=DEV, local_dtype=torch.bfloat16)
    theta, local = theta_full[3:3 + n], locals_[0][1:1 + n]      # different phases on purpose
    off = synth.offsets_from_sizes(sizes)
    codes, luts, qp = B.pseudograd_quantize(theta, local, off)
    torch.cuda.synchronize()
    o_codes, o_luts, o_qp, o_d = oracle_mod.pseudograd_quantize(
        np.ascontiguousarray(t2n(theta)), bf16_bits(local.contiguous()), off, local_is_bf16=True)
    check_qparams(B.qparams_to_numpy(qp), o_qp)
    check_codes(t2n(codes), o_codes, o_d, off, o_qp)
    check_luts(t2n(luts), o_luts, o_codes, off, o_qp)


def test_stage1_zero_delta_joiner(B, oracle_mod):
    """A node that joins without blocking contributes an all-zero pseudo-gradient (Section 2.4.2)."""
    sizes = [4096, 100_001, 1]
    theta, _, off = synth.make_inputs(sizes, 0, device=DEV)
    local = theta.clone()
    codes, luts, qp = B.pseudograd_quantize(theta, local, off)
    torch.cuda.synchronize()
    g_qp = B.qparams_to_numpy(qp)
    assert np.all(g_qp["status"] == B.STATUS_DEGENERATE)
    assert np.all(t2n(codes) == 0)
    assert np.all(t2n(luts)[:, 0] == 0.0) and np.all(np.isfinite(t2n(luts)))
    o_codes, o_luts, o_qp, _ = oracle_mod.pseudograd_quantize(t2n(theta), t2n(local), off)
    check_qparams(g_qp, o_qp)
    assert np.array_equal(t2n(luts), o_luts)


def test_stage1_outlier_and_constant_segment(B, oracle_mod):
    sizes = [50_000, 8192, 30_000]
    theta, locals_, off = synth.make_inputs(sizes, 1, device=DEV)
    local = locals_[0]
    local[off[1]:off[2]] = theta[off[1]:off[2]] - 0.125            # constant pseudo-gradient 0.125
    local[17] = theta[17] - 3.0                                     # one huge outlier
    local[off[2] + 5] = theta[off[2] + 5] + 7.0
    _check_stage1(B, oracle_mod, theta, local, off, "outlier+constant")


def test_stage1_is_repeatable(B):
    """Two calls on the same inputs.  The statistics are merged with fp64 atomic additions whose order
    varies from launch to launch (blocks claim their chunks dynamically), so the mean and standard
    deviation repeat only to a few units in the last place; once rounded to the fp32 pair the bucket index
    uses they coincide except in the rare case that the fp64 value sits at a rounding boundary.  Given
    equal (lo, 1 / width) everything else is exact: codes are pure fp32 arithmetic and the bucket sums
    are integers, whose order of addition does not matter."""
    theta, locals_, off = synth.make_inputs(synth.ragged_sizes(1_000_000), 1, device=DEV)
    c1, l1, q1 = B.pseudograd_quantize(theta, locals_[0], off)
    c2, l2, q2 = B.pseudograd_quantize(theta, locals_[0], off)
    torch.cuda.synchronize()
    q1, q2 = B.qparams_to_numpy(q1), B.qparams_to_numpy(q2)
    sd = np.maximum(q1["std"], 1e-300)
    assert np.all(np.abs(q1["mean"] - q2["mean"]) <= 1e-12 * sd) and np.all(np.abs(q1["std"] - q2["std"]) <= 1e-12 * sd)
    same = (q1["lo"] == q2["lo"]) & (q1["inv_w"] == q2["inv_w"])
    assert same.sum() >= len(same) - 1
    c1, c2, l1, l2 = t2n(c1), t2n(c2), t2n(l1), t2n(l2)
    for s in np.flatnonzero(same):
        assert np.array_equal(c1[off[s]:off[s + 1]], c2[off[s]:off[s + 1]])
        counts = np.bincount(c1[off[s]:off[s + 1]], minlength=256)
        assert np.array_equal(l1[s][counts > 0], l2[s][counts > 0])
    assert np.count_nonzero(c1 != c2) <= max(1, 1e-5 * c1.size)
    assert np.allclose(l1, l2, rtol=1e-6, atol=0)


def test_empty_input(B):
    off = [0, 0]
    theta = torch.empty(0, dtype=torch.float32, device=DEV)
    codes, luts, qp = B.pseudograd_quantize(theta, theta.clone(), off)
    torch.cuda.synchronize()
    g = B.qparams_to_numpy(qp)
    assert g["status"][0] == B.STATUS_EMPTY and np.all(t2n(luts) == 0)


# ---------------------------------------------------------------------------------------------
# stage 2 (fed with the oracle's stage-1 outputs)
# ---------------------------------------------------------------------------------------------

def _oracle_peers(oracle_mod, sizes, W, kind="mixture", seed=synth.BASE_SEED):
    theta, locals_, off = synth.make_inputs(sizes, W, kind=kind, device="cpu", seed=seed)
    st = [oracle_mod.pseudograd_quantize(theta.numpy(), l.numpy(), off) for l in locals_]
    return theta, off, st


def _run_stage2(B, oracle_mod, off, st, W, divisor, local=None, with_acc=False, alias=False):
    peer_codes = [torch.from_numpy(s[0]).to(DEV) for s in st[:W]]
    peer_luts = [torch.from_numpy(s[1]).to(DEV) for s in st[:W]]
    n = off[-1]
    local_t = torch.from_numpy(local).to(DEV) if local is not None else None
    acc_t = None
    if with_acc:
        acc_t = local_t if (alias and local_t is not None) else torch.empty(n, dtype=torch.float32, device=DEV)
    codes, luts, qp = B.reduce_chunk(peer_codes, peer_luts, off, divisor, local_fp32=local_t, acc_out=acc_t)
    torch.cuda.synchronize()
    o_acc, o_codes, o_luts, o_qp = oracle_mod.reduce([s[0] for s in st[:W]], [s[1] for s in st[:W]], off,
                                                     divisor, local_fp32=local)
    check_qparams(B.qparams_to_numpy(qp), o_qp)
    flips = check_codes(t2n(codes), o_codes, o_acc, off, o_qp)
    check_luts(t2n(luts), o_luts, o_codes, off, o_qp)
    if with_acc:
        mag = np.abs(local).astype(np.float64) if local is not None else np.zeros(n)
        so = np.asarray(off)
        for s_ in st[:W]:
            for k in range(len(off) - 1):
                mag[so[k]:so[k + 1]] += np.abs(s_[1][k][s_[0][so[k]:so[k + 1]]])
        unequal = check_acc(t2n(acc_t), o_acc, np.maximum(np.abs(o_acc), mag / divisor))
        assert unequal == 0, "fp32 accumulation is a fixed sequence of rounded operations: must be bit-equal"
    return flips


@pytest.mark.parametrize("W", list(range(1, 17)))
def test_stage2_all_w(B, oracle_mod, W):
    sizes = [100_000, 4096, 3, 77_777, 0, 40_001]
    _, off, st = _oracle_peers(oracle_mod, sizes, W)
    say(f"[stage2] W={W} recompute")
    _run_stage2(B, oracle_mod, off, st, W, divisor=W)
    say(f"[stage2] W={W} materialise")
    _run_stage2(B, oracle_mod, off, st, W, divisor=W, with_acc=True)


def test_segment_count_at_the_limit(B, oracle_mod):
    """65,536 quantisation groups (the largest T the library takes) of 0 .. 96 elements - empty ones,
    single values, a few hundred blocks' worth of segment changes per chunk - through all three calls."""
    T, W = 65_536, 3
    rng = np.random.default_rng(20241201)
    sizes = rng.integers(0, 97, size=T).tolist()
    sizes[5], sizes[77], sizes[T - 1] = 0, 1, 1
    theta, off, st = _oracle_peers(oracle_mod, sizes, W)
    n = off[-1]
    say(f"[limit] T={T} n={n}")
    assert B.workspace_bytes(T) > 0
    # stage 1 on worker 0's inputs
    _, locals_, _ = synth.make_inputs(sizes, 1, device="cpu")
    _check_stage1(B, oracle_mod, theta.to(DEV), locals_[0].to(DEV), off, "limit")
    # stage 2, both forms
    _run_stage2(B, oracle_mod, off, st, W, divisor=W)
    _run_stage2(B, oracle_mod, off, st, W, divisor=W, with_acc=True)
    # stage 3 from the oracle's reduced codes
    _, o_c2, o_l2, _ = oracle_mod.reduce([s_[0] for s_ in st], [s_[1] for s_ in st], off, W)
    th_o = theta.numpy().copy()
    m_o = (np.random.default_rng(7).standard_normal(n) * 1e-3).astype(np.float32)
    th_t, m_t = torch.from_numpy(th_o).to(DEV), torch.from_numpy(m_o).to(DEV)
    old_th, old_m = th_o.copy(), m_o.copy()
    B.outer_step(th_t, m_t, 0.7, 0.9, delta_codes=torch.from_numpy(o_c2).to(DEV),
                 delta_lut=torch.from_numpy(o_l2).to(DEV), seg_offsets=off)
    oracle_mod.outer_step(th_o, m_o, 0.7, 0.9, delta_codes=o_c2, delta_luts=o_l2, seg_offsets=off)
    torch.cuda.synchronize()
    so = np.asarray(off)
    g = np.concatenate([o_l2[k][o_c2[so[k]:so[k + 1]]] for k in range(T)]) if n else np.zeros(0, np.float32)
    check_outer(t2n(m_t), m_o, old_m, np.abs(g), "momentum")
    check_outer(t2n(th_t), th_o, old_th, 0.7 * np.abs(g.astype(np.float64) + 0.9 * m_o), "theta")
    # one more group is refused on the host
    with pytest.raises(B.DilocoError):
        B.pseudograd_quantize(theta.to(DEV), locals_[0].to(DEV), off + [n], codes_out=None)


@pytest.mark.parametrize("T", [479, 480, 481, 959, 960, 961, 1920, 1921])
def test_segment_table_sizes_around_the_launch_limits(B, oracle_mod, T):
    """A table of up to 480 offsets goes up in one launch; longer ones as 32-bit lengths, 960 per launch,
    followed by a prefix sum: table sizes on both sides of every limit, stage 1 and the coded outer step."""
    rng = np.random.default_rng(T)
    sizes = rng.integers(0, 300, size=T).tolist()
    sizes[0], sizes[T - 1] = 5000, 4097
    theta, locals_, off = synth.make_inputs(sizes, 1, device=DEV)
    codes, luts, qp = _check_stage1(B, oracle_mod, theta, locals_[0], off, f"T={T}")
    o_codes, o_luts, _, _ = oracle_mod.pseudograd_quantize(t2n(theta), t2n(locals_[0]), off)
    n = off[-1]
    th_o, m_o = t2n(theta).copy(), np.zeros(n, dtype=np.float32)
    th_t, m_t = theta.clone(), torch.zeros(n, dtype=torch.float32, device=DEV)
    B.outer_step(th_t, m_t, 0.7, 0.9, delta_codes=torch.from_numpy(o_codes).to(DEV),
                 delta_lut=torch.from_numpy(o_luts).to(DEV), seg_offsets=off)
    oracle_mod.outer_step(th_o, m_o, 0.7, 0.9, delta_codes=o_codes, delta_luts=o_luts, seg_offsets=off)
    torch.cuda.synchronize()
    check_outer(t2n(m_t), m_o, np.zeros(n, dtype=np.float32), np.abs(m_o), "momentum")
    check_outer(t2n(th_t), th_o, t2n(theta), 0.7 * 1.9 * np.abs(m_o), "theta")


def test_segment_table_with_a_segment_of_more_than_2_pow_32_elements(B, oracle_mod):
    """600 quantisation groups, the first of 2^32 + 5 elements: long tables travel to the device as 32-bit
    segment lengths unless a length does not fit, which is this case (64-bit offsets, several launches).
    The outer step decodes every element through its segment's codebook, so a wrong offset anywhere shows;
    the head of the buffer and everything from just before the first boundary on are compared with the oracle."""
    free, _ = torch.cuda.mem_get_info()
    if free < 50e9:
        pytest.skip(f"needs about 45 GB of free HBM, have {free / 1e9:.0f} GB")
    sizes = [(1 << 32) + 5] + [1000] * 599
    off = synth.offsets_from_sizes(sizes)
    n, T = off[-1], len(sizes)
    say(f"[big segment] n={n} T={T}")
    theta = synth.fill_theta_outer(torch.empty(n, dtype=torch.float32, device=DEV))
    mom = torch.zeros(n, dtype=torch.float32, device=DEV)
    codes = synth.fill_coded_contribution(torch.empty(n, dtype=torch.uint8, device=DEV), 0)
    luts = synth.synthetic_codebooks(T, 0, device=DEV)
    luts += torch.arange(T, device=DEV, dtype=torch.float32)[:, None] * 1e-3      # every group's codebook is distinct
    head, tail = 10_000, off[1] - 5_000
    th_head, th_tail = t2n(theta[:head]), t2n(theta[tail:])
    B.outer_step(theta, mom, 0.7, 0.9, delta_codes=codes, delta_lut=luts, seg_offsets=off)
    torch.cuda.synchronize()
    h_luts = t2n(luts)
    for name, a, b, th_old, seg_local, lut_local in (
            ("head", 0, head, th_head, [0, head], h_luts[:1]),
            ("tail", tail, n, th_tail, [0] + [o - tail for o in off[1:]], h_luts)):
        th_o, m_o = th_old.copy(), np.zeros(b - a, dtype=np.float32)
        oracle_mod.outer_step(th_o, m_o, 0.7, 0.9, delta_codes=t2n(codes[a:b]), delta_luts=np.ascontiguousarray(lut_local),
                              seg_offsets=seg_local)
        check_outer(t2n(mom[a:b]), m_o, np.zeros(b - a, dtype=np.float32), np.abs(m_o), f"momentum ({name})")
        check_outer(t2n(theta[a:b]), th_o, th_old, 0.7 * 1.9 * np.abs(m_o), f"theta ({name})")
    # first step from a zero buffer: m' = g exactly, everywhere in the big segment
    step = 1 << 28
    for a in range(0, off[1], step):
        b = min(a + step, off[1])
        assert torch.equal(mom[a:b], luts[0][codes[a:b].long()])


@pytest.mark.parametrize("W,divisor", [(0, 1), (0, 3), (1, 2), (4, 5), (13, 14), (16, 17)])
@pytest.mark.parametrize("alias", [False, True])
def test_stage2_local_addend(B, oracle_mod, W, divisor, alias):
    sizes = [65_536, 12_289, 150_000]
    theta, off, st = _oracle_peers(oracle_mod, sizes, max(W, 1))
    local = oracle_mod.pseudograd(theta.numpy(), synth.fill_theta_local(
        torch.empty_like(theta), theta, 99).numpy())
    say(f"[stage2] W={W} +local divisor={divisor} alias={alias}")
    _run_stage2(B, oracle_mod, off, st, W, divisor, local=local, with_acc=True, alias=alias)
    if not alias:
        _run_stage2(B, oracle_mod, off, st, W, divisor, local=local, with_acc=False)


def test_stage2_divisor_one_and_retry_with_fewer_peers(B, oracle_mod):
    sizes = [200_000]
    _, off, st = _oracle_peers(oracle_mod, sizes, 6)
    _run_stage2(B, oracle_mod, off, st, 6, divisor=1, with_acc=True)
    _run_stage2(B, oracle_mod, off, st, 6, divisor=6)
    _run_stage2(B, oracle_mod, off, st, 5, divisor=5)        # the retry: same buffers, one peer less


def test_stage2_heavy_tails_w14(B, oracle_mod):
    sizes = [300_000, 50_000]
    _, off, st = _oracle_peers(oracle_mod, sizes, 14, kind="student_t3")
    _run_stage2(B, oracle_mod, off, st, 14, divisor=14, with_acc=True)
    _run_stage2(B, oracle_mod, off, st, 14, divisor=14)


def test_stage2_misaligned_chunk(B, oracle_mod):
    """A ring chunk that starts at an odd element offset: every stream has its own phase."""
    sizes = [123_457]
    n = sizes[0]
    _, off, st = _oracle_peers(oracle_mod, sizes, 3)
    bufs = [torch.zeros(n + 16, dtype=torch.uint8, device=DEV) for _ in range(3)]
    peer_codes = []
    for p in range(3):
        v = bufs[p][p + 1:p + 1 + n]
        v.copy_(torch.from_numpy(st[p][0]))
        peer_codes.append(v)
    peer_luts = [torch.from_numpy(s[1]).to(DEV) for s in st]
    local_np = (np.random.default_rng(5).normal(0, 1e-3, n)).astype(np.float32)
    local_buf = torch.zeros(n + 8, dtype=torch.float32, device=DEV)
    local_v = local_buf[3:3 + n]
    local_v.copy_(torch.from_numpy(local_np))
    out_buf = torch.zeros(n + 16, dtype=torch.uint8, device=DEV)
    codes, luts, qp = B.reduce_chunk(peer_codes, peer_luts, off, 4, local_fp32=local_v, acc_out=local_v,
                                     codes_out=out_buf[5:5 + n])
    torch.cuda.synchronize()
    o_acc, o_codes, o_luts, o_qp = oracle_mod.reduce([s[0] for s in st], [s[1] for s in st], off, 4,
                                                     local_fp32=local_np)
    check_qparams(B.qparams_to_numpy(qp), o_qp)
    check_codes(t2n(codes), o_codes, o_acc, off, o_qp)
    check_luts(t2n(luts), o_luts, o_codes, off, o_qp)
    assert np.array_equal(t2n(local_v), o_acc)
    assert int(out_buf[:5].sum()) == 0 and int(out_buf[5 + n:].sum()) == 0
    assert float(local_buf[:3].abs().sum()) == 0 and float(local_buf[3 + n:].abs().sum()) == 0


# ---------------------------------------------------------------------------------------------
# stage 3
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("coded", [False, True, "fp32 with workspace"])
@pytest.mark.parametrize("out", [None, torch.float32, torch.bfloat16])
def test_stage3_outer_step(B, oracle_mod, coded, out):
    # the fp32 form walks static shares without a workspace and claims chunks with one
    ws = B.new_workspace(1, DEV) if coded == "fp32 with workspace" else None
    coded = coded is True
    sizes = [100_000, 4097, 1, 250_000]
    n = sum(sizes)
    off = synth.offsets_from_sizes(sizes)
    rng = np.random.default_rng(11)
    theta = rng.normal(0, 0.02, n).astype(np.float32)
    mom = rng.normal(0, 2e-3, n).astype(np.float32)
    g = (rng.normal(0, 1e-3, n)).astype(np.float32)
    o_codes, o_luts, _ = oracle_mod.quantize_segments(g, off)
    th_t, m_t = torch.from_numpy(theta).to(DEV), torch.from_numpy(mom).to(DEV)
    out_t = torch.empty(n, dtype=out, device=DEV) if out is not None else None
    th_o, m_o = theta.copy(), mom.copy()
    lr, beta = 0.7, 0.9
    for step in range(2):
        old_th, old_m = th_o.copy(), m_o.copy()
        if coded:
            B.outer_step(th_t, m_t, lr, beta, delta_codes=torch.from_numpy(o_codes).to(DEV),
                         delta_lut=torch.from_numpy(o_luts).to(DEV), seg_offsets=off, theta_local_out=out_t)
            o_out = oracle_mod.outer_step(th_o, m_o, lr, beta, delta_codes=o_codes, delta_luts=o_luts,
                                          seg_offsets=off,
                                          local_out_dtype={None: None, torch.float32: "fp32",
                                                           torch.bfloat16: "bf16"}[out])
            gg = np.concatenate([o_luts[s][o_codes[off[s]:off[s + 1]]] for s in range(len(sizes))])
        else:
            B.outer_step(th_t, m_t, lr, beta, delta_fp32=torch.from_numpy(g).to(DEV), theta_local_out=out_t,
                         workspace=ws)
            o_out = oracle_mod.outer_step(th_o, m_o, lr, beta, delta_fp32=g,
                                          local_out_dtype={None: None, torch.float32: "fp32",
                                                           torch.bfloat16: "bf16"}[out])
            gg = g
        torch.cuda.synchronize()
        step_scale = lr * np.abs(gg.astype(np.float64) + beta * m_o)
        check_outer(t2n(m_t), m_o, old_m, np.abs(gg), "momentum")
        check_outer(t2n(th_t), th_o, old_th, step_scale, "theta")
        if out is torch.float32:
            assert torch.equal(out_t, th_t)
        if out is torch.bfloat16:
            assert torch.equal(out_t, th_t.to(torch.bfloat16))          # rounding of the GPU's own theta
            ob = o_out.view(np.uint16).astype(np.int64)
            gb = bf16_bits(out_t).astype(np.int64)
            assert np.abs(gb - ob).max() <= 1                           # at most one bf16 step from the oracle's


# ---------------------------------------------------------------------------------------------
# chained: GPU stage into GPU stage, configuration 0 end to end
# ---------------------------------------------------------------------------------------------

def test_chained_config0(B, oracle_mod):
    W = synth.config_peers(0)
    theta, locals_, off = synth.make_inputs(synth.config_segment_sizes(0), W, device=DEV)
    n = theta.numel()
    g1 = [B.pseudograd_quantize(theta, l, off) for l in locals_]
    codes2, luts2, qp2 = B.reduce_chunk([g[0] for g in g1], [g[1] for g in g1], off, W)
    mom = torch.zeros(n, dtype=torch.float32, device=DEV)
    theta_new = theta.clone()
    B.outer_step(theta_new, mom, 0.7, 0.9, delta_codes=codes2, delta_lut=luts2, seg_offsets=off)
    torch.cuda.synchronize()

    th_np = t2n(theta)
    o1 = [oracle_mod.pseudograd_quantize(th_np, t2n(l), off) for l in locals_]
    flips1 = 0
    for p in range(W):
        check_qparams(B.qparams_to_numpy(g1[p][2]), o1[p][2])
        flips1 += check_codes(t2n(g1[p][0]), o1[p][0], o1[p][3], off, o1[p][2])
    o_acc, o_c2, o_l2, o_q2 = oracle_mod.reduce([o[0] for o in o1], [o[1] for o in o1], off, W)
    check_qparams(B.qparams_to_numpy(qp2), o_q2)
    # with no flip upstream the GPU's stage 2 saw the oracle's inputs bit for bit and the stage's own
    # bar applies; a flipped upstream code changes that element's sum and can move the fp32 range by
    # an ulp, which shifts about 1e-5 of the codes by one bucket
    flips = check_codes(t2n(codes2), o_c2, o_acc, off, o_q2, budget=1e-6 if flips1 == 0 else 1e-5)
    th_o, m_o = th_np.copy(), np.zeros(n, dtype=np.float32)
    oracle_mod.outer_step(th_o, m_o, 0.7, 0.9, delta_codes=o_c2, delta_luts=o_l2, seg_offsets=off)
    g_dec = o_l2[0][o_c2]
    w2 = 12 * o_q2["std"][0] / 256
    diff = np.abs(t2n(theta_new).astype(np.float64) - th_o)
    same = t2n(codes2) == o_c2
    scale = np.maximum(np.abs(th_o), 0.7 * 1.9 * np.abs(g_dec))
    assert np.all(diff[same] <= 1e-5 * scale[same])
    assert np.all(diff[~same] <= 0.7 * 1.9 * 1.01 * w2 + 1e-5 * scale[~same])   # a flipped code moves by one bucket
    say(f"[chained] config0: stage-1 flips={flips1} stage-2 flips={flips}")


# ---------------------------------------------------------------------------------------------
# data-dependent conditions are reported per segment, never as a fault
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("bad", [float("nan"), float("inf"), -float("inf")])
def test_nonfinite_input_is_flagged_not_fatal(B, oracle_mod, bad):
    sizes = [20_000, 5_000, 70_000]
    theta, locals_, off = synth.make_inputs(sizes, 1, device=DEV)
    local = locals_[0]
    local[off[1] + 17] = bad                                   # poisons segment 1 only
    codes, luts, qp = B.pseudograd_quantize(theta, local, off)
    torch.cuda.synchronize()
    g_qp = B.qparams_to_numpy(qp)
    o_codes, o_luts, o_qp, o_d = oracle_mod.pseudograd_quantize(t2n(theta), t2n(local), off)
    assert list(g_qp["status"]) == list(o_qp["status"])
    assert g_qp["status"][1] & B.STATUS_NONFINITE and g_qp["status"][0] == 0 and g_qp["status"][2] == 0
    # the clean segments are unaffected and still match the oracle exactly
    for s in (0, 2):
        a, b = off[s], off[s + 1]
        check_qparams(g_qp[s:s + 1], o_qp[s:s + 1])
        check_codes(t2n(codes[a:b]), o_codes[a:b], o_d[a:b], [0, b - a], o_qp[s:s + 1])
        check_luts(t2n(luts[s]), o_luts[s], o_codes[a:b], [0, b - a], o_qp[s:s + 1])
    # a later call on clean data is unaffected (no state is kept)
    local[off[1] + 17] = theta[off[1] + 17]
    _check_stage1(B, oracle_mod, theta, local, off, "after non-finite")


@pytest.mark.parametrize("materialise", [False, True])
def test_outputs_written_over_consumed_inputs(B, oracle_mod, materialise):
    """codes_out over one contribution's codes, and the fp32 hand-back over the fp32 average."""
    W = 4
    sizes = [100_000, 4096, 3, 77_777, 0, 40_001]
    theta, off, st = _oracle_peers(oracle_mod, sizes, W)
    n = off[-1]
    peer_codes = [torch.from_numpy(s_[0]).to(DEV) for s_ in st]
    peer_luts = [torch.from_numpy(s_[1]).to(DEV) for s_ in st]
    acc_t = torch.empty(n, dtype=torch.float32, device=DEV)
    codes, luts, qp = B.reduce_chunk(peer_codes, peer_luts, off, W, acc_out=acc_t if materialise else None,
                                     codes_out=peer_codes[2])
    torch.cuda.synchronize()
    assert codes.data_ptr() == peer_codes[2].data_ptr()
    o_acc, o_codes, o_luts, o_qp = oracle_mod.reduce([s_[0] for s_ in st], [s_[1] for s_ in st], off, W)
    check_qparams(B.qparams_to_numpy(qp), o_qp)
    check_codes(t2n(codes), o_codes, o_acc, off, o_qp)
    check_luts(t2n(luts), o_luts, o_codes, off, o_qp)
    for p in (0, 1, 3):
        assert np.array_equal(t2n(peer_codes[p]), st[p][0])          # the other contributions are untouched
    # outer step from the oracle's fp32 average, new weights written over that average
    delta_t = torch.from_numpy(o_acc).to(DEV)
    th_o = theta.numpy().copy()
    m_o = (np.random.default_rng(3).standard_normal(n) * 1e-3).astype(np.float32)
    th_t, m_t = torch.from_numpy(th_o).to(DEV), torch.from_numpy(m_o).to(DEV)
    old_th, old_m = th_o.copy(), m_o.copy()
    B.outer_step(th_t, m_t, 0.7, 0.9, delta_fp32=delta_t, theta_local_out=delta_t)
    oracle_mod.outer_step(th_o, m_o, 0.7, 0.9, delta_fp32=o_acc)
    torch.cuda.synchronize()
    check_outer(t2n(m_t), m_o, old_m, np.abs(o_acc), "momentum")
    check_outer(t2n(th_t), th_o, old_th, 0.7 * np.abs(o_acc.astype(np.float64) + 0.9 * m_o), "theta")
    assert torch.equal(delta_t, th_t)


@pytest.mark.parametrize("bad", [float("nan"), float("inf")])
@pytest.mark.parametrize("materialise", [False, True])
def test_nonfinite_codebook_entry_in_the_reduce(B, oracle_mod, bad, materialise):
    """A contribution whose codebook carries a NaN / Inf (its sender's tensor was not finite): the
    reduce flags that tensor and leaves the others exact; so do the stored accumulation and the outer
    step taken from the result."""
    W = 3
    sizes = [20_000, 5_000, 70_000]
    theta, off, st = _oracle_peers(oracle_mod, sizes, W)
    luts1 = st[1][1].copy()
    busiest = int(np.bincount(st[1][0][off[1]:off[2]], minlength=256).argmax())
    luts1[1][busiest] = bad                                          # peer 1, tensor 1, its fullest bucket
    st = [st[0], (st[1][0], luts1, st[1][2], st[1][3]), st[2]]
    n = off[-1]
    peer_codes = [torch.from_numpy(s_[0]).to(DEV) for s_ in st]
    peer_luts = [torch.from_numpy(s_[1]).to(DEV) for s_ in st]
    acc_t = torch.empty(n, dtype=torch.float32, device=DEV) if materialise else None
    codes, luts, qp = B.reduce_chunk(peer_codes, peer_luts, off, W, acc_out=acc_t)
    torch.cuda.synchronize()
    o_acc, o_codes, o_luts, o_qp = oracle_mod.reduce([s_[0] for s_ in st], [s_[1] for s_ in st], off, W)
    g_qp = B.qparams_to_numpy(qp)
    assert list(g_qp["status"]) == list(o_qp["status"])
    assert g_qp["status"][1] & B.STATUS_NONFINITE and g_qp["status"][0] == 0 and g_qp["status"][2] == 0
    for s in (0, 2):
        a, b = off[s], off[s + 1]
        check_qparams(g_qp[s:s + 1], o_qp[s:s + 1])
        check_codes(t2n(codes[a:b]), o_codes[a:b], o_acc[a:b], [0, b - a], o_qp[s:s + 1])
        check_luts(t2n(luts[s]), o_luts[s], o_codes[a:b], [0, b - a], o_qp[s:s + 1])
    if materialise:
        got = t2n(acc_t)
        assert np.array_equal(got, o_acc, equal_nan=True)            # the same fp32 operations, NaN where the oracle has NaN
    # the outer step from the oracle's result: finite tensors move exactly as the oracle's do
    th_o, m_o = theta.numpy().copy(), np.zeros(n, dtype=np.float32)
    th_t, m_t = torch.from_numpy(th_o).to(DEV), torch.from_numpy(m_o).to(DEV)
    B.outer_step(th_t, m_t, 0.7, 0.9, delta_codes=torch.from_numpy(o_codes).to(DEV),
                 delta_lut=torch.from_numpy(o_luts).to(DEV), seg_offsets=off)
    oracle_mod.outer_step(th_o, m_o, 0.7, 0.9, delta_codes=o_codes, delta_luts=o_luts, seg_offsets=off)
    torch.cuda.synchronize()
    for s in (0, 2):
        a, b = off[s], off[s + 1]
        g = o_luts[s][o_codes[a:b]]
        check_outer(t2n(m_t[a:b]), m_o[a:b], np.zeros(b - a, dtype=np.float32), np.abs(g), "momentum")
        check_outer(t2n(th_t[a:b]), th_o[a:b], theta.numpy()[a:b], 0.7 * 1.9 * np.abs(g), "theta")
    a, b = off[1], off[2]
    assert np.array_equal(np.isfinite(t2n(m_t[a:b])), np.isfinite(m_o[a:b]))


def test_large_mean_small_spread(B, oracle_mod):
    """Statistics about a pivot: a pseudo-gradient whose mean is 10^4 standard deviations."""
    sizes = [300_000, 4096]
    theta, locals_, off = synth.make_inputs(sizes, 1, device=DEV)
    local = locals_[0] - 10.0                                  # d = theta - local has mean ~ +10, std ~ 2e-3
    _check_stage1(B, oracle_mod, theta, local, off, "large mean")


def test_values_on_bucket_edges(B, oracle_mod):
    """A tensor with a few thousand values placed on the bucket edges themselves: lo + k / inv_w for every k, and
    the fp32 neighbours just below and above.  The edges depend on the statistics of the tensor that holds
    them, so the values are re-placed a few times until they stop moving.  On an edge the bucket is decided by
    the rounding of two fp32 operations; both sides must take the same one, element by element."""
    rng = np.random.default_rng(4)
    n = 300_000
    x = rng.normal(0.0, 1e-3, n).astype(np.float32)
    slots = rng.choice(n, size=257 * 9, replace=False).reshape(257, 9)
    for _ in range(8):
        _, _, q = oracle_mod.quantize(x)
        lo, w = np.float64(q["lo"]), 1.0 / np.float64(q["inv_w"])
        for k in range(257):
            e = np.float32(lo + k * w)
            below, above = np.nextafter(e, np.float32(-1)), np.nextafter(e, np.float32(1))
            x[slots[k]] = [e, below, above] * 3
    o_codes, o_lut, o_q = oracle_mod.quantize(x)
    t = ((x[slots.ravel()] - np.float32(o_q["lo"])) * np.float32(o_q["inv_w"])).astype(np.float64)
    on_edge = np.abs(t - np.round(t)) < 1e-3
    assert on_edge.mean() > 0.9, on_edge.mean()          # the placement converged: the values sit on the final edges
    theta = torch.zeros(n, dtype=torch.float32, device=DEV)
    local = torch.from_numpy(-x).to(DEV)                  # theta - local = x exactly
    codes, luts, qp = B.pseudograd_quantize(theta, local, [0, n])
    torch.cuda.synchronize()
    g_q = B.qparams_to_numpy(qp)
    check_qparams(g_q, np.array([o_q]), require_exact=1.0)
    assert np.array_equal(t2n(codes), o_codes)            # not one flip, on the edges or anywhere else
    check_luts(t2n(luts), o_lut.reshape(1, 256), o_codes, [0, n], np.array([o_q]))
    both_sides = len(set(o_codes[slots[100]].tolist()))
    say(f"[edges] {int(on_edge.sum())} of {on_edge.size} planted values within 1e-3 of an edge; "
        f"the nine values around edge 100 fall into {both_sides} buckets")
    assert both_sides == 2


def test_few_distinct_values_reconstruct(B, oracle_mod):
    """A tensor with 16 well separated levels: every bucket holds one distinct value.  The oracle
    decodes it bit-exactly; the library's fixed-point bucket sums round each offset to 2^-22 of a
    bucket width, so it decodes to within that (far inside the 1e-6 codebook tolerance)."""
    n = 160_000
    levels = ((torch.arange(16, device=DEV, dtype=torch.float32) - 7.5) * 1.33e-4)
    d = levels[torch.randint(0, 16, (n,), device=DEV, generator=torch.Generator(device=DEV).manual_seed(5))]
    theta = torch.zeros(n, dtype=torch.float32, device=DEV)
    local = -d                                                 # theta - local = d exactly
    codes, luts, qp = B.pseudograd_quantize(theta, local, [0, n])
    torch.cuda.synchronize()
    o_codes, o_luts, o_qp, o_d = oracle_mod.pseudograd_quantize(t2n(theta), t2n(local), [0, n])
    assert np.array_equal(o_luts[0][o_codes], t2n(d))          # the oracle is exact here
    assert np.array_equal(t2n(codes), o_codes)
    w = 12.0 * float(o_qp["std"][0]) / 256.0
    dec = t2n(luts)[0][t2n(codes)]
    assert np.abs(dec.astype(np.float64) - t2n(d)).max() <= 2.0 ** -21 * w
    check_luts(t2n(luts), o_luts, o_codes, [0, n], o_qp)


# ---------------------------------------------------------------------------------------------
# stage 1 with the codes held back for the write window (the path large buffers take), forced at
# small sizes through the library's instrumentation call: ragged segments, heads and tails, a
# misaligned view, bf16, and windows so short or so long that either every flush is forced by a full
# staging area or nearly every iteration falls inside a window
# ---------------------------------------------------------------------------------------------

@pytest.fixture
def builtin_write_phase_after(B):
    yield
    B.tune_write_phase(-1)


@pytest.mark.parametrize("timing", [(40, 10), (100000, 1), (10, 9)])
@pytest.mark.parametrize("local_dtype", [torch.float32, torch.bfloat16])
def test_stage1_staged_code_writes(B, oracle_mod, builtin_write_phase_after, timing, local_dtype):
    B.tune_write_phase(*timing)
    sizes = synth.ragged_sizes(1_500_000) + [4096 * 9 + 5, 130, 4096 * 33]
    theta, locals_, off = synth.make_inputs(sizes, 1, device=DEV, local_dtype=local_dtype)
    _check_stage1(B, oracle_mod, theta, locals_[0], off, f"staged writes, timing {timing}")
    # a view that starts 3 elements into its buffer, output codes 5 bytes into theirs
    n = theta.numel()
    th_buf = torch.zeros(n + 8, dtype=torch.float32, device=DEV)
    lo_buf = torch.zeros(n + 8, dtype=local_dtype, device=DEV)
    co_buf = torch.zeros(n + 16, dtype=torch.uint8, device=DEV)
    th_buf[3:3 + n] = theta
    lo_buf[3:3 + n] = locals_[0]
    codes, luts, qp = B.pseudograd_quantize(th_buf[3:3 + n], lo_buf[3:3 + n], off, codes_out=co_buf[5:5 + n])
    B.tune_write_phase(0)
    ref = B.pseudograd_quantize(theta, locals_[0], off)
    torch.cuda.synchronize()
    assert torch.equal(codes, ref[0]) and torch.allclose(luts, ref[1], rtol=1e-6, atol=0)
    assert int(co_buf[:5].sum()) == 0 and int(co_buf[5 + n:].sum()) == 0          # nothing written outside
