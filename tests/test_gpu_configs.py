"""The five benchmark configurations against the oracle (needs an MI355X).

Configurations 0 and 1 run at their full size, element by element.  Configuration 2 (the one
bench.py times: 10,211,381,248 elements, 381 tensors, W = 4) runs at full size in the benchmark's
launch configuration and is checked on sampled tensors the oracle can process whole, plus
properties that hold at any size; so are the call variants bench.py --extras times (bf16
theta_local, stored accumulation, outer step from fp32 and with the new weights handed back).  Configurations 3 and 4 keep their structure (14 heavy-tailed
coded peers with the accumulation stored over theta_local; 14 ring chunks of a size that is not a
multiple of anything, 13 coded peers + un-quantised local addend, bf16 theta_local) on the first
attention block's tensors, a size the oracle finishes in seconds, and also run at full size: the
reduce at W = 14 on all 381 tensors, checked on sampled tensors, and one whole ring chunk of
729,384,375 elements at its odd offset inside full-size buffers.
"""
import sys
import time

import numpy as np
import pytest
import torch

from paper_2412_01152_amd import synth
from parity_utils import (bf16_bits, check_codes, check_luts, check_outer, check_qparams, t2n)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
LR, BETA = 0.7, 0.9


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()
    from conftest import progress
    progress(msg)


@pytest.fixture(scope="module")
def B():
    from paper_2412_01152_amd import binding
    binding.load()
    assert torch.cuda.is_available()
    return binding


@pytest.fixture(autouse=True)
def _free_gpu():
    yield
    torch.cuda.empty_cache()


def _decode(codes, luts, off):
    return np.concatenate([luts[s][codes[off[s]:off[s + 1]]] for s in range(len(off) - 1)])


def _full_chain(B, oracle_mod, sizes, W, kind, local_dtype=torch.float32, materialise=False):
    """Stage-isolated run of the three stages on a workload small enough for the oracle."""
    theta, locals_, off = synth.make_inputs(sizes, W, kind=kind, device=DEV, local_dtype=local_dtype)
    n = theta.numel()
    th = t2n(theta)
    t0 = time.time()
    o1 = []
    for p, l in enumerate(locals_):
        if local_dtype == torch.bfloat16:
            o1.append(oracle_mod.pseudograd_quantize(th, bf16_bits(l), off, local_is_bf16=True))
        else:
            o1.append(oracle_mod.pseudograd_quantize(th, t2n(l), off))
    say(f"  oracle stage 1 x{W}: {time.time() - t0:.1f}s")
    flips1 = 0
    for p, l in enumerate(locals_):
        c, lu, qp = B.pseudograd_quantize(theta, l, off)
        torch.cuda.synchronize()
        check_qparams(B.qparams_to_numpy(qp), o1[p][2])
        flips1 += check_codes(t2n(c), o1[p][0], o1[p][3], off, o1[p][2])
        check_luts(t2n(lu), o1[p][1], o1[p][0], off, o1[p][2])
    pc = [torch.from_numpy(o[0]).to(DEV) for o in o1]
    pl = [torch.from_numpy(o[1]).to(DEV) for o in o1]
    acc_t = locals_[0].float() if materialise else None      # stored over (a copy of) theta_local
    if materialise and local_dtype == torch.float32:
        acc_t = locals_[0]
    c2, l2, q2 = B.reduce_chunk(pc, pl, off, W, acc_out=acc_t)
    torch.cuda.synchronize()
    t0 = time.time()
    o_acc, o_c2, o_l2, o_q2 = oracle_mod.reduce([o[0] for o in o1], [o[1] for o in o1], off, W)
    say(f"  oracle stage 2: {time.time() - t0:.1f}s")
    check_qparams(B.qparams_to_numpy(q2), o_q2)
    flips2 = check_codes(t2n(c2), o_c2, o_acc, off, o_q2)
    check_luts(t2n(l2), o_l2, o_c2, off, o_q2)
    if materialise:
        assert np.array_equal(t2n(acc_t), o_acc)
    mom = torch.zeros(n, dtype=torch.float32, device=DEV)
    th_g = theta.clone()
    B.outer_step(th_g, mom, LR, BETA, delta_codes=torch.from_numpy(o_c2).to(DEV),
                 delta_lut=torch.from_numpy(o_l2).to(DEV), seg_offsets=off)
    torch.cuda.synchronize()
    th_o, m_o = th.copy(), np.zeros(n, dtype=np.float32)
    oracle_mod.outer_step(th_o, m_o, LR, BETA, delta_codes=o_c2, delta_luts=o_l2, seg_offsets=off)
    check_outer(t2n(mom), m_o, np.zeros(n, dtype=np.float32), np.abs(m_o), "momentum")
    check_outer(t2n(th_g), th_o, th, LR * (1 + BETA) * np.abs(m_o), "theta")
    say(f"  N={n} T={len(sizes)} W={W}: stage-1 flips={flips1} stage-2 flips={flips2}")


def test_config0_full(B, oracle_mod):
    _full_chain(B, oracle_mod, synth.config_segment_sizes(0), synth.config_peers(0), "mixture")


def test_config1_full_layer_w8(B, oracle_mod):
    _full_chain(B, oracle_mod, synth.config_segment_sizes(1), synth.config_peers(1), "mixture")


def _attention_block_sizes():
    s = synth.layer_tensor_sizes()
    return [s[0], s[1], s[2], s[3], s[7], s[8]]          # wq, wk, wv, wo and the two norm vectors


def test_config3_structure_w14_heavy_tails_accumulate_over_theta_local(B, oracle_mod):
    _full_chain(B, oracle_mod, _attention_block_sizes(), 14, "student_t3", materialise=True)


def test_config4_structure_ring_chunks_bf16(B, oracle_mod):
    """14 contiguous chunks (element count not divisible by 14: chunk starts are odd offsets),
    each its own quantisation group; chunk owner adds its un-quantised fp32 data to 13 coded
    contributions and divides by 14; theta_local arrives as bf16."""
    sizes = _attention_block_sizes()
    n = sum(sizes) + 5                                    # make it indivisible by 14
    sizes = sizes + [5]
    chunk_sizes = synth.ring_chunk_sizes(n, 14)
    assert n % 14 != 0 and chunk_sizes[0] % 2 == 1
    W = 13
    theta, locals_, _ = synth.make_inputs([n], W + 1, device=DEV, local_dtype=torch.bfloat16)
    th = t2n(theta)
    chunk_off = synth.offsets_from_sizes(chunk_sizes)
    # every peer quantises chunk by chunk (one group per chunk): oracle first
    t0 = time.time()
    o1 = [oracle_mod.pseudograd_quantize(th, bf16_bits(l), chunk_off, local_is_bf16=True) for l in locals_]
    say(f"  oracle stage 1 x{W + 1} (bf16): {time.time() - t0:.1f}s")
    g0 = B.pseudograd_quantize(theta, locals_[0], chunk_off)
    torch.cuda.synchronize()
    check_qparams(B.qparams_to_numpy(g0[2]), o1[0][2])
    check_codes(t2n(g0[0]), o1[0][0], o1[0][3], chunk_off, o1[0][2])
    check_luts(t2n(g0[1]), o1[0][1], o1[0][0], chunk_off, o1[0][2])
    # the owner's own pseudo-gradient stays fp32 (peer index W), the other 13 arrive coded
    local_fp32 = torch.from_numpy(o1[W][3]).to(DEV)
    pcs = [torch.from_numpy(o[0]).to(DEV) for o in o1[:W]]
    pls = [torch.from_numpy(o[1]).to(DEV) for o in o1[:W]]
    codes_out = torch.empty(n, dtype=torch.uint8, device=DEV)
    luts_out = torch.empty((14, 256), dtype=torch.float32, device=DEV)
    ws = B.new_workspace(1, DEV)
    total_flips = 0
    o_c2_all = np.empty(n, dtype=np.uint8)
    o_l2_all = np.empty((14, 256), dtype=np.float32)
    for c in range(14):
        a, b = chunk_off[c], chunk_off[c + 1]
        loc_v = local_fp32[a:b]
        c2, l2, q2 = B.reduce_chunk([pc[a:b] for pc in pcs], [pl[c:c + 1] for pl in pls], [0, b - a], 14,
                                    local_fp32=loc_v, acc_out=loc_v, codes_out=codes_out[a:b],
                                    lut_out=luts_out[c:c + 1], workspace=ws)
        torch.cuda.synchronize()
        o_acc, o_c2, o_l2, o_q2 = oracle_mod.reduce(
            [np.ascontiguousarray(o[0][a:b]) for o in o1[:W]], [o[1][c:c + 1] for o in o1[:W]], [0, b - a], 14,
            local_fp32=np.ascontiguousarray(o1[W][3][a:b]))
        check_qparams(B.qparams_to_numpy(q2), o_q2)
        total_flips += check_codes(t2n(c2), o_c2, o_acc, [0, b - a], o_q2)
        check_luts(t2n(l2), o_l2, o_c2, [0, b - a], o_q2)
        assert np.array_equal(t2n(loc_v), o_acc)
        o_c2_all[a:b] = o_c2
        o_l2_all[c] = o_l2[0]
    # outer step from the requantised chunks (the oracle's, so the stage is checked in isolation),
    # new worker weights handed back as bf16
    codes_out.copy_(torch.from_numpy(o_c2_all))
    luts_out.copy_(torch.from_numpy(o_l2_all))
    mom = torch.zeros(n, dtype=torch.float32, device=DEV)
    th_g = theta.clone()
    handback = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    B.outer_step(th_g, mom, LR, BETA, delta_codes=codes_out, delta_lut=luts_out, seg_offsets=chunk_off,
                 theta_local_out=handback)
    torch.cuda.synchronize()
    th_o, m_o = th.copy(), np.zeros(n, dtype=np.float32)
    oracle_mod.outer_step(th_o, m_o, LR, BETA, delta_codes=o_c2_all, delta_luts=o_l2_all, seg_offsets=chunk_off)
    check_outer(t2n(th_g), th_o, th, LR * (1 + BETA) * np.abs(m_o), "theta")
    assert torch.equal(handback, th_g.to(torch.bfloat16))
    say(f"  14 chunks of {chunk_sizes[0]} (last {chunk_sizes[-1]}): flips={total_flips}")


# ---------------------------------------------------------------------------------------------
# configuration 2 at full size, in bench.py's launch configuration
# ---------------------------------------------------------------------------------------------

def test_config2_fullsize_sampled_tensors(B, oracle_mod):
    sizes = synth.config_segment_sizes(2)
    off = synth.offsets_from_sizes(sizes)
    N, T, W = off[-1], len(sizes), 4
    free, _ = torch.cuda.mem_get_info()
    if free < 190e9:
        pytest.skip(f"needs about 185 GB of free HBM, have {free / 1e9:.0f} GB")
    # sampled tensors: the embedding and the output head (525M elements each: the largest counts and the
    # longest residency of the blocks in one segment), final norm (4,096), layer 7 wk (4.2M), layer 41 wq
    # (16.8M), layer 20 ffn_norm, layer 3 w_down (58.7M)
    sample = [0, T - 1, T - 2, 1 + 9 * 7 + 1, 1 + 9 * 41 + 0, 1 + 9 * 20 + 8, 1 + 9 * 3 + 6]
    say(f"[config2] N={N} T={T}; sampled tensors {sample} sizes {[sizes[s] for s in sample]}")
    theta = synth.fill_theta_outer(torch.empty(N, dtype=torch.float32, device=DEV))
    local = torch.empty(N, dtype=torch.float32, device=DEV)
    mom = torch.zeros(N, dtype=torch.float32, device=DEV)
    peer_codes = [torch.empty(N, dtype=torch.uint8, device=DEV) for _ in range(W)]
    peer_luts = [torch.empty((T, 256), dtype=torch.float32, device=DEV) for _ in range(W)]
    qp = B.new_qparams(T, DEV)
    ws = B.new_workspace(T, DEV)
    th_s = {s: t2n(theta[off[s]:off[s + 1]]) for s in sample}
    o1 = {s: [] for s in sample}
    flips = 0
    for p in list(range(1, W)) + [0]:
        synth.fill_theta_local(local, theta, p, "mixture")
        B.pseudograd_quantize(theta, local, off, codes_out=peer_codes[p], lut_out=peer_luts[p],
                              qparams_out=qp, workspace=ws)
        torch.cuda.synchronize()
        g_qp = B.qparams_to_numpy(qp)
        assert int(g_qp["n"].sum()) == N and np.all(g_qp["status"] == 0)
        for s in sample:
            a, b = off[s], off[s + 1]
            o = oracle_mod.pseudograd_quantize(th_s[s], t2n(local[a:b]), [0, b - a])
            check_qparams(g_qp[s:s + 1], o[2])
            flips += check_codes(t2n(peer_codes[p][a:b]), o[0], o[3], [0, b - a], o[2])
            check_luts(t2n(peer_luts[p][s]), o[1], o[0], [0, b - a], o[2])
            o1[s].append((p, o))
            # hand the oracle's codes to the next stage (stage-isolated)
            peer_codes[p][a:b].copy_(torch.from_numpy(o[0]))
            peer_luts[p][s].copy_(torch.from_numpy(o[1][0]))
        say(f"[config2] peer {p}: stage 1 checked on {len(sample)} tensors")
    # any-size property on a tensor outside the sample (layer 0 w_gate, 58.7M elements) of peer 0: the
    # codebook is the bucket mean, so decoding preserves the tensor's sum
    a, b = off[5], off[6]
    d64 = (theta[a:b].double() - local[a:b].double())
    dec = peer_luts[0][5][peer_codes[0][a:b].long()].double()
    assert abs(float(dec.sum() - d64.sum())) <= 2 ** -22 * float(d64.abs().sum())
    assert float((dec - d64).abs().max()) < 1.0                      # finite, no wild decode
    del d64, dec
    torch.cuda.empty_cache()

    codes2 = torch.empty(N, dtype=torch.uint8, device=DEV)
    lut2 = torch.empty((T, 256), dtype=torch.float32, device=DEV)
    B.reduce_chunk(peer_codes, peer_luts, off, W, codes_out=codes2, lut_out=lut2, qparams_out=qp, workspace=ws)
    torch.cuda.synchronize()
    g_qp = B.qparams_to_numpy(qp)
    assert int(g_qp["n"].sum()) == N and np.all(g_qp["status"] == 0)
    o2 = {}
    for s in sample:
        a, b = off[s], off[s + 1]
        by_peer = dict(o1[s])
        o_acc, o_c2, o_l2, o_q2 = oracle_mod.reduce([by_peer[p][0] for p in range(W)],
                                                    [by_peer[p][1] for p in range(W)], [0, b - a], W)
        check_qparams(g_qp[s:s + 1], o_q2)
        flips += check_codes(t2n(codes2[a:b]), o_c2, o_acc, [0, b - a], o_q2)
        check_luts(t2n(lut2[s]), o_l2, o_c2, [0, b - a], o_q2)
        o2[s] = (o_c2, o_l2)
        codes2[a:b].copy_(torch.from_numpy(o_c2))
        lut2[s].copy_(torch.from_numpy(o_l2[0]))
    say("[config2] stage 2 checked")
    # requantisation keeps the sum of the fp32 average it encodes (any size): recompute the average
    # of layer 0's w_gate with torch and compare sums
    a, b = off[5], off[6]
    acc = torch.zeros(b - a, dtype=torch.float32, device=DEV)
    for p in range(W):
        acc += peer_luts[p][5][peer_codes[p][a:b].long()]
    acc *= 0.25
    dec2 = lut2[5][codes2[a:b].long()]
    assert abs(float(dec2.double().sum() - acc.double().sum())) <= 2 ** -22 * float(acc.double().abs().sum())
    del acc, dec2
    torch.cuda.empty_cache()

    B.outer_step(theta, mom, LR, BETA, delta_codes=codes2, delta_lut=lut2, seg_offsets=off, workspace=ws)
    torch.cuda.synchronize()
    for s in sample:
        a, b = off[s], off[s + 1]
        th_o, m_o = th_s[s].copy(), np.zeros(b - a, dtype=np.float32)
        oracle_mod.outer_step(th_o, m_o, LR, BETA, delta_codes=o2[s][0], delta_luts=o2[s][1], seg_offsets=[0, b - a])
        check_outer(t2n(mom[a:b]), m_o, np.zeros(b - a, dtype=np.float32), np.abs(m_o), "momentum")
        check_outer(t2n(theta[a:b]), th_o, th_s[s], LR * (1 + BETA) * np.abs(m_o), "theta")
    # first step from a zero buffer: m' = g everywhere, theta moved by lr (1 + beta) g (any size)
    a, b = off[5], off[6]
    g = lut2[5][codes2[a:b].long()]
    assert torch.equal(mom[a:b], g)
    say(f"[config2] stage 3 checked; total one-bucket flips on sampled tensors: {flips}")


# ---------------------------------------------------------------------------------------------
# configuration 2 at full size, EVERY element of all three stages against the oracle: stage 1 on this
# worker's 10,211,381,248 pseudo-gradient values, the reduce of its codes with three more coded
# contributions, the outer step from the oracle's requantised result.  (The other three contributions
# are synthetic codes and codebooks, so that the host runs stage 1 once, not four times.)
# ---------------------------------------------------------------------------------------------

def test_config2_fullsize_every_element_against_the_oracle(B, oracle_mod):
    import psutil
    sizes = synth.config_segment_sizes(2)
    off = synth.offsets_from_sizes(sizes)
    N, T, W = off[-1], len(sizes), 4
    free, _ = torch.cuda.mem_get_info()
    if free < 190e9:
        pytest.skip(f"needs about 185 GB of free HBM, have {free / 1e9:.0f} GB")
    if psutil.virtual_memory().available < 175e9:
        pytest.skip(f"needs about 140 GB of host memory, {psutil.virtual_memory().available / 1e9:.0f} GB available")
    t_all = time.time()
    theta = synth.fill_theta_outer(torch.empty(N, dtype=torch.float32, device=DEV))
    local = synth.fill_theta_local(torch.empty(N, dtype=torch.float32, device=DEV), theta, 0, "mixture")
    ws = B.new_workspace(T, DEV)
    codes1, lut1, qp1 = B.pseudograd_quantize(theta, local, off, workspace=ws)
    torch.cuda.synchronize()
    th_h, lo_h = t2n(theta), t2n(local)
    t0 = time.time()
    o_codes, o_luts, o_qp, o_d = oracle_mod.pseudograd_quantize(th_h, lo_h, off)
    say(f"[every element] oracle stage 1 on {N} elements: {time.time() - t0:.1f}s")
    del lo_h
    exact = check_qparams(B.qparams_to_numpy(qp1), o_qp)
    flips = check_codes(t2n(codes1), o_codes, o_d, off, o_qp)
    say(f"[every element] stage 1 codes compared ({time.time() - t_all:.0f}s)")
    worst = check_luts(t2n(lut1), o_luts, o_codes, off, o_qp)
    say(f"[every element] stage 1: {exact}/{T} ranges bit-equal, flips={flips}, worst lut rel={worst:.2e}")
    del o_d, codes1, local
    torch.cuda.empty_cache()

    # stage 2: the oracle's stage-1 codes as contribution 0 (stage-isolated), three synthetic ones
    peers = [torch.from_numpy(o_codes).to(DEV)]
    luts = [torch.from_numpy(o_luts).to(DEV)]
    for p in range(1, W):
        peers.append(synth.fill_coded_contribution(torch.empty(N, dtype=torch.uint8, device=DEV), p))
        luts.append(synth.synthetic_codebooks(T, p, device=DEV))
    acc = torch.empty(N, dtype=torch.float32, device=DEV)
    codes2 = torch.empty(N, dtype=torch.uint8, device=DEV)
    _, lut2, qp2 = B.reduce_chunk(peers, luts, off, W, codes_out=codes2, workspace=ws)           # recompute form
    _, lut2m, qp2m = B.reduce_chunk(peers, luts, off, W, acc_out=acc, codes_out=peers[W - 1],      # materialise form,
                                    workspace=ws)                                                  # codes over a consumed input
    torch.cuda.synchronize()
    h_codes = [o_codes] + [None] * (W - 1)
    # the host's copies of the synthetic contributions come from the generator again (the last one's device
    # buffer now holds the materialise call's codes)
    tmp = torch.empty(N, dtype=torch.uint8, device=DEV)
    for p in range(1, W):
        h_codes[p] = t2n(synth.fill_coded_contribution(tmp, p))
    del tmp
    say(f"[every element] stage 2 ran on the GPU, inputs on the host ({time.time() - t_all:.0f}s)")
    t0 = time.time()
    o_acc, o_c2, o_l2, o_q2 = oracle_mod.reduce(h_codes, [t2n(l) for l in luts], off, W)
    say(f"[every element] oracle reduce: {time.time() - t0:.1f}s")
    del h_codes, o_codes
    for name, g_codes, g_lut, g_qp in (("recompute", codes2, lut2, qp2), ("materialise", peers[W - 1], lut2m, qp2m)):
        exact = check_qparams(B.qparams_to_numpy(g_qp), o_q2)
        flips = check_codes(t2n(g_codes), o_c2, o_acc, off, o_q2)
        say(f"[every element] stage 2 ({name}) codes compared ({time.time() - t_all:.0f}s)")
        worst = check_luts(t2n(g_lut), o_l2, o_c2, off, o_q2)
        say(f"[every element] stage 2 ({name}): {exact}/{T} ranges bit-equal, flips={flips}, worst lut rel={worst:.2e}")
    assert np.array_equal(t2n(acc), o_acc)              # the stored accumulation: a fixed sequence of fp32 operations
    say(f"[every element] stored accumulation bit-equal ({time.time() - t_all:.0f}s)")
    del o_acc, acc, peers
    torch.cuda.empty_cache()

    # stage 3 from the oracle's requantised result, two steps (the second with a non-zero momentum)
    codes2.copy_(torch.from_numpy(o_c2))
    lut2.copy_(torch.from_numpy(o_l2))
    mom = torch.zeros(N, dtype=torch.float32, device=DEV)
    m_h = np.zeros(N, dtype=np.float32)
    # the oracle's new theta and momentum are copied up piece by piece and the comparison itself (the
    # tolerance formula of parity_utils.check_outer) is evaluated on the device: 4 x 10^10 values
    piece = 1 << 28
    for step in range(2):
        B.outer_step(theta, mom, LR, BETA, delta_codes=codes2, delta_lut=lut2, seg_offsets=off, workspace=ws)
        oracle_mod.outer_step(th_h, m_h, LR, BETA, delta_codes=o_c2, delta_luts=o_l2, seg_offsets=off)
        torch.cuda.synchronize()
        worst = 0.0
        for s in range(T):
            for a in range(off[s], off[s + 1], piece):
                b = min(a + piece, off[s + 1])
                g = lut2[s][codes2[a:b].long()].abs().double()                  # the oracle's codes and codebook
                m_o = torch.from_numpy(m_h[a:b]).to(DEV).double()
                t_o = torch.from_numpy(th_h[a:b]).to(DEV).double()
                for got, want, scale, what in ((mom[a:b], m_o, torch.maximum(m_o.abs(), g), "momentum"),
                                               (theta[a:b], t_o, torch.maximum(t_o.abs(), LR * (g + BETA * m_o.abs())),
                                                "theta")):
                    rel = ((got.double() - want).abs() / scale.clamp_min(1e-300)).max()
                    assert float(rel) <= 1e-5, f"{what}, step {step}, tensor {s}: {float(rel):.3e}"
                    worst = max(worst, float(rel))
        say(f"[every element] outer step {step + 1}: worst relative deviation {worst:.2e} ({time.time() - t_all:.0f}s)")
    say(f"[every element] all three stages, {N} elements each: {time.time() - t_all:.0f}s")


# ---------------------------------------------------------------------------------------------
# the whole 10B buffer as ONE quantisation group (every block's sums go to the same accumulators,
# counts beyond 2^32): properties that hold at any size, against fp64 reductions done by torch
# ---------------------------------------------------------------------------------------------

def test_fullsize_single_group_properties(B):
    N = synth.offsets_from_sizes(synth.config_segment_sizes(2))[-1]
    free, _ = torch.cuda.mem_get_info()
    if free < 110e9:
        pytest.skip(f"needs about 105 GB of free HBM, have {free / 1e9:.0f} GB")
    theta = synth.fill_theta_outer(torch.empty(N, dtype=torch.float32, device=DEV))
    local = synth.fill_theta_local(torch.empty(N, dtype=torch.float32, device=DEV), theta, 0, "mixture")
    codes, lut, qp = B.pseudograd_quantize(theta, local, [0, N])
    torch.cuda.synchronize()
    q = B.qparams_to_numpy(qp)[0]
    assert int(q["n"]) == N and int(q["status"]) == 0
    # statistics in fp64, chunk by chunk (two passes, as the definition has it)
    step = 1 << 28
    tot = 0.0
    for a in range(0, N, step):
        tot += float((theta[a:a + step] - local[a:a + step]).double().sum())
    mean = tot / N
    ss = 0.0
    for a in range(0, N, step):
        ss += float(((theta[a:a + step] - local[a:a + step]).double() - mean).pow(2).sum())
    std = (ss / (N - 1)) ** 0.5
    assert abs(q["mean"] - mean) <= 1e-9 * std and abs(q["std"] - std) <= 1e-9 * std
    assert abs(float(q["lo"]) - (mean - 6 * std)) <= 1e-6 * std
    assert abs(float(q["inv_w"]) - 256 / (12 * std)) <= 1e-6 * 256 / (12 * std)
    # codes: every element in the bucket the returned range gives it; decoding keeps the sum
    lo, inv_w = torch.tensor(q["lo"], device=DEV), torch.tensor(q["inv_w"], device=DEV)
    hist = torch.zeros(256, dtype=torch.int64, device=DEV)
    bucket_sum = torch.zeros(256, dtype=torch.float64, device=DEV)
    dec_sum = 0.0
    abs_sum = 0.0
    for a in range(0, N, step):
        d = theta[a:a + step] - local[a:a + step]
        k = ((d - lo) * inv_w).floor_().clamp_(0, 255).to(torch.uint8)
        assert torch.equal(k, codes[a:a + step])
        hist += torch.bincount(k.long(), minlength=256)
        bucket_sum += torch.bincount(k.long(), weights=d.double(), minlength=256)
        dec_sum += float(lut[0][k.long()].double().sum())
        abs_sum += float(d.double().abs().sum())
        del d, k
    assert int(hist.sum()) == N and int(hist.min()) > 0
    assert abs(dec_sum - tot) <= 2 ** -22 * abs_sum
    # the codebook: every bucket's average, within the per-call bar
    means = (bucket_sum / hist.double()).cpu().numpy()
    w = 12 * std / 256
    assert np.all(np.abs(t2n(lut[0]).astype(np.float64) - means) <= 1e-6 * np.maximum(np.abs(means), w))
    say(f"[single group] N={N}: mean {mean:.3e} std {std:.3e}, busiest bucket holds {int(hist.max())} elements")


# ---------------------------------------------------------------------------------------------
# stage 2 and two outer steps over the whole 10B buffer (381 tensors, W = 4), EVERY element against
# the same arithmetic done by torch's elementwise fp32 operations
# ---------------------------------------------------------------------------------------------

def test_fullsize_reduce_and_outer_every_element(B):
    sizes = synth.config_segment_sizes(2)
    off = synth.offsets_from_sizes(sizes)
    N, T, W = off[-1], len(sizes), 4
    free, _ = torch.cuda.mem_get_info()
    if free < 190e9:
        pytest.skip(f"needs about 185 GB of free HBM, have {free / 1e9:.0f} GB")
    peers = [synth.fill_coded_contribution(torch.empty(N, dtype=torch.uint8, device=DEV), p) for p in range(W)]
    luts = [synth.synthetic_codebooks(T, p, device=DEV) for p in range(W)]
    acc = torch.empty(N, dtype=torch.float32, device=DEV)
    codes2 = torch.empty(N, dtype=torch.uint8, device=DEV)
    ws = B.new_workspace(T, DEV)
    _, lut2, qp = B.reduce_chunk(peers, luts, off, W, acc_out=acc, codes_out=codes2, workspace=ws)
    torch.cuda.synchronize()
    q = B.qparams_to_numpy(qp)
    assert int(q["n"].sum()) == N and np.all(q["status"] == 0)
    step = 1 << 27

    def pieces():
        for s in range(T):
            for a in range(off[s], off[s + 1], step):
                yield s, a, min(a + step, off[s + 1])

    for s, a, b in pieces():
        r = luts[0][s][peers[0][a:b].long()]
        for p in range(1, W):
            r = r + luts[p][s][peers[p][a:b].long()]                # fp32, in contribution order
        r = r * 0.25
        assert torch.equal(acc[a:b], r), f"tensor {s}: stored accumulation"
        k = ((r - float(q["lo"][s])) * float(q["inv_w"][s])).floor_().clamp_(0, 255).to(torch.uint8)
        assert torch.equal(codes2[a:b], k), f"tensor {s}: codes"
    del peers
    torch.cuda.empty_cache()
    say("[every element] stage 2: accumulation and codes equal torch's on all elements")

    theta = synth.fill_theta_outer(torch.empty(N, dtype=torch.float32, device=DEV))
    mom = torch.zeros(N, dtype=torch.float32, device=DEV)
    for _ in range(2):
        B.outer_step(theta, mom, LR, BETA, delta_codes=codes2, delta_lut=lut2, seg_offsets=off, workspace=ws)
    torch.cuda.synchronize()
    theta0 = synth.fill_theta_outer(acc)                             # the same seeded values again
    worst = 0.0
    for s, a, b in pieces():
        g = lut2[s][codes2[a:b].long()].double()
        m1 = g
        t1 = theta0[a:b].double() - LR * (g + BETA * m1)
        m2 = BETA * m1 + g
        t2 = t1 - LR * (g + BETA * m2)
        scale = torch.maximum(t2.abs(), LR * (1 + BETA) * g.abs() * 2)
        worst = max(worst, float(((theta[a:b].double() - t2).abs() / scale.clamp_min(1e-300)).max()),
                    float(((mom[a:b].double() - m2).abs() / m2.abs().clamp_min(1e-300)).max()))
    assert worst <= 1e-5, worst
    say(f"[every element] two outer steps: worst relative deviation {worst:.2e}")


# ---------------------------------------------------------------------------------------------
# the call variants bench.py --extras times, at the same full size: bf16 theta_local in stage 1,
# stage 2 storing its fp32 accumulation, the outer step from that fp32 array with the workers' new
# weights handed back in the same pass (fp32, then bf16 from codes); sampled tensors + any-size properties
# ---------------------------------------------------------------------------------------------

def test_config2_fullsize_call_variants_sampled(B, oracle_mod):
    sizes = synth.config_segment_sizes(2)
    off = synth.offsets_from_sizes(sizes)
    N, T, W = off[-1], len(sizes), 4
    free, _ = torch.cuda.mem_get_info()
    if free < 215e9:
        pytest.skip(f"needs about 210 GB of free HBM, have {free / 1e9:.0f} GB")
    # layer 5 wv (4.2M), layer 33 wo (16.8M), layer 12 attn_norm (4,096), layer 26 w_up (58.7M)
    sample = [1 + 9 * 5 + 2, 1 + 9 * 33 + 3, 1 + 9 * 12 + 7, 1 + 9 * 26 + 5]
    say(f"[variants] N={N}; sampled tensors {sample} sizes {[sizes[s] for s in sample]}")
    theta = synth.fill_theta_outer(torch.empty(N, dtype=torch.float32, device=DEV))
    local16 = torch.empty(N, dtype=torch.bfloat16, device=DEV)
    acc = torch.empty(N, dtype=torch.float32, device=DEV)          # also the scratch the fills go through
    peer_codes = [torch.empty(N, dtype=torch.uint8, device=DEV) for _ in range(W)]
    peer_luts = [torch.empty((T, 256), dtype=torch.float32, device=DEV) for _ in range(W)]
    qp = B.new_qparams(T, DEV)
    ws = B.new_workspace(T, DEV)
    th_s = {s: t2n(theta[off[s]:off[s + 1]]) for s in sample}
    o1 = {s: [] for s in sample}
    flips = 0
    for p in range(W):
        synth.fill_theta_local(local16, theta, p, "mixture")       # bf16(theta + delta)
        B.pseudograd_quantize(theta, local16, off, codes_out=peer_codes[p], lut_out=peer_luts[p],
                              qparams_out=qp, workspace=ws)
        torch.cuda.synchronize()
        g_qp = B.qparams_to_numpy(qp)
        assert int(g_qp["n"].sum()) == N and np.all(g_qp["status"] == 0)
        for s in sample:
            a, b = off[s], off[s + 1]
            o = oracle_mod.pseudograd_quantize(th_s[s], bf16_bits(local16[a:b]), [0, b - a], local_is_bf16=True)
            check_qparams(g_qp[s:s + 1], o[2])
            flips += check_codes(t2n(peer_codes[p][a:b]), o[0], o[3], [0, b - a], o[2])
            check_luts(t2n(peer_luts[p][s]), o[1], o[0], [0, b - a], o[2])
            o1[s].append(o)
            peer_codes[p][a:b].copy_(torch.from_numpy(o[0]))        # stage-isolated: the oracle's codes go on
            peer_luts[p][s].copy_(torch.from_numpy(o[1][0]))
    say(f"[variants] stage 1 with bf16 theta_local checked for {W} workers")
    del local16
    torch.cuda.empty_cache()

    codes2 = torch.empty(N, dtype=torch.uint8, device=DEV)
    lut2 = torch.empty((T, 256), dtype=torch.float32, device=DEV)
    B.reduce_chunk(peer_codes, peer_luts, off, W, acc_out=acc, codes_out=codes2, lut_out=lut2, qparams_out=qp,
                   workspace=ws)
    torch.cuda.synchronize()
    g_qp = B.qparams_to_numpy(qp)
    assert int(g_qp["n"].sum()) == N and np.all(g_qp["status"] == 0)
    o_accs = {}
    for s in sample:
        a, b = off[s], off[s + 1]
        o_acc, o_c2, o_l2, o_q2 = oracle_mod.reduce([o[0] for o in o1[s]], [o[1] for o in o1[s]], [0, b - a], W)
        check_qparams(g_qp[s:s + 1], o_q2)
        flips += check_codes(t2n(codes2[a:b]), o_c2, o_acc, [0, b - a], o_q2)
        check_luts(t2n(lut2[s]), o_l2, o_c2, [0, b - a], o_q2)
        assert np.array_equal(t2n(acc[a:b]), o_acc)                 # a fixed sequence of fp32 operations
        o_accs[s] = (o_acc, o_c2, o_l2)
        codes2[a:b].copy_(torch.from_numpy(o_c2))                   # stage-isolated, as above
        lut2[s].copy_(torch.from_numpy(o_l2[0]))
    del peer_codes
    torch.cuda.empty_cache()
    say("[variants] stage 2 storing the accumulation checked")

    # outer step from the stored fp32 average, new weights handed back in fp32
    mom = torch.zeros(N, dtype=torch.float32, device=DEV)
    handback = torch.empty(N, dtype=torch.float32, device=DEV)
    B.outer_step(theta, mom, LR, BETA, delta_fp32=acc, theta_local_out=handback, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(handback, theta) and torch.equal(mom, acc)    # any size: first step, m' = g
    th1 = {}
    for s in sample:
        a, b = off[s], off[s + 1]
        th_o, m_o = th_s[s].copy(), np.zeros(b - a, dtype=np.float32)
        oracle_mod.outer_step(th_o, m_o, LR, BETA, delta_fp32=o_accs[s][0])
        check_outer(t2n(mom[a:b]), m_o, np.zeros(b - a, dtype=np.float32), np.abs(m_o), "momentum")
        check_outer(t2n(theta[a:b]), th_o, th_s[s], LR * (1 + BETA) * np.abs(m_o), "theta")
        th1[s] = (th_o, m_o)                                        # the oracle's state goes on, on both sides
        theta[a:b].copy_(torch.from_numpy(th_o))
        mom[a:b].copy_(torch.from_numpy(m_o))
    del handback
    torch.cuda.empty_cache()
    # a second step, from the codes, new weights handed back in bf16
    handback16 = torch.empty(N, dtype=torch.bfloat16, device=DEV)
    B.outer_step(theta, mom, LR, BETA, delta_codes=codes2, delta_lut=lut2, seg_offsets=off,
                 theta_local_out=handback16, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(handback16, theta.to(torch.bfloat16))         # any size: round to nearest even
    for s in sample:
        a, b = off[s], off[s + 1]
        th_o, m_o = th1[s][0].copy(), th1[s][1].copy()
        o_c2, o_l2 = o_accs[s][1], o_accs[s][2]
        g = o_l2[0][o_c2]
        oracle_mod.outer_step(th_o, m_o, LR, BETA, delta_codes=o_c2, delta_luts=o_l2, seg_offsets=[0, b - a])
        check_outer(t2n(mom[a:b]), m_o, th1[s][1], np.abs(g), "momentum, second step")
        check_outer(t2n(theta[a:b]), th_o, th1[s][0], LR * (np.abs(g) + BETA * np.abs(m_o)), "theta, second step")
    say(f"[variants] outer step from fp32 and from codes with hand-back checked; flips on sampled tensors: {flips}")


# ---------------------------------------------------------------------------------------------
# configuration 3 at full size: 14 heavy-tailed coded peers resident (143 GB of codes), the
# accumulation stored over theta_local, checked on sampled tensors
# ---------------------------------------------------------------------------------------------

def test_config3_fullsize_sampled_tensors(B, oracle_mod):
    sizes = synth.config_segment_sizes(3)
    off = synth.offsets_from_sizes(sizes)
    N, T, W = off[-1], len(sizes), 14
    free, _ = torch.cuda.mem_get_info()
    if free < 245e9:
        pytest.skip(f"needs about 240 GB of free HBM, have {free / 1e9:.0f} GB")
    # final norm (4,096), layer 11 wv (4.2M), layer 30 wo (16.8M), layer 17 w_gate (58.7M)
    sample = [T - 2, 1 + 9 * 11 + 2, 1 + 9 * 30 + 3, 1 + 9 * 17 + 4]
    say(f"[config3] N={N} T={T} W={W}; sampled tensors {sample} sizes {[sizes[s] for s in sample]}")
    theta = synth.fill_theta_outer(torch.empty(N, dtype=torch.float32, device=DEV))
    local = torch.empty(N, dtype=torch.float32, device=DEV)
    peer_codes = [torch.empty(N, dtype=torch.uint8, device=DEV) for _ in range(W)]
    peer_luts = [torch.empty((T, 256), dtype=torch.float32, device=DEV) for _ in range(W)]
    qp = B.new_qparams(T, DEV)
    ws = B.new_workspace(T, DEV)
    th_s = {s: t2n(theta[off[s]:off[s + 1]]) for s in sample}
    o1 = {s: [] for s in sample}
    t0 = time.time()
    flips1 = 0
    for p in range(W):
        synth.fill_theta_local(local, theta, p, "student_t3")
        B.pseudograd_quantize(theta, local, off, codes_out=peer_codes[p], lut_out=peer_luts[p], qparams_out=qp,
                              workspace=ws)
        torch.cuda.synchronize()
        g_qp = B.qparams_to_numpy(qp)
        assert int(g_qp["n"].sum()) == N and np.all(g_qp["status"] == 0)
        # stage 1 on heavy-tailed data at full size, checked on the sampled tensors; these then get the
        # oracle's own stage-1 output (stage 2 is checked in isolation)
        for s in sample:
            a, b = off[s], off[s + 1]
            o = oracle_mod.pseudograd_quantize(th_s[s], t2n(local[a:b]), [0, b - a])
            check_qparams(g_qp[s:s + 1], o[2])
            flips1 += check_codes(t2n(peer_codes[p][a:b]), o[0], o[3], [0, b - a], o[2])
            check_luts(t2n(peer_luts[p][s]), o[1], o[0], [0, b - a], o[2])
            o1[s].append(o)
            peer_codes[p][a:b].copy_(torch.from_numpy(o[0]))
            peer_luts[p][s].copy_(torch.from_numpy(o[1][0]))
    say(f"[config3] {W} peers ready ({time.time() - t0:.1f}s)")
    codes2 = torch.empty(N, dtype=torch.uint8, device=DEV)
    lut2 = torch.empty((T, 256), dtype=torch.float32, device=DEV)
    B.reduce_chunk(peer_codes, peer_luts, off, W, acc_out=local, codes_out=codes2, lut_out=lut2, qparams_out=qp,
                   workspace=ws)
    torch.cuda.synchronize()
    g_qp = B.qparams_to_numpy(qp)
    assert int(g_qp["n"].sum()) == N and np.all(g_qp["status"] == 0)
    flips = 0
    o2 = {}
    for s in sample:
        a, b = off[s], off[s + 1]
        o_acc, o_c2, o_l2, o_q2 = oracle_mod.reduce([o[0] for o in o1[s]], [o[1] for o in o1[s]], [0, b - a], W)
        check_qparams(g_qp[s:s + 1], o_q2)
        flips += check_codes(t2n(codes2[a:b]), o_c2, o_acc, [0, b - a], o_q2)
        check_luts(t2n(lut2[s]), o_l2, o_c2, [0, b - a], o_q2)
        assert np.array_equal(t2n(local[a:b]), o_acc)                 # a fixed sequence of fp32 operations
        o2[s] = (o_c2, o_l2)
    # any size: the requantised embedding tensor decodes to the same sum as the stored accumulation
    a, b = off[0], off[1]
    dec = lut2[0][codes2[a:b].long()].double()
    acc = local[a:b].double()
    assert abs(float(dec.sum() - acc.sum())) <= 2 ** -22 * float(acc.abs().sum())
    say(f"[config3] stage 1 (x{W}) and stage 2 at W=14 checked on {len(sample)} tensors; one-bucket flips: "
        f"{flips1} / {flips}")
    # the outer step from the requantised average, over the full buffer (the coded contributions are
    # consumed: their memory goes to the momentum buffer), checked on the sampled tensors from the
    # oracle's own codes
    del peer_codes, dec, acc
    torch.cuda.empty_cache()
    for s in sample:
        a, b = off[s], off[s + 1]
        codes2[a:b].copy_(torch.from_numpy(o2[s][0]))
        lut2[s].copy_(torch.from_numpy(o2[s][1][0]))
    mom = torch.zeros(N, dtype=torch.float32, device=DEV)
    handback = local.view(torch.bfloat16)[:N]                         # new worker weights over the consumed average
    B.outer_step(theta, mom, LR, BETA, delta_codes=codes2, delta_lut=lut2, seg_offsets=off,
                 theta_local_out=handback, workspace=ws)
    torch.cuda.synchronize()
    for s in sample:
        a, b = off[s], off[s + 1]
        th_o, m_o = th_s[s].copy(), np.zeros(b - a, dtype=np.float32)
        oracle_mod.outer_step(th_o, m_o, LR, BETA, delta_codes=o2[s][0], delta_luts=o2[s][1], seg_offsets=[0, b - a])
        check_outer(t2n(mom[a:b]), m_o, np.zeros(b - a, dtype=np.float32), np.abs(m_o), "momentum")
        check_outer(t2n(theta[a:b]), th_o, th_s[s], LR * (1 + BETA) * np.abs(m_o), "theta")
    assert torch.equal(handback, theta.to(torch.bfloat16))           # any size: round to nearest even
    say("[config3] outer step checked on the sampled tensors")


def _stage1_every_element(B, oracle_mod, off, kind, local_dtype, label):
    """Stage 1 on a full-size buffer, every element and every range against the oracle."""
    import psutil
    N, T = off[-1], len(off) - 1
    free, _ = torch.cuda.mem_get_info()
    if free < 100e9:
        pytest.skip(f"needs about 95 GB of free HBM, have {free / 1e9:.0f} GB")
    if psutil.virtual_memory().available < 175e9:
        pytest.skip(f"needs about 145 GB of host memory, {psutil.virtual_memory().available / 1e9:.0f} GB available")
    t_all = time.time()
    theta = synth.fill_theta_outer(torch.empty(N, dtype=torch.float32, device=DEV))
    local = synth.fill_theta_local(torch.empty(N, dtype=local_dtype, device=DEV), theta, 0, kind)
    codes, lut, qp = B.pseudograd_quantize(theta, local, off)
    torch.cuda.synchronize()
    bf16 = local_dtype == torch.bfloat16
    th_h, lo_h = t2n(theta), (bf16_bits(local) if bf16 else t2n(local))
    del theta, local
    say(f"[{label}] inputs on the host ({time.time() - t_all:.0f}s)")
    o_codes, o_luts, o_qp, o_d = oracle_mod.pseudograd_quantize(th_h, lo_h, off, local_is_bf16=bf16)
    del th_h, lo_h
    a, b = off[min(1, T - 1)], off[min(1, T - 1) + 1]
    say(f"[{label}] oracle done ({time.time() - t_all:.0f}s); largest |d| / sigma = "
        f"{float(np.abs(o_d[a:b]).max() / o_qp['std'][min(1, T - 1)]):.0f} in group {min(1, T - 1)}")
    exact = check_qparams(B.qparams_to_numpy(qp), o_qp, require_exact=1.0 if T < 100 else None)
    flips = check_codes(t2n(codes), o_codes, o_d, off, o_qp)
    say(f"[{label}] codes compared ({time.time() - t_all:.0f}s)")
    worst = check_luts(t2n(lut), o_luts, o_codes, off, o_qp)
    clipped = float(np.mean((o_codes[a:b] == 0) | (o_codes[a:b] == 255)))
    say(f"[{label}] {exact}/{T} ranges bit-equal, flips={flips}, worst lut rel={worst:.2e}; "
        f"{100 * clipped:.2f} % of group {min(1, T - 1)} in the two end buckets ({time.time() - t_all:.0f}s)")


def test_config3_fullsize_stage1_every_element_heavy_tails(B, oracle_mod):
    """Stage 1 on the full 10B buffer of Student-t (nu = 3) pseudo-gradients - values beyond 100 sigma occur."""
    _stage1_every_element(B, oracle_mod, synth.offsets_from_sizes(synth.config_segment_sizes(3)), "student_t3",
                          torch.float32, "config3 every element")


def test_config4_fullsize_stage1_every_element_bf16_ring_chunks(B, oracle_mod):
    """Stage 1 with a bf16 theta_local on the full 10B buffer cut into the 14 ring chunks (groups of 729,384,375
    elements starting at odd offsets)."""
    _stage1_every_element(B, oracle_mod, synth.offsets_from_sizes(synth.config_segment_sizes(4)), "mixture",
                          torch.bfloat16, "config4 every element")


# ---------------------------------------------------------------------------------------------
# configuration 4 at full size: one whole ring chunk (729,384,375 elements, starting at an odd
# element offset of the full-size buffers), 13 coded contributions + the fp32 local addend
# ---------------------------------------------------------------------------------------------

def test_config4_fullsize_ring_chunks(B, oracle_mod):
    """Chunk 0 (starts at element 0), chunk 1 (odd offset) and chunk 13 (the short last one, 729,384,373
    elements) of the full-size buffers, each reduced whole and compared with the oracle."""
    N = synth.n_elements(2)
    coff = synth.offsets_from_sizes(synth.ring_chunk_sizes(N, 14))
    W = 13
    assert coff[1] % 2 == 1 and coff[2] - coff[1] == 729_384_375 and coff[14] - coff[13] == 729_384_373
    free, _ = torch.cuda.mem_get_info()
    if free < 190e9:
        pytest.skip(f"needs about 185 GB of free HBM, have {free / 1e9:.0f} GB")
    # full-size buffers, as the benchmark holds them; only the chunk under test is filled
    local = torch.empty(N, dtype=torch.float32, device=DEV)
    peer_codes = [torch.empty(N, dtype=torch.uint8, device=DEV) for _ in range(W)]
    codes2 = torch.empty(N, dtype=torch.uint8, device=DEV)
    lut2 = torch.empty((14, 256), dtype=torch.float32, device=DEV)
    peer_luts = [synth.synthetic_codebooks(14, p, device=DEV) for p in range(W)]
    for c in (0, 1, 13):
        a, b = coff[c], coff[c + 1]
        n = b - a
        say(f"[config4] chunk {c}: elements [{a}, {b}) of {N}, W={W} coded + fp32 local")
        synth.fill_delta(local[a:b], W, "mixture", seed=synth.BASE_SEED + c)
        for p in range(W):
            synth.fill_coded_contribution(peer_codes[p][a:b], p, seed=synth.BASE_SEED + c)
        torch.cuda.synchronize()
        h_local = t2n(local[a:b])
        h_codes = [t2n(pc[a:b]) for pc in peer_codes]
        h_luts = [t2n(pl[c:c + 1]) for pl in peer_luts]
        codes_g, lut_g, qp_g = B.reduce_chunk([pc[a:b] for pc in peer_codes], [pl[c:c + 1] for pl in peer_luts],
                                              [0, n], 14, local_fp32=local[a:b], acc_out=local[a:b],
                                              codes_out=codes2[a:b], lut_out=lut2[c:c + 1])
        torch.cuda.synchronize()
        t0 = time.time()
        o_acc, o_c2, o_l2, o_q2 = oracle_mod.reduce(h_codes, h_luts, [0, n], 14, local_fp32=h_local)
        say(f"[config4] oracle reduce of chunk {c}: {time.time() - t0:.1f}s")
        del h_codes
        check_qparams(B.qparams_to_numpy(qp_g), o_q2, require_exact=1.0)
        flips = check_codes(t2n(codes_g), o_c2, o_acc, [0, n], o_q2)
        check_luts(t2n(lut_g), o_l2, o_c2, [0, n], o_q2)
        assert np.array_equal(t2n(local[a:b]), o_acc)
        say(f"[config4] chunk {c}: one-bucket flips: {flips} of {n}")
        del o_acc, o_c2, h_local


# ---------------------------------------------------------------------------------------------
# one quantisation group per matrix row (Section 2.2 says "for each tensor"; the group is whatever the
# caller declares): one decoder layer as 43,010 groups whose scales differ row by row, every element
# and every group against the oracle, stage 1 and the reduce
# ---------------------------------------------------------------------------------------------

def test_per_row_groups_one_layer(B, oracle_mod):
    row_sizes = synth.layer_row_sizes()
    off = synth.offsets_from_sizes(row_sizes)
    N, T = off[-1], len(row_sizes)
    say(f"[rows] N={N} in {T} groups of 4,096 / 14,336 elements")
    theta = synth.fill_theta_outer(torch.empty(N, dtype=torch.float32, device=DEV))
    local = synth.fill_theta_local(torch.empty(N, dtype=torch.float32, device=DEV), theta, 0, "mixture")
    # rows with log-normally spread scales (sigma_ln = 1): theta_local = theta - scale_row * delta
    g = torch.Generator(device=DEV).manual_seed(synth.BASE_SEED + 77)
    scale = torch.exp(torch.randn(T, device=DEV, generator=g))
    local = theta - (theta - local) * torch.repeat_interleave(scale, torch.tensor(row_sizes, device=DEV))
    ws = B.new_workspace(T, DEV)
    codes, luts, qp = B.pseudograd_quantize(theta, local, off, workspace=ws)
    torch.cuda.synchronize()
    t0 = time.time()
    o_codes, o_luts, o_qp, o_d = oracle_mod.pseudograd_quantize(t2n(theta), t2n(local), off)
    say(f"[rows] oracle stage 1: {time.time() - t0:.1f}s")
    exact = check_qparams(B.qparams_to_numpy(qp), o_qp)
    flips = check_codes(t2n(codes), o_codes, o_d, off, o_qp)
    worst = check_luts(t2n(luts), o_luts, o_codes, off, o_qp)
    say(f"[rows] stage 1: {exact}/{T} groups with bit-equal range, flips={flips}, worst lut rel={worst:.2e}")
    # the reduce of two such contributions (the second: the first one's codes reversed inside each row
    # would need new codebooks, so simply the same contribution twice with divisor 2: the average decodes
    # to the contribution itself) and of contribution + fp32 addend, both forms
    pc, pl = torch.from_numpy(o_codes).to(DEV), torch.from_numpy(o_luts).to(DEV)
    addend = torch.from_numpy(o_d).to(DEV).flip(0).contiguous()
    h_addend = t2n(addend)
    for form, kw_g, kw_o in (("W=2", dict(), dict()),
                             ("W=1 + fp32 addend, in place", dict(local_fp32=addend, acc_out=addend),
                              dict(local_fp32=h_addend))):
        Wc = 2 if not kw_g else 1
        c2, l2, q2 = B.reduce_chunk([pc] * Wc, [pl] * Wc, off, 2, workspace=ws, **kw_g)
        torch.cuda.synchronize()
        o_acc, o_c2, o_l2, o_q2 = oracle_mod.reduce([o_codes] * Wc, [o_luts] * Wc, off, 2, **kw_o)
        exact = check_qparams(B.qparams_to_numpy(q2), o_q2)
        flips = check_codes(t2n(c2), o_c2, o_acc, off, o_q2)
        check_luts(t2n(l2), o_l2, o_c2, off, o_q2)
        if kw_g:
            assert np.array_equal(t2n(addend), o_acc)
        say(f"[rows] reduce {form}: {exact}/{T} groups with bit-equal range, flips={flips}")
