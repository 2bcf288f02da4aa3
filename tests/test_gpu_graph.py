"""The three calls recorded into one HIP graph: the library enqueues kernels only (no allocation, no
memset node, no copy, no synchronisation), so a caller may capture a whole outer synchronisation
and replay it.  Every replay, on fresh inputs and with eager work and synchronisations between the
replays, must give what the same calls give when launched eagerly (which the parity tests tie to
the oracle); stage 1 of the first replay is also checked against the oracle directly."""
import numpy as np
import pytest
import torch

from paper_2412_01152_amd import synth
from parity_utils import check_codes, check_luts, check_qparams, t2n

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
LR, BETA = 0.7, 0.9


def _same_qparams(B, a, b):
    qa, qb = B.qparams_to_numpy(a), B.qparams_to_numpy(b)
    for f in ("lo", "inv_w", "n", "status"):
        assert np.array_equal(qa[f], qb[f]), f
    # the fp64 sums behind mean and std are accumulated by atomics, whose order may differ
    np.testing.assert_allclose(qa["mean"], qb["mean"], rtol=1e-12, atol=1e-300)
    np.testing.assert_allclose(qa["std"], qb["std"], rtol=1e-12, atol=1e-300)


def test_outer_synchronisation_captured_once_replayed_thrice(oracle_mod):
    from paper_2412_01152_amd import binding as B
    B.load()
    W = 3
    sizes = [100_000, 4096, 3, 77_777, 0, 300_001]
    off = synth.offsets_from_sizes(sizes)
    n, T = off[-1], len(sizes)

    def inputs(seed):
        theta, locals_, _ = synth.make_inputs(sizes, W, kind="mixture", device="cpu", seed=seed)
        mom = torch.randn(n, generator=torch.Generator().manual_seed(seed)) * 1e-3
        return theta, locals_, mom

    # static buffers the graph reads and writes
    theta_s = torch.empty(n, dtype=torch.float32, device=DEV)
    local_s = torch.empty(n, dtype=torch.float32, device=DEV)
    mom_s = torch.empty(n, dtype=torch.float32, device=DEV)
    peer_codes = [torch.empty(n, dtype=torch.uint8, device=DEV) for _ in range(W - 1)]
    peer_luts = [torch.empty((T, 256), dtype=torch.float32, device=DEV) for _ in range(W - 1)]
    c1, c2 = (torch.empty(n, dtype=torch.uint8, device=DEV) for _ in range(2))
    l1, l2 = (torch.empty((T, 256), dtype=torch.float32, device=DEV) for _ in range(2))
    q1, q2 = B.new_qparams(T, DEV), B.new_qparams(T, DEV)
    ws = B.new_workspace(T, DEV)

    def three_calls(theta, local, mom, pc, pl, c1, l1, q1, c2, l2, q2, ws):
        B.pseudograd_quantize(theta, local, off, codes_out=c1, lut_out=l1, qparams_out=q1, workspace=ws)
        B.reduce_chunk([c1] + pc, [l1] + pl, off, W, codes_out=c2, lut_out=l2, qparams_out=q2, workspace=ws)
        B.outer_step(theta, mom, LR, BETA, delta_codes=c2, delta_lut=l2, seg_offsets=off, workspace=ws)

    def load(seed):
        theta, locals_, mom = inputs(seed)
        theta_s.copy_(theta)
        local_s.copy_(locals_[0])
        mom_s.copy_(mom)
        for p in range(1, W):                                  # the other workers' contributions (eager set-up)
            c, l, _ = B.pseudograd_quantize(theta_s, locals_[p].to(DEV), off)
            peer_codes[p - 1].copy_(c)
            peer_luts[p - 1].copy_(l)
        torch.cuda.synchronize()
        return theta, locals_, mom

    # warm-up on a side stream (first-use queries happen here, outside any capture), then capture
    load(1)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        three_calls(theta_s, local_s, mom_s, peer_codes, peer_luts, c1, l1, q1, c2, l2, q2, ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        three_calls(theta_s, local_s, mom_s, peer_codes, peer_luts, c1, l1, q1, c2, l2, q2, ws)

    for rep, seed in enumerate((11, 12, 13)):
        theta, locals_, mom = load(seed)
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (c1, l1, q1, c2, l2, q2, theta_s, mom_s)]

        # the same calls, eagerly, on separate buffers holding the same inputs
        e_theta, e_local, e_mom = theta.to(DEV), locals_[0].to(DEV), mom.to(DEV)
        e = [torch.empty_like(t) for t in (c1, l1, q1, c2, l2, q2)]
        three_calls(e_theta, e_local, e_mom, [c.clone() for c in peer_codes], [l.clone() for l in peer_luts],
                    *e, B.new_workspace(T, DEV))
        torch.cuda.synchronize()
        assert torch.equal(got[0], e[0]) and torch.equal(got[3], e[3]), f"replay {rep}: codes"
        assert torch.equal(got[1], e[1]) and torch.equal(got[4], e[4]), f"replay {rep}: codebooks"
        _same_qparams(B, got[2], e[2])
        _same_qparams(B, got[5], e[5])
        assert torch.equal(got[6], e_theta) and torch.equal(got[7], e_mom), f"replay {rep}: outer step"

        if rep == 0:       # stage 1 reads nothing the library made: straight against the oracle as well
            o_codes, o_luts, o_qp, d = oracle_mod.pseudograd_quantize(theta.numpy(), locals_[0].numpy(), off)
            check_qparams(B.qparams_to_numpy(got[2]), o_qp)
            check_codes(t2n(got[0]), o_codes, d, off, o_qp)
            check_luts(t2n(got[1]), o_luts, o_codes, off, o_qp)
