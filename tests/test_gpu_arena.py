"""The arena (one allocation, carved views) and the timed placement of the outer state."""
import pytest
import torch

from paper_2412_01152_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_carve_is_aligned_disjoint_and_bounded():
    from paper_2412_01152_amd.arena import ALIGN, Arena
    arena = Arena(DEV, nbytes=1 << 24)
    a = arena.carve(1000, torch.float32)
    b = arena.carve(333, torch.uint8)
    c = arena.carve(77, torch.bfloat16)
    ptrs = [(t.data_ptr(), t.numel() * t.element_size()) for t in (a, b, c)]
    for p, _ in ptrs:
        assert p % ALIGN == 0
    for (p0, n0), (p1, _) in zip(ptrs, ptrs[1:]):
        assert p0 + n0 <= p1
    assert a.dtype == torch.float32 and a.numel() == 1000 and c.dtype == torch.bfloat16
    d = arena.carve(10, torch.float32, at=1 << 20)
    assert d.data_ptr() == arena.buf.data_ptr() + (1 << 20)
    with pytest.raises(RuntimeError):
        arena.carve(1 << 24, torch.uint8)
    a.fill_(1.0)
    b.fill_(2)
    assert float(a.sum()) == 1000.0 and int(b.sum()) == 666       # the views do not overlap


def test_place_outer_state_returns_a_candidate_and_library_works_on_carved_views():
    from paper_2412_01152_amd import binding as B
    from paper_2412_01152_amd.arena import GiB, Arena, place_outer_state
    B.load()
    n = 3_000_001
    off = [0, 1_000_000, n]
    arena = Arena(DEV, nbytes=3 * GiB)
    shift = place_outer_state(arena, n, off, [0, 1, 2], tail_bytes=3 * n)
    assert shift in (0, GiB, 2 * GiB) and arena.pos == 0
    theta = arena.carve(n, torch.float32, at=shift)
    local = arena.carve(n, torch.float32)
    mom = arena.carve(n, torch.float32).zero_()
    codes = arena.carve(n, torch.uint8)
    synth.fill_theta_outer(theta)
    synth.fill_theta_local(local, theta, 0, "mixture")
    ref = B.pseudograd_quantize(theta.clone(), local.clone(), off)          # separate allocations
    got = B.pseudograd_quantize(theta, local, off, codes_out=codes)
    torch.cuda.synchronize()
    assert torch.equal(ref[0], got[0]) and torch.allclose(ref[1], got[1], rtol=1e-6, atol=0)
    th0 = theta.clone()
    B.outer_step(theta, mom, 0.7, 0.9, delta_codes=got[0], delta_lut=got[1], seg_offsets=off)
    torch.cuda.synchronize()
    g = torch.cat([got[1][s][got[0][off[s]:off[s + 1]].long()] for s in range(2)])
    assert torch.equal(mom, g)                                             # first step from zero: m' = g
    assert torch.allclose(theta, th0 - 0.7 * 1.9 * g, rtol=1e-5, atol=1e-7)


def test_role_bases_are_a_third_of_the_arena_apart():
    from paper_2412_01152_amd.arena import ALIGN, GiB, Arena, role_bases
    arena = Arena(DEV, nbytes=3 * GiB)
    r = role_bases(arena)
    assert list(r) == ["read", "state", "out"] and all(v % ALIGN == 0 for v in r.values())
    assert r["state"] - r["read"] == r["out"] - r["state"] == GiB
    a = arena.carve(1000, torch.float32, at=r["read"])
    b = arena.carve(1000, torch.float32, at=r["state"])
    c = arena.carve(1000, torch.uint8, at=r["out"])
    assert b.data_ptr() - a.data_ptr() == GiB and c.data_ptr() - b.data_ptr() == GiB
