"""Ring-order solver (Section 2.5: the Hamiltonian cycle whose slowest link is fastest).  Host code,
no GPU.  The enumerating oracle is pinned on hand-worked cases; the library's exact solver is compared
with it on small random matrices and checked by properties on larger ones."""
import os

import numpy as np
import pytest


@pytest.fixture(scope="module")
def B():
    from paper_2412_01152_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    binding.load()
    return binding


@pytest.fixture(scope="module")
def O():
    from oracle import ring_order
    return ring_order


def _valid(order, n):
    return sorted(order) == list(range(n)) and order[0] == 0


# ---- the oracle against cases worked by hand ----------------------------------------------------

def test_oracle_three_nodes_has_two_directed_cycles(O):
    w = [[0, 5, 1],
         [2, 0, 7],
         [9, 3, 0]]
    # 0->1->2->0: min(5, 7, 9) = 5;  0->2->1->0: min(1, 3, 2) = 1
    b, order = O.best_ring(w)
    assert b == 5 and order == [0, 1, 2]
    assert O.cycle_bottleneck(w, [0, 2, 1]) == 1


def test_oracle_four_nodes_symmetric_by_hand(O):
    # square 0-1-2-3-0 with fast sides (10, 8, 9, 7) and slow diagonals (1, 2): the three undirected
    # cycles are the square (min 7) and the two that use both diagonals (min 1)
    w = np.zeros((4, 4))
    for (u, v), x in {(0, 1): 10, (1, 2): 8, (2, 3): 9, (3, 0): 7, (0, 2): 1, (1, 3): 2}.items():
        w[u][v] = w[v][u] = x
    b, order = O.best_ring(w.tolist())
    assert b == 7 and order in ([0, 1, 2, 3], [0, 3, 2, 1])


def test_oracle_weak_node_forces_the_bottleneck(O):
    # node 4's two best links are 3 and 2; every ring passes through it, so no ring beats 2
    w = np.full((5, 5), 10.0)
    w[4, :] = w[:, 4] = [3, 2, 1, 1, 0]
    b, _ = O.best_ring(w.tolist())
    assert b == 2


def test_oracle_trivial_sizes(O):
    assert O.best_ring([[0.0]]) == (float("inf"), [0])
    assert O.best_ring([[0, 4], [6, 0]]) == (4, [0, 1])


# ---- the library against the oracle --------------------------------------------------------------

@pytest.mark.parametrize("n", range(1, 9))
@pytest.mark.parametrize("symmetric", [False, True])
def test_solver_matches_enumeration(B, O, n, symmetric):
    rng = np.random.default_rng(1000 + 10 * n + symmetric)
    for trial in range(6):
        w = rng.uniform(0.1, 4.0, (n, n)) if trial % 2 else rng.integers(1, 6, (n, n)).astype(float)   # ties too
        if symmetric:
            w = np.maximum(w, w.T)
        order, b = B.ring_order(w)
        b_ref, _ = O.best_ring(w.tolist())
        assert _valid(order, n)
        assert b == b_ref
        assert O.cycle_bottleneck(w.tolist(), order) == b


@pytest.mark.parametrize("n", [12, 14, 16, 20])
def test_planted_ring_is_recovered(B, O, n):
    """A hidden ring of fast links in a sea of slow ones: the only ring with a bottleneck above the
    slow level is the planted one, in its direction."""
    rng = np.random.default_rng(n)
    perm = [0] + list(rng.permutation(np.arange(1, n)))
    w = rng.uniform(0.5, 4.0, (n, n))
    fast = rng.uniform(10.0, 20.0, n)
    for i in range(n):
        w[perm[i], perm[(i + 1) % n]] = fast[i]
    order, b = B.ring_order(w)
    assert order == [int(p) for p in perm]
    assert b == fast.min()


@pytest.mark.parametrize("n", [10, 13, 16])
def test_bounds_on_larger_random_graphs(B, O, n):
    rng = np.random.default_rng(50 + n)
    w = rng.uniform(0.5, 4.0, (n, n))
    order, b = B.ring_order(w)
    assert _valid(order, n) and O.cycle_bottleneck(w.tolist(), order) == b
    off = w + np.diag(np.full(n, -np.inf))
    assert b <= off.max(axis=1).min() and b <= off.max(axis=0).min()      # every node needs a way out and a way in
    # never worse than the identity ring or a greedy nearest-neighbour ring
    greedy, left = [0], set(range(1, n))
    while left:
        nxt = max(left, key=lambda v: w[greedy[-1], v])
        greedy.append(nxt)
        left.remove(nxt)
    assert b >= O.cycle_bottleneck(w.tolist(), greedy)
    assert b >= O.cycle_bottleneck(w.tolist(), list(range(n)))


def test_bad_arguments(B):
    with pytest.raises(B.DilocoError):
        B.ring_order(np.ones((21, 21)))
    with pytest.raises(B.DilocoError):
        B.ring_order(np.zeros((0, 0)))
    bad = np.ones((4, 4))
    bad[1, 2] = -1.0
    with pytest.raises(B.DilocoError):
        B.ring_order(bad)
    bad[1, 2] = np.nan
    with pytest.raises(B.DilocoError):
        B.ring_order(bad)
    bad[1, 2] = 1.0
    bad[2, 2] = np.nan                       # the diagonal is ignored
    assert B.ring_order(bad)[1] == 1.0
