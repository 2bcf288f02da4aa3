"""Oracle for the bandwidth-aware ring order (Section 2.5): the definition written out.

TEST INFRASTRUCTURE ONLY.  Enumerates every Hamiltonian cycle of the complete directed graph (node 0
fixed as the start, so (n - 1)! orders) and keeps the one whose slowest edge is fastest:
max over cycles C of min over edges (u, v) in C of w(u, v).  Feasible up to about n = 9.
"""
from itertools import permutations


def cycle_bottleneck(w, order):
    """Slowest directed edge of the ring order[0] -> order[1] -> ... -> order[-1] -> order[0]."""
    n = len(order)
    if n == 1:
        return float("inf")
    return min(w[order[i]][order[(i + 1) % n]] for i in range(n))


def best_ring(w):
    """(bottleneck, order) over all Hamiltonian cycles; w[u][v] = bandwidth from u to v."""
    n = len(w)
    best, best_order = None, None
    for rest in permutations(range(1, n)):
        order = (0,) + rest
        b = cycle_bottleneck(w, order)
        if best is None or b > best:
            best, best_order = b, list(order)
    return best, best_order
