// Bandwidth-aware ring order (Section 2.5): among all Hamiltonian cycles of the complete directed
// graph whose edge (u, v) carries the measured bandwidth from node u to node v, find one whose
// slowest edge is as fast as possible.  Host code only; nothing here touches the device.
//
// Method.  The answer is one of the n (n - 1) edge weights.  For a threshold t the question "is
// there a Hamiltonian cycle using only edges of weight >= t" is monotone in t, so a binary search
// over the sorted distinct weights finds the largest feasible t.  Feasibility is the classic subset
// recurrence with node 0 as the fixed start: ends[S] = set of nodes v such that some path
// 0 -> ... -> v visits exactly the nodes of S; ends[S + u] gains u when u has an allowed edge from a
// member of ends[S].  Sets are machine words, so one threshold costs O(2^(n-1) n) word operations
// (n = 16: half a million), and the whole search a few milliseconds.
#include <math.h>
#include <stdint.h>

#include <algorithm>
#include <vector>

#include "../../include/diloco_mi355.h"

namespace {

struct Graph {
    uint32_t n;
    uint32_t in_mask[DILOCO_MAX_RING_NODES];    // in_mask[u]: nodes p with an allowed edge p -> u
};

Graph allowed_edges(const double* w, uint32_t n, double t) {
    Graph g;
    g.n = n;
    for (uint32_t u = 0; u < n; ++u) {
        uint32_t m = 0;
        for (uint32_t p = 0; p < n; ++p)
            if (p != u && w[(size_t)p * n + u] >= t) m |= 1u << p;
        g.in_mask[u] = m;
    }
    return g;
}

// Fills ends[S] for every subset S (as a bit set over all n nodes) that contains node 0.
// Returns true when a Hamiltonian cycle exists.
bool hamiltonian(const Graph& g, std::vector<uint32_t>& ends) {
    const uint32_t n = g.n, full = (n == 32 ? 0xffffffffu : (1u << n) - 1u);
    std::fill(ends.begin(), ends.end(), 0u);
    ends[1] = 1u;                                          // the path that is just node 0
    for (uint32_t S = 1; S <= full; S += 2) {              // odd S: contains node 0
        const uint32_t e = ends[S];
        if (!e) continue;
        for (uint32_t rest = full & ~S; rest; rest &= rest - 1) {
            const uint32_t u = (uint32_t)__builtin_ctz(rest);
            if (e & g.in_mask[u]) ends[S | (1u << u)] |= 1u << u;
        }
        if (S == full) break;
    }
    return (ends[full] & g.in_mask[0]) != 0;               // close the cycle back into node 0
}

void read_cycle(const Graph& g, const std::vector<uint32_t>& ends, uint32_t* order) {
    const uint32_t n = g.n, full = (1u << n) - 1u;
    uint32_t S = full;
    uint32_t v = (uint32_t)__builtin_ctz(ends[full] & g.in_mask[0]);
    for (uint32_t pos = n - 1; pos >= 1; --pos) {
        order[pos] = v;
        const uint32_t prev_set = S & ~(1u << v);
        const uint32_t p = (uint32_t)__builtin_ctz(ends[prev_set] & g.in_mask[v]);
        S = prev_set;
        v = p;
    }
    order[0] = 0;
}

}  // namespace

extern "C" int32_t diloco_ring_order(const double* bandwidth, uint32_t n, uint32_t* order_out,
                                     double* bottleneck_out) {
    if (!bandwidth || !order_out) return DILOCO_ERR_NULL;
    if (n < 1 || n > DILOCO_MAX_RING_NODES) return DILOCO_ERR_SIZE;
    for (uint32_t u = 0; u < n; ++u)
        for (uint32_t v = 0; v < n; ++v)
            if (u != v && !(bandwidth[(size_t)u * n + v] >= 0.0 && isfinite(bandwidth[(size_t)u * n + v])))
                return DILOCO_ERR_SIZE;
    if (n == 1) {
        order_out[0] = 0;
        if (bottleneck_out) *bottleneck_out = INFINITY;    // a ring of one node has no edge
        return DILOCO_OK;
    }
    std::vector<double> weights;
    weights.reserve((size_t)n * (n - 1));
    for (uint32_t u = 0; u < n; ++u)
        for (uint32_t v = 0; v < n; ++v)
            if (u != v) weights.push_back(bandwidth[(size_t)u * n + v]);
    std::sort(weights.begin(), weights.end());
    weights.erase(std::unique(weights.begin(), weights.end()), weights.end());

    std::vector<uint32_t> ends((size_t)1 << n);
    // weights[0] (every edge allowed) is always feasible: the graph is complete
    size_t lo = 0, hi = weights.size() - 1;
    while (lo < hi) {
        const size_t mid = lo + (hi - lo + 1) / 2;
        if (hamiltonian(allowed_edges(bandwidth, n, weights[mid]), ends))
            lo = mid;
        else
            hi = mid - 1;
    }
    const Graph g = allowed_edges(bandwidth, n, weights[lo]);
    if (!hamiltonian(g, ends)) return DILOCO_ERR_SIZE;      // cannot happen on a complete graph
    read_cycle(g, ends, order_out);
    if (bottleneck_out) *bottleneck_out = weights[lo];
    return DILOCO_OK;
}
