"""CPU oracle for HAGs of a SEQUENTIAL Aggregate -- TEST INFRASTRUCTURE ONLY (plain Python, small graphs).

Follows the paper's treatment of ordered neighbour lists: Algorithm 3 with the sequential branch
of Redundancy (nodes whose list starts with the pair), the ordered cover of Equation 2, the
execution order of Algorithm 2.  Nothing here is shared with the library.

Conventions where the paper is silent or loose (each is a reading, listed in the design notes):
  * N(v) is an ordered list (a node may occur in it more than once).
  * Redundancy(v1, v2) counts the u in V whose CURRENT list starts with (v1, v2): the listing writes
    cover(u)[1], cover(u)[2], but aggregation nodes stand for the prefixes they cover, so the first
    two in-neighbours of u in the HAG are what can be merged.
  * The rewrite loop replaces the leading pair (v1, v2) of exactly those lists by the new node w.
  * Stop when the best redundancy is <= 1; ties go to the lexicographically smallest (v1, v2).
  * Unified ids: originals 0..n-1, aggregation nodes n.. in creation order; w = (v1, v2) means
    "the state after v1's sequence, then v2".
"""
from __future__ import annotations

import numpy as np


def lists_of(rowptr, col):
    return [list(map(int, col[rowptr[v]:rowptr[v + 1]])) for v in range(rowptr.size - 1)]


def redundancy(lists, v1, v2):
    """Redundancy(v1, v2) of Algorithm 3 for a sequential Aggregate."""
    return sum(1 for l in lists if len(l) >= 2 and l[0] == v1 and l[1] == v2)


def search(rowptr, col, capacity):
    """Algorithm 3, sequential case, by brute force: every leading pair recounted in every iteration.

    Returns (merges [(v1, v2, redundancy)], final ordered lists)."""
    n = rowptr.size - 1
    lists = lists_of(rowptr, col)
    merges = []
    while len(merges) < capacity:
        count = {}
        for l in lists:
            if len(l) >= 2:
                count[(l[0], l[1])] = count.get((l[0], l[1]), 0) + 1
        if not count:
            break
        best = max(count.values())
        if best <= 1:
            break
        v1, v2 = min(k for k, c in count.items() if c == best)
        w = n + len(merges)
        for l in lists:
            if len(l) >= 2 and l[0] == v1 and l[1] == v2:
                l[:2] = [w]
        merges.append((v1, v2, best))
    return merges, lists


def cover(n, merges, x):
    """Equation 2: the ordered list of original nodes that HAG node x stands for."""
    if x < n:
        return [x]
    v1, v2 = merges[x - n][0], merges[x - n][1]
    return cover(n, merges, v1) + cover(n, merges, v2)


def cover_check(rowptr, col, merges, lists):
    """Theorem 2 for ordered covers: expanding the HAG list of every v must give N(v), in order.

    0 = equivalent, 1 + v = first node whose cover differs, -1 = malformed (a merge refers to a later node)."""
    n = rowptr.size - 1
    for i, m in enumerate(merges):
        if not (0 <= m[0] < n + i and 0 <= m[1] < n + i):
            return -1
    orig = lists_of(rowptr, col)
    for v in range(n):
        got = []
        for x in lists[v]:
            if not 0 <= x < n + len(merges):
                return -1
            got += cover(n, merges, x)
        if got != orig[v]:
            return 1 + v
    return 0


def aggregations(merges, lists):
    """Binary aggregations of a HAG (Section 4.1): k in-neighbours cost k - 1; an aggregation node has two."""
    return sum(max(len(l) - 1, 0) for l in lists) + len(merges)


def distinct_prefixes(rowptr, col):
    """Number of distinct prefixes of length >= 2 over all neighbour lists: the lower bound of Theorem 3's proof."""
    seen = set()
    for l in lists_of(rowptr, col):
        for i in range(2, len(l) + 1):
            seen.add(tuple(l[:i]))
    return len(seen)


# An order-dependent aggregator for equivalence tests: s_1 = tanh(x_1), s_i = tanh(0.5 s_{i-1} + x_i - 0.25 s_{i-1} x_i).
def _start(x):
    return np.tanh(x)


def _step(s, x):
    return np.tanh(0.5 * s + x - 0.25 * s * x)


def naive_forward(rowptr, col, x):
    """Algorithm 1's Aggregate line with the sequential toy aggregator, list order, fp64."""
    n = rowptr.size - 1
    y = np.zeros((n, x.shape[1]), dtype=np.float64)
    for v, l in enumerate(lists_of(rowptr, col)):
        if l:
            s = _start(x[l[0]].astype(np.float64))
            for u in l[1:]:
                s = _step(s, x[u].astype(np.float64))
            y[v] = s
    return y


def hag_forward(n, merges, lists, x):
    """Algorithm 2 over a sequential HAG: aggregation nodes in creation order hold prefix states."""
    state = {}

    def value(u):                      # state after u's sequence
        return _start(x[u].astype(np.float64)) if u < n else state[u]

    for i, (v1, v2, _) in enumerate(merges):
        assert v2 < n, "only the first element of a list can be an aggregation node"
        state[n + i] = _step(value(v1), x[v2].astype(np.float64))
    y = np.zeros((n, x.shape[1]), dtype=np.float64)
    for v, l in enumerate(lists):
        if l:
            s = value(l[0])
            for u in l[1:]:
                assert u < n
                s = _step(s, x[u].astype(np.float64))
            y[v] = s
    return y
