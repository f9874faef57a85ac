"""HAGs of a sequential Aggregate (ordered neighbour lists): pins of the oracle (oracle/sequential.py) and
the library's host search (hag_seq_search) against it.  CPU only: there is no device path for sequential
aggregators."""
import os

import numpy as np
import pytest

from oracle import lstm
from oracle import sequential as S
from paper_1906_03707_amd import binding as B

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def ordered_graph(n, mean_len, seed, shared=0.7):
    """Ordered neighbour lists with shared prefixes: a list continues a random earlier list's prefix with
    probability `shared`, else draws fresh nodes (repeats allowed); some lists are empty or single."""
    rng = np.random.default_rng(seed)
    lists = []
    for v in range(n):
        k = int(rng.poisson(mean_len))
        if lists and rng.random() < shared:
            base = lists[int(rng.integers(len(lists)))]
            l = base[: int(rng.integers(0, len(base) + 1))]
        else:
            l = []
        while len(l) < k:
            l.append(int(rng.integers(n)))
        lists.append(l[:k] if k < len(l) else l)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    rowptr[1:] = np.cumsum([len(l) for l in lists])
    col = np.array([u for l in lists for u in l], dtype=np.int32)
    return rowptr, col


def parse_golden():
    nbrs, hag, merges, by_cap = {}, {}, [], None
    for line in open(os.path.join(GOLD, "seq_prefix_example.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, val = line.split(":", 1)
        if key.startswith("nbrs"):
            nbrs[int(key.split()[1])] = [int(t) for t in val.split()]
        elif key.startswith("hag"):
            hag[int(key.split()[1])] = [int(t) for t in val.split()]
        elif key == "merge":
            merges.append(tuple(int(t) for t in val.split()))
        elif key.startswith("aggregations by capacity"):
            by_cap = [int(t) for t in val.split()]
    n = len(nbrs)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    rowptr[1:] = np.cumsum([len(nbrs[v]) for v in range(n)])
    col = np.array([u for v in range(n) for u in nbrs[v]], dtype=np.int32)
    return rowptr, col, merges, [hag[v] for v in range(n)], by_cap


def library_search(rowptr, col, capacity):
    left, right, red, hrowptr, hcol = B.hag_seq_search(rowptr, col, capacity)
    merges = [(int(a), int(b), int(c)) for a, b, c in zip(left, right, red)]
    lists = [list(map(int, hcol[hrowptr[v]:hrowptr[v + 1]])) for v in range(rowptr.size - 1)]
    return merges, lists


def test_hand_worked_example_oracle_and_library():
    rowptr, col, merges, hag, by_cap = parse_golden()
    for cap, want in enumerate(by_cap):
        for search in (S.search, library_search):
            m, l = search(rowptr, col, cap)
            assert m == merges[:min(cap, len(merges))]
            assert S.aggregations(m, l) == want
            assert S.cover_check(rowptr, col, m, l) == 0
    m, l = library_search(rowptr, col, 99)
    assert l == hag and S.distinct_prefixes(rowptr, col) == by_cap[-1]


def test_ordered_cover_catches_planted_errors():
    rowptr, col, merges, hag, _ = parse_golden()
    assert S.cover_check(rowptr, col, merges, hag) == 0
    swapped = [list(l) for l in hag]
    swapped[3] = [3, 4]                                    # right members, wrong order
    assert S.cover_check(rowptr, col, merges, swapped) == 4
    assert S.cover_check(rowptr, col, [(4, 3, 3), merges[1]], hag) == 1        # the pair of w6 the other way round
    short = [list(l) for l in hag]
    short[0] = [6]                                         # a member dropped
    assert S.cover_check(rowptr, col, merges, short) == 1
    assert S.cover_check(rowptr, col, [(3, 7, 3), merges[1]], hag) == -1       # refers to a node created later


@pytest.mark.parametrize("seed", range(8))
def test_library_search_equals_brute_force(seed):
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(5, 120))
    rowptr, col = ordered_graph(n, float(rng.uniform(1, 8)), seed, shared=float(rng.uniform(0.2, 0.9)))
    e = int(rowptr[-1])
    for cap in (0, 1, 3, n // 2, e + 5):
        m_o, l_o = S.search(rowptr, col, cap)
        m_l, l_l = library_search(rowptr, col, cap)
        assert m_l == m_o and l_l == l_o
        assert S.cover_check(rowptr, col, m_l, l_l) == 0
        # per-merge accounting: a merge of redundancy r saves r - 1 aggregations; r never grows
        reds = [r for _, _, r in m_l]
        assert all(r >= 2 for r in reds)
        naive = sum(max(int(k) - 1, 0) for k in np.diff(rowptr))
        assert S.aggregations(m_l, l_l) == naive - sum(r - 1 for r in reds)
        # only a list's first entry can be an aggregation node
        assert all(x < n for l in l_l for x in l[1:])


@pytest.mark.parametrize("seed", range(4))
def test_theorem3_global_optimum_with_enough_capacity(seed):
    # With capacity >= |E| Algorithm 3 reaches the lower bound of Theorem 3's proof: one aggregation per
    # distinct prefix of length >= 2.  The bound is counted here directly, with a set of tuples.
    rowptr, col = ordered_graph(1500, 6.0, 200 + seed, shared=0.8)
    merges, lists = library_search(rowptr, col, int(rowptr[-1]))
    assert S.aggregations(merges, lists) == S.distinct_prefixes(rowptr, col)
    assert S.cover_check(rowptr, col, merges, lists) == 0
    # and any smaller capacity gives a prefix of the same merge list with more aggregations left
    half, lists_half = library_search(rowptr, col, len(merges) // 2)
    assert half == merges[:len(merges) // 2] and S.aggregations(half, lists_half) > S.aggregations(merges, lists)


def test_equivalent_hag_gives_identical_states():
    # same operations in the same order: the sequential toy aggregator gives bit-identical results
    rowptr, col = ordered_graph(300, 5.0, 300, shared=0.8)
    x = np.random.default_rng(301).standard_normal((300, 4)).astype(np.float32)
    merges, lists = library_search(rowptr, col, 10**6)
    assert len(merges) > 20
    assert np.array_equal(S.naive_forward(rowptr, col, x), S.hag_forward(300, merges, lists, x))
    # a planted order swap inside one list changes the result
    v = next(i for i, l in enumerate(lists) if len(l) >= 3 and l[1] != l[2])
    bad = [list(l) for l in lists]
    bad[v][1], bad[v][2] = bad[v][2], bad[v][1]
    assert not np.array_equal(S.naive_forward(rowptr, col, x), S.hag_forward(300, merges, bad, x))


def test_invalid_input_is_rejected():
    with pytest.raises(B.HagError):
        B.hag_seq_search(np.array([0, 2, 1], dtype=np.int64), np.array([0, 1], dtype=np.int32), 1)
    with pytest.raises(B.HagError):
        B.hag_seq_search(np.array([0, 1], dtype=np.int64), np.array([5], dtype=np.int32), 1)


def test_lstm_plan_counts_match_the_oracle():
    # hag_seq_create (host part of the device path): cell evaluations, aggregation nodes and the length of the
    # longest chain of evaluations, against the oracle's execution of the same prefix HAG
    rng = np.random.default_rng(5)
    n = 80
    routes = [rng.permutation(n)[:8] for _ in range(4)]
    rowptr, col = [0], []
    for v in range(n):
        col += list(routes[int(rng.integers(0, 4))][:int(rng.integers(0, 9))]) + list(rng.integers(0, n, int(rng.integers(0, 3))))
        rowptr.append(len(col))
    rowptr, col = np.asarray(rowptr, dtype=np.int64), np.asarray(col, dtype=np.int32)
    x = rng.normal(size=(n, 3))
    w_ih, w_hh, b = rng.normal(size=(8, 3)), rng.normal(size=(8, 2)), rng.normal(size=8)
    longest = int(np.diff(rowptr).max())
    for cap in (0, 3, col.size):
        plan = B.SeqHag(rowptr, col, cap)
        merges, lists = S.search(rowptr, col, cap)
        if cap == 0:
            assert (plan.cells, plan.merges) == (col.size, 0)
        else:
            _, cells = lstm.hag_aggregate(n, merges, lists, x, w_ih, w_hh, b)
            assert (plan.cells, plan.merges) == (cells, len(merges))
        # sharing never lengthens a chain: the state after k elements is still k evaluations deep
        assert plan.ranks == longest
        # one launch per depth of the shared prefixes, one more for the private remainders
        private = any(len(l) > (1 if cap else 0) for l in lists)
        assert plan.launches >= int(private) and plan.launches <= longest + 1
        if cap == 0:
            assert plan.launches == 1


def replay_plan(plan, n, x, w_ih, w_hh, b, order=0):
    """The plan of hag_seq_create executed step by step with the oracle's cell, one level after the other, checking
    on the way what the device relies on: a path starts only from a state that an EARLIER group (order 0: level,
    order 1: depth of the start state) has written, every
    state row is written at most once, paths of a level are sorted by length."""
    n_states, paths, step_x, step_out, level_ptr, final_state = plan.plan(order)
    hidden = w_hh.shape[1]
    h_rows, c_rows = np.full((max(n_states, 1), hidden), np.nan), np.full((max(n_states, 1), hidden), np.nan)
    written_at = np.full(max(n_states, 1), -1)
    out = np.zeros((n, hidden))
    by_path = np.zeros(n, dtype=bool)
    assert level_ptr[0] == 0 and level_ptr[-1] == len(paths)
    for level in range(len(level_ptr) - 1):
        lens = paths[level_ptr[level]:level_ptr[level + 1], 2]
        assert (np.diff(lens) <= 0).all() and (lens >= 1).all()
        for start, beg, length, node in paths[level_ptr[level]:level_ptr[level + 1]]:
            if start >= 0:
                assert 0 <= written_at[start] < level
                h, c = h_rows[start], c_rows[start]
            else:
                h, c = np.zeros(hidden), np.zeros(hidden)
            for t in range(beg, beg + length):
                assert 0 <= step_x[t] < n
                h, c = lstm.cell(x[step_x[t]], h, c, w_ih, w_hh, b)
                if step_out[t] >= 0:
                    assert written_at[step_out[t]] < 0
                    written_at[step_out[t]] = level
                    h_rows[step_out[t]], c_rows[step_out[t]] = h, c
            if node >= 0:
                assert final_state[node] == -2 and not by_path[node]
                by_path[node] = True
                out[node] = h
    for v in range(n):
        if final_state[v] >= 0:
            assert written_at[final_state[v]] >= 0
            out[v] = h_rows[final_state[v]]
        else:
            assert (final_state[v] == -2) == by_path[v]
    return out, int(paths[:, 2].sum()), int((step_out >= 0).sum())


@pytest.mark.parametrize("seed", [5, 6, 7])
def test_lstm_plan_replayed_on_the_host_equals_the_naive_walk(seed):
    rng = np.random.default_rng(seed)
    n = 90
    routes = [rng.permutation(n)[:9] for _ in range(5)]
    rowptr, col = [0], []
    for v in range(n):
        col += list(routes[int(rng.integers(0, 5))][:int(rng.integers(0, 10))]) + list(rng.integers(0, n, int(rng.integers(0, 4))))
        rowptr.append(len(col))
    rowptr, col = np.asarray(rowptr, dtype=np.int64), np.asarray(col, dtype=np.int32)
    x = rng.normal(size=(n, 3))
    w_ih, w_hh, b = rng.normal(0, 0.5, (8, 3)), rng.normal(0, 0.5, (8, 2)), rng.normal(0, 0.5, 8)
    want, _ = lstm.naive_aggregate(rowptr, col, x, w_ih, w_hh, b)
    for cap in (0, 4, col.size):
        plan = B.SeqHag(rowptr, col, cap)
        got, cells, kept = replay_plan(plan, n, x, w_ih, w_hh, b)
        assert np.array_equal(got, want)                  # the same cells in the same order along every list
        got1, cells1, kept1 = replay_plan(plan, n, x, w_ih, w_hh, b, order=1)      # the order of the one-launch pass
        assert np.array_equal(got1, want) and (cells1, kept1) == (cells, kept)
        assert sorted(map(tuple, plan.plan(0)[1])) == sorted(map(tuple, plan.plan(1)[1]))   # the same paths, regrouped
        assert cells == plan.cells
        if cap == 0:
            assert kept == 0 and plan.launches == (1 if col.size else 0)
        else:
            assert kept < plan.cells                      # most states never leave the path that computes them


def test_lstm_plan_of_degenerate_inputs():
    # no nodes, no lists, one-entry lists, one list far longer than the rest, one node repeated: the plan replayed on the host
    rng = np.random.default_rng(3)
    cases = {
        "all empty": (np.zeros(6, dtype=np.int64), np.zeros(0, dtype=np.int32)),
        "one entry each": (np.arange(0, 41, dtype=np.int64), rng.integers(0, 5, 40).astype(np.int32)),
        "one long list": (np.concatenate([[0], np.cumsum([300] + [2] * 99)]).astype(np.int64),
                          np.concatenate([rng.integers(0, 100, 300), np.tile([7, 9], 99)]).astype(np.int32)),
        "one node repeated": (np.array([0, 50, 75, 75], dtype=np.int64), np.full(75, 2, dtype=np.int32)),
    }
    w_ih, w_hh, b = rng.normal(0, 0.4, (8, 3)), rng.normal(0, 0.4, (8, 2)), rng.normal(0, 0.4, 8)
    for name, (rowptr, col) in cases.items():
        n = rowptr.size - 1
        x = rng.normal(size=(n, 3))
        want, cells_naive = lstm.naive_aggregate(rowptr, col, x, w_ih, w_hh, b)
        for cap in (0, max(n // 4, 1), max(int(col.size), 1)):
            plan = B.SeqHag(rowptr, col, cap)
            assert plan.cells <= cells_naive and plan.ranks == (int(np.diff(rowptr).max()) if col.size else 0)
            for order in (0, 1):
                got, cells, _ = replay_plan(plan, n, x, w_ih, w_hh, b, order)
                assert np.array_equal(got, want), (name, cap, order)
                assert cells == plan.cells
    empty = B.SeqHag(np.zeros(1, dtype=np.int64), np.zeros(0, dtype=np.int32), 4)
    assert (empty.cells, empty.launches, empty.ranks) == (0, 0, 0)


def test_lstm_workspace_sizes():
    # host arithmetic only: the training workspace holds the forward one plus 24 H bytes per cell and more; unsupported
    # sizes give 0
    rng = np.random.default_rng(2)
    rowptr = np.concatenate([[0], np.cumsum(rng.integers(0, 6, 50))]).astype(np.int64)
    col = rng.integers(0, 50, rowptr[-1]).astype(np.int32)
    plan = B.SeqHag(rowptr, col, 10)
    for d, hidden in ((8, 8), (64, 64), (128, 128), (100, 24)):
        fwd, train = plan.workspace_bytes(d, hidden), plan.train_workspace_bytes(d, hidden)
        assert fwd > 0 and train >= fwd + plan.cells * 24 * hidden
    assert plan.train_workspace_bytes(8, 136) == 0 and plan.train_workspace_bytes(200, 64) == 0 and plan.train_workspace_bytes(6, 8) == 0
