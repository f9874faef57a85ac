"""Seeded random sweep of the search (host logic, no GPU): Algorithm 3 as the library runs it
(lazy bounds, candidate lists, thresholded sweeps) against the oracle's brute force, on graphs of
four families, with capacities up to 3|V| so that most searches run until no pair is shared twice,
and with the laziness knobs (candidates kept per node, sweep threshold) varied: whatever the
laziness, the merge list must be the same."""
import numpy as np
import pytest

import oracle
from paper_1906_03707_amd import binding as B
from paper_1906_03707_amd import synth


@pytest.mark.parametrize("chunk", range(4))
def test_random_searches_match_brute_force(monkeypatch, chunk):
    rng = np.random.default_rng(31000 + chunk)
    for it in range(10):
        kind = int(rng.integers(0, 4))
        seed = int(rng.integers(1 << 30))
        if kind == 0:
            rowptr, col = synth.random_graph(int(rng.integers(20, 300)), float(rng.uniform(0.02, 0.5)), seed=seed,
                                             directed=bool(rng.integers(0, 2)))
        elif kind == 1:
            rowptr, col = synth.holme_kim(int(rng.integers(100, 900)), int(rng.integers(2, 10)), float(rng.uniform(0, 1)), seed=seed)
        elif kind == 2:
            rowptr, col = synth.sbm(n_blocks=int(rng.integers(2, 8)), block=int(rng.integers(10, 90)),
                                    p_in=float(rng.uniform(0.1, 0.8)), p_out=float(rng.uniform(0, 0.05)), seed=seed)
        else:
            rowptr, col = synth.dcsbm(n=int(rng.integers(400, 1300)), n_blocks=int(rng.integers(2, 10)),
                                      mean_degree=float(rng.uniform(6, 20)), seed=seed)
        n = rowptr.size - 1
        cap = int(rng.choice([n // 2, n, 2 * n, 3 * n]))
        keep, pct = int(rng.choice([1, 2, 4, 12, 12])), int(rng.choice([50, 50, 65, 30, 90]))
        monkeypatch.setenv("HAG_SEARCH_KEEP", str(keep))
        monkeypatch.setenv("HAG_SEARCH_THETA_PCT", str(pct))
        ref = oracle.search(rowptr, col, cap)
        left, right, red = B.hag_search(rowptr, col, cap).get_merges()
        tag = f"chunk {chunk} case {it} family {kind} n={n} e={col.size} capacity={cap} keep={keep} pct={pct}"
        assert ref.a == left.size, tag
        assert np.array_equal(left, ref.left) and np.array_equal(right, ref.right) and np.array_equal(red, ref.red), tag
