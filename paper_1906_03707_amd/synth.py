"""Seeded synthetic inputs: graphs, features and upstream gradients.

This module holds no aggregation or search arithmetic; it only draws inputs, so
both the CPU oracle's tests and the HIP library's tests may use it.  The graphs
stand in for the datasets of the paper's Table 2 (node counts and degree
structure only); none of those datasets is reproduced here.

Every graph is undirected (symmetric CSR), has no self-loops and no duplicate
edges, and lists the in-neighbours of each row in ascending order.
CSR convention: ``rowptr`` int64 [n+1], ``col`` int32 [E]; rows are
destinations, columns are in-neighbours.
"""
from __future__ import annotations

import numpy as np

SEED_BASE = 190603707  # + config id; features +1000, gradients +2000


def _csr_from_undirected(n: int, a: np.ndarray, b: np.ndarray):
    """Symmetrise unique undirected pairs (a<b) into a sorted CSR."""
    import scipy.sparse as sp

    r = np.concatenate([a, b])
    c = np.concatenate([b, a])
    m = sp.coo_matrix((np.ones(r.size, dtype=np.int8), (r, c)), shape=(n, n)).tocsr()
    m.sort_indices()
    return m.indptr.astype(np.int64), m.indices.astype(np.int32)


def _unique_pairs(n: int, a: np.ndarray, b: np.ndarray):
    lo = np.minimum(a, b).astype(np.int64)
    hi = np.maximum(a, b).astype(np.int64)
    keep = lo != hi
    key = np.unique(lo[keep] * n + hi[keep])
    return (key // n), (key % n)


def sbm(n_blocks=32, block=128, p_in=0.2, p_out=0.001, seed=SEED_BASE + 1):
    """Stochastic block model (config 1)."""
    rng = np.random.default_rng(seed)
    n = n_blocks * block
    blk = np.arange(n) // block
    u = rng.random((n, n), dtype=np.float32)
    p = np.where(blk[:, None] == blk[None, :], np.float32(p_in), np.float32(p_out))
    iu, ju = np.nonzero(np.triu(u < p, k=1))
    return _csr_from_undirected(n, iu, ju)


def holme_kim(n=56944, m=14, p_triad=0.5, seed=SEED_BASE + 2):
    """Power-law cluster graph (config 2): growth with preferential attachment,
    each further link of a new node closing a triangle with probability p_triad."""
    rng = np.random.default_rng(seed)
    # draw all random numbers up front; the loop only consumes them
    nbrs = [[] for _ in range(n)]
    repeated = list(range(m))  # one entry per edge endpoint (+ the m seed nodes once)
    r_pick = rng.random((n, 4 * m))
    r_triad = rng.random((n, m))
    src_l, dst_l = [], []
    for v in range(m, n):
        targets = set()
        k = 0
        rp = r_pick[v]
        t = repeated[int(rp[k] * len(repeated))]
        k += 1
        targets.add(t)
        last = t
        count = 1
        while count < m:
            cand = -1
            if r_triad[v, count] < p_triad and nbrs[last]:
                nb = nbrs[last]
                c = nb[int(rp[k % rp.size] * len(nb))]
                k += 1
                if c != v and c not in targets:
                    cand = c
            if cand < 0:
                tries = 0
                while True:
                    c = repeated[int(rp[k % rp.size] * len(repeated))]
                    k += 1
                    tries += 1
                    if c not in targets:
                        cand = c
                        break
                    if tries > 64:  # pathological: fall back to a fresh draw
                        rp = rng.random(rp.size)
                        tries = 0
            targets.add(cand)
            last = cand
            count += 1
        for t in targets:
            nbrs[v].append(t)
            nbrs[t].append(v)
            src_l.append(v)
            dst_l.append(t)
        repeated.extend(targets)
        repeated.extend([v] * m)
    a, b = _unique_pairs(n, np.asarray(src_l), np.asarray(dst_l))
    return _csr_from_undirected(n, a, b)


def dcsbm(n=232965, n_blocks=41, zipf=1.1, mean_degree=490.0, intra=0.8, gamma=2.2,
          seed=SEED_BASE + 3):
    """Degree-corrected stochastic block model (configs 3 and 5).

    Block sizes follow rank^-zipf; node weights follow a power law with exponent
    gamma, truncated so that no expected degree exceeds n/10; a fraction `intra`
    of the edge draws has both endpoints in one block.  Endpoints are drawn in
    proportion to node weight.  Duplicates and loops are dropped and the draw is
    repeated until the target number of distinct undirected edges is reached."""
    rng = np.random.default_rng(seed)
    w = 1.0 / np.arange(1, n_blocks + 1) ** zipf
    sizes = np.floor(w / w.sum() * n).astype(np.int64)
    sizes[0] += n - sizes.sum()
    blk = np.repeat(np.arange(n_blocks), sizes)            # nodes are numbered block-major
    theta = (1.0 - rng.random(n)) ** (-1.0 / (gamma - 1.0))  # Pareto, density ~ theta^-gamma
    cap = (n / 10.0) / mean_degree * theta.mean()
    for _ in range(8):                                      # truncate, then re-centre
        theta = np.minimum(theta, cap)
        cap = (n / 10.0) / mean_degree * theta.mean()
    cum = np.cumsum(theta)
    total = cum[-1]
    starts = np.concatenate([[0], np.cumsum(sizes)])
    blk_lo = np.concatenate([[0.0], cum[starts[1:] - 1]])   # weight before each block
    blk_w = np.diff(blk_lo)
    target = int(round(n * mean_degree / 2.0))
    keys = np.empty(0, dtype=np.int64)
    need = target
    while keys.size < target:
        draw = int(need * 1.08) + 1024
        a = np.searchsorted(cum, rng.random(draw) * total, side="right").astype(np.int64)
        np.minimum(a, n - 1, out=a)
        is_intra = rng.random(draw) < intra
        ba = blk[a]
        # intra: second endpoint by weight inside the first endpoint's block
        pos_in = blk_lo[ba] + rng.random(draw) * blk_w[ba]
        # inter: second endpoint by weight over the whole graph, other block required
        pos_out = rng.random(draw) * total
        b = np.searchsorted(cum, np.where(is_intra, pos_in, pos_out), side="right").astype(np.int64)
        np.minimum(b, n - 1, out=b)
        ok = (a != b) & (is_intra | (blk[b] != ba))
        lo = np.minimum(a[ok], b[ok])
        hi = np.maximum(a[ok], b[ok])
        keys = np.union1d(keys, lo * n + hi)
        need = max(target - keys.size, 0)
        del a, b, ba, pos_in, pos_out, ok, lo, hi, is_intra
    if keys.size > target:
        keys = np.sort(rng.choice(keys, size=target, replace=False))
    return _csr_from_undirected(n, keys // n, keys % n)


def er_batch(n_graphs=5000, size=74, p=0.9, seed=SEED_BASE + 4):
    """Batch of disjoint Erdos-Renyi graphs, block-diagonal CSR, graph-major ids (config 4).

    Returns (rowptr, col, graph_ptr) with graph_ptr int64 [n_graphs+1]."""
    rng = np.random.default_rng(seed)
    iu, ju = np.triu_indices(size, k=1)
    hit = rng.random((n_graphs, iu.size), dtype=np.float32) < np.float32(p)
    g, e = np.nonzero(hit)
    a = g.astype(np.int64) * size + iu[e]
    b = g.astype(np.int64) * size + ju[e]
    n = n_graphs * size
    rowptr, col = _csr_from_undirected(n, a, b)
    return rowptr, col, np.arange(n_graphs + 1, dtype=np.int64) * size


def random_graph(n, p, seed, directed=False):
    """Small G(n,p) graph for property tests; directed=True gives an unsymmetric CSR."""
    rng = np.random.default_rng(seed)
    m = rng.random((n, n)) < p
    np.fill_diagonal(m, False)
    if not directed:
        m = np.triu(m, 1)
        m = m | m.T
    rows, cols = np.nonzero(m)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(np.bincount(rows, minlength=n), out=rowptr[1:])
    return rowptr, cols.astype(np.int32)


def features_f32(n, d, seed):
    """N(0,1) fp32 features; -0.0 never occurs (values are compared bit-wise for max)."""
    x = np.random.default_rng(seed).standard_normal((n, d), dtype=np.float32)
    x += np.float32(0.0)  # turns -0.0 into +0.0
    return x


def features_i32(n, d, seed, lo=-1000, hi=1000):
    return np.random.default_rng(seed).integers(lo, hi + 1, size=(n, d), dtype=np.int32)


CONFIGS = {
    1: dict(name="sbm4096", d=64, ops=("sum",), capacity_div=4),
    2: dict(name="holme_kim56944", d=128, ops=("sum", "mean"), capacity_div=4),
    3: dict(name="dcsbm232965", d=128, ops=("sum",), capacity_div=4),
    4: dict(name="er_batch5000x74", d=64, ops=("sum",), capacity_div=4),
    5: dict(name="dcsbm232965_sweep", d=(16, 128, 512), ops=("max", "sum"), capacity_div=(0, 8, 4, 2)),
}


def graph_for_config(cfg: int):
    """(rowptr, col, graph_ptr or None) of benchmark config `cfg` (1-based)."""
    if cfg == 1:
        return (*sbm(), None)
    if cfg == 2:
        return (*holme_kim(), None)
    if cfg in (3, 5):
        return (*dcsbm(), None)
    if cfg == 4:
        return er_batch()
    raise ValueError(cfg)
