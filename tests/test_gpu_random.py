"""Seeded random sweep of the device path: random graphs of three families (G(n,p) directed or not,
power-law cluster graphs, ragged batches of small graphs), random feature widths, random schedule
knobs (rows cut by source id, split rows, sub-group / workgroup threshold, unfused levels), every op
and dtype, HAG path and naive-CSR baseline, forward and backward, against the CPU oracle.

Bars as everywhere: int32 and max (values, argmax) bit-exact, fp32 sums within 1e-5 * sum|terms|.
Half of the max cases use quantised features, so that ties between original rows and aggregation
rows are common."""
import numpy as np
import pytest

import oracle
from paper_1906_03707_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 1e-5
KNOBS = ("HAG_PARTITION_MIN_ROWS", "HAG_PART_MIN", "HAG_PART_SHARE_PCT", "HAG_PART_MEAN_MIN", "HAG_PART_CLASS_SHIFT",
         "HAG_PART_SHIFT", "HAG_BLOCK_MAX", "HAG_SUB_MAX", "HAG_STAGE_EXTRA_ROWS")


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1906_03707_amd import binding
    binding.lib()
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.cpu().numpy()


def check_all(h, rowptr, col, d, seed, tag):
    n = rowptr.size - 1
    h.upload()
    x, gy = synth.features_f32(n, d, seed), synth.features_f32(n, d, seed + 1)
    xi, gi = synth.features_i32(n, d, seed + 2), synth.features_i32(n, d, seed + 3)
    xq = np.round(x * (1 + seed % 3)).astype(np.float32) + 0.0 if seed % 2 else x    # "+ 0.0": no -0.0
    for name, fwd, bwd in (("hag", h.forward, h.backward), ("naive", h.naive_forward, h.naive_backward)):
        for op in ("sum", "mean", "gcn"):
            y_ref, s, _ = oracle.naive_forward(rowptr, col, x, op)
            g_ref, gs = oracle.naive_backward(rowptr, col, gy, op)
            y = host(fwd(dev(x), op)).astype(np.float64)
            g = host(bwd(dev(gy), op)).astype(np.float64)
            assert np.all(np.abs(y - y_ref) <= TOL * s), (tag, name, op, "forward")
            assert np.all(np.abs(g - g_ref) <= TOL * gs), (tag, name, op, "backward")
        y_ref, _, am_ref = oracle.naive_forward(rowptr, col, xq, "max")
        y, am = fwd(dev(xq), "max")
        assert np.array_equal(host(y).astype(np.float64), y_ref) and np.array_equal(host(am), am_ref), (tag, name, "max f32")
        g_ref, gs = oracle.naive_backward(rowptr, col, gy, "max", am_ref)
        g = host(bwd(dev(gy), "max", argmax=am)).astype(np.float64)
        assert np.all(np.abs(g - g_ref) <= TOL * gs), (tag, name, "max backward")
        y_ref, _, _ = oracle.naive_forward(rowptr, col, xi, "sum")
        assert np.array_equal(host(fwd(dev(xi), "sum")), y_ref), (tag, name, "i32 sum")
        g_ref, _ = oracle.naive_backward(rowptr, col, gi, "sum")
        assert np.array_equal(host(bwd(dev(gi), "sum")), g_ref), (tag, name, "i32 sum backward")
        y_ref, _, am_ref = oracle.naive_forward(rowptr, col, xi, "max")
        y, am = fwd(dev(xi), "max")
        assert np.array_equal(host(y), y_ref) and np.array_equal(host(am), am_ref), (tag, name, "i32 max")


@pytest.mark.parametrize("chunk", range(4))
def test_random_graphs_widths_and_schedules(B, monkeypatch, chunk):
    rng = np.random.default_rng(20260 + chunk)
    for it in range(10):
        for k in KNOBS:
            monkeypatch.delenv(k, raising=False)
        env = {}
        if rng.random() < 0.5:
            env.update(HAG_PARTITION_MIN_ROWS="0", HAG_PART_MIN=str(rng.choice([4, 16, 64])), HAG_PART_SHARE_PCT="0",
                       HAG_PART_MEAN_MIN="0", HAG_PART_CLASS_SHIFT=str(rng.choice([-1, 0, 2, 5])),
                       HAG_PART_SHIFT=str(rng.integers(0, 8)))
        if rng.random() < 0.5:
            env["HAG_BLOCK_MAX"] = str(rng.choice([16, 40, 200]))
        if rng.random() < 0.4:
            env["HAG_SUB_MAX"] = str(rng.choice([4, 16, 100]))
        if rng.random() < 0.3:
            env["HAG_STAGE_EXTRA_ROWS"] = "-1000000"
        for k, v in env.items():
            monkeypatch.setenv(k, v)
        d = int(rng.choice([4, 8, 12, 16, 36, 64, 100, 128, 260]))
        kind = int(rng.integers(0, 3))
        if kind == 0:
            n = int(rng.integers(30, 1500))
            p = float(rng.uniform(0.01, 0.3)) if n < 400 else float(rng.uniform(0.005, 0.05))
            rowptr, col = synth.random_graph(n, p, seed=int(rng.integers(1 << 30)), directed=bool(rng.integers(0, 2)))
            h = B.hag_search(rowptr, col, int(n * rng.uniform(0, 1)))
        elif kind == 1:
            n = int(rng.integers(200, 2500))
            rowptr, col = synth.holme_kim(n, int(rng.integers(2, 12)), 0.5, seed=int(rng.integers(1 << 30)))
            h = B.hag_search(rowptr, col, n // int(rng.choice([2, 4, 8])))
        else:
            sizes = rng.integers(1, int(rng.choice([10, 40, 90])), size=int(rng.integers(70, 300)))
            rows, cols, off = [], [], 0
            for sz in sizes:
                m = np.triu(rng.random((sz, sz)) < rng.uniform(0.2, 0.9), 1)
                r, c = np.nonzero(m | m.T)
                rows.append(r + off)
                cols.append(c + off)
                off += sz
            rows, cols = np.concatenate(rows), np.concatenate(cols)
            rowptr = np.concatenate([[0], np.cumsum(np.bincount(rows, minlength=off))]).astype(np.int64)
            col = cols.astype(np.int32)
            graph_ptr = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
            h = B.hag_search_batched(rowptr, col, graph_ptr, float(rng.choice([0.25, 0.5])))
        st = h.stats()
        tag = f"chunk {chunk} case {it} family {kind} n={st['n']} e={st['e']} a={st['a']} levels={st['levels']} d={d} {env}"
        check_all(h, rowptr, col, d, int(rng.integers(1 << 30)), tag)
