"""Pins of the layer-level oracle (oracle/layers.py): a hand-worked GraphSAGE-P layer, finite differences,
the C oracle's aggregations (themselves pinned against scipy), and a dense-matrix form of the GCN layer."""
import os

import numpy as np
import scipy.sparse as sp

import oracle
from oracle import layers as L
from paper_1906_03707_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def parse(name):
    out, nbrs = {}, {}
    for line in open(os.path.join(GOLD, name)):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, val = line.split(":", 1)
        if key.startswith("nbrs"):
            nbrs[int(key.split()[1])] = [int(t) for t in val.split()]
        else:
            out[key] = np.array([[float(t) for t in row.split()] for row in val.split(";")])
    n = len(nbrs)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    col = []
    for v in range(n):
        col += nbrs[v]
        rowptr[v + 1] = len(col)
    return rowptr, np.array(col, dtype=np.int32), out


def test_sage_pool_layer_hand_worked_example():
    rowptr, col, g = parse("sage_pool_path3.txt")
    out, ctx = L.sage_pool_layer(rowptr, col, g["h"], g["w1"], g["w2"])
    assert np.array_equal(np.maximum(ctx["pre_p"], 0), g["p"])
    assert np.array_equal(ctx["cat"][:, :2], g["a"]) and np.array_equal(ctx["arg"], g["argmax"].astype(np.int64))
    assert np.array_equal(out, g["out"])
    g_h, g_w1, g_w2 = L.sage_pool_layer_backward(ctx, np.ones_like(out))
    assert np.array_equal(g_h, g["g_h"]) and np.array_equal(g_w1, g["g_w1"]) and np.array_equal(g_w2, g["g_w2"])


def test_max_pool_aggregate_matches_c_oracle_incl_ties_and_empty_rows():
    rowptr, col = synth.random_graph(60, 0.03, seed=5, directed=True)
    assert (np.diff(rowptr) == 0).any() and (np.diff(rowptr) > 2).any()     # empty rows and real maxima
    x = np.round(synth.features_f32(60, 6, 6) * 2) / 2                 # few distinct values: ties
    a, arg = L.max_pool_aggregate(rowptr, col, x.astype(np.float64))
    y, _, am = oracle.naive_forward(rowptr, col, x.astype(np.float32), "max")
    assert np.array_equal(a, y) and np.array_equal(arg, am)


def test_gcn_aggregate_is_the_normalised_adjacency_product():
    rowptr, col = synth.random_graph(80, 0.08, seed=7, directed=True)
    n = 80
    z = np.random.default_rng(8).standard_normal((n, 5))
    a = sp.csr_matrix((np.ones(col.size), col, rowptr), shape=(n, n)) + sp.identity(n)
    dinv = 1.0 / (np.diff(rowptr) + 1.0)
    want = (a @ z) * dinv[:, None]
    np.testing.assert_allclose(L.gcn_aggregate(rowptr, col, z), want, rtol=0, atol=1e-13)
    g = np.random.default_rng(9).standard_normal((n, 5))
    np.testing.assert_allclose(L.gcn_aggregate_transposed(rowptr, col, g), a.T @ (g * dinv[:, None]), rtol=0, atol=1e-13)
    # and the C oracle's gcn op on the same (fp32) input
    z32 = z.astype(np.float32)
    y, _, _ = oracle.naive_forward(rowptr, col, z32, "gcn")
    np.testing.assert_allclose(L.gcn_aggregate(rowptr, col, z32.astype(np.float64)), y, rtol=0, atol=1e-13)


def finite_difference(f, w, eps=1e-6):
    g = np.zeros_like(w)
    for idx in np.ndindex(*w.shape):
        w[idx] += eps
        hi = f()
        w[idx] -= 2 * eps
        lo = f()
        w[idx] += eps
        g[idx] = (hi - lo) / (2 * eps)
    return g


def test_layer_gradients_match_finite_differences():
    rowptr, col = synth.random_graph(25, 0.2, seed=11)
    rng = np.random.default_rng(12)
    x = rng.standard_normal((25, 4))
    labels = rng.integers(0, 3, 25)
    w1, w2 = rng.standard_normal((4, 5)), rng.standard_normal((5, 3))
    r = L.gcn2(rowptr, col, x, w1, w2, labels)
    np.testing.assert_allclose(r["g_w1"], finite_difference(lambda: L.gcn2(rowptr, col, x, w1, w2, labels)["loss"], w1), atol=1e-7)
    np.testing.assert_allclose(r["g_w2"], finite_difference(lambda: L.gcn2(rowptr, col, x, w1, w2, labels)["loss"], w2), atol=1e-7)
    pool = [rng.standard_normal((4, 3)), rng.standard_normal((5, 3))]
    comb = [rng.standard_normal((7, 5)), rng.standard_normal((8, 3))]
    r = L.sage_pool2(rowptr, col, x, pool, comb, labels)
    for i in range(2):
        np.testing.assert_allclose(r["g_pool"][i],
                                   finite_difference(lambda: L.sage_pool2(rowptr, col, x, pool, comb, labels)["loss"], pool[i]), atol=1e-7)
        np.testing.assert_allclose(r["g_comb"][i],
                                   finite_difference(lambda: L.sage_pool2(rowptr, col, x, pool, comb, labels)["loss"], comb[i]), atol=1e-7)


def test_sage_lstm_layer_against_library_modules():
    # the layer composed from a library LSTM (run list by list), concatenation and a library linear map, in fp64
    torch = __import__("pytest").importorskip("torch")
    rng = np.random.default_rng(17)
    n, d, hidden, out = 9, 4, 3, 5
    rowptr = np.array([0, 3, 3, 5, 9, 10, 12, 12, 14, 15], dtype=np.int64)
    col = np.array([2, 0, 1, 4, 4, 6, 5, 0, 2, 3, 1, 1, 8, 7, 0], dtype=np.int32)
    h = rng.normal(size=(n, d))
    w_ih, w_hh, b = rng.normal(0, 0.5, (4 * hidden, d)), rng.normal(0, 0.5, (4 * hidden, hidden)), rng.normal(0, 0.5, 4 * hidden)
    w2 = rng.normal(0, 0.5, (hidden + d, out))
    got = L.sage_lstm_layer(rowptr, col, h, w_ih, w_hh, b, w2, relu_out=True)
    net = torch.nn.LSTM(d, hidden, batch_first=True).double()
    lin = torch.nn.Linear(hidden + d, out, bias=False).double()
    with torch.no_grad():
        net.weight_ih_l0.copy_(torch.from_numpy(w_ih)); net.weight_hh_l0.copy_(torch.from_numpy(w_hh))
        net.bias_ih_l0.copy_(torch.from_numpy(b)); net.bias_hh_l0.zero_()
        lin.weight.copy_(torch.from_numpy(w2.T))
        ht = torch.from_numpy(h)
        a = torch.zeros((n, hidden), dtype=torch.float64)
        for v in range(n):
            ids = col[rowptr[v]:rowptr[v + 1]].astype(np.int64)
            if ids.size:
                a[v] = net(ht[torch.from_numpy(ids)][None])[1][0][0, 0]
        want = torch.relu(lin(torch.cat([a, ht], dim=1))).numpy()
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)
    assert (got[[1, 6]] == np.maximum(np.concatenate([np.zeros((2, hidden)), h[[1, 6]]], axis=1) @ w2, 0)).all()   # empty lists: a_v = 0


def test_sage_lstm2_gradients_against_library_autograd():
    # the 2-layer model built from library modules (LSTM run list by list, Linear, ReLU, cross entropy), differentiated
    # by the library, in fp64
    torch = __import__("pytest").importorskip("torch")
    rng = np.random.default_rng(23)
    n, d, hidden, classes = 8, 3, 4, 3
    rowptr = np.array([0, 3, 3, 5, 9, 10, 12, 12, 14], dtype=np.int64)
    col = np.array([2, 0, 1, 4, 4, 6, 5, 0, 2, 3, 1, 1, 7, 0], dtype=np.int32)
    dims = [d, 5, classes]
    cells = [(rng.normal(0, 0.5, (4 * hidden, dims[i])), rng.normal(0, 0.5, (4 * hidden, hidden)), rng.normal(0, 0.5, 4 * hidden)) for i in range(2)]
    comb = [rng.normal(0, 0.5, (hidden + dims[i], dims[i + 1])) for i in range(2)]
    x = rng.normal(size=(n, d))
    labels = rng.integers(0, classes, n)
    got = L.sage_lstm2(rowptr, col, x, cells, comb, labels)
    t = lambda a: torch.from_numpy(np.asarray(a)).clone().requires_grad_()
    xt, ct, wt = t(x), [tuple(t(a) for a in c) for c in cells], [t(w) for w in comb]
    h = xt
    for i in range(2):
        rows = []
        for v in range(n):
            ids = col[rowptr[v]:rowptr[v + 1]].astype(np.int64)
            if ids.size == 0:
                rows.append(torch.zeros(hidden, dtype=torch.float64))
                continue
            hv, cv = torch.zeros(hidden, dtype=torch.float64), torch.zeros(hidden, dtype=torch.float64)
            for u in ids:
                hv, cv = torch._VF.lstm_cell(h[u][None], (hv[None], cv[None]), ct[i][0], ct[i][1], ct[i][2], None)
                hv, cv = hv[0], cv[0]
            rows.append(hv)
        h = torch.cat([torch.stack(rows), h], dim=1) @ wt[i]
        if i == 0:
            h = torch.relu(h)
    loss = torch.nn.functional.cross_entropy(h, torch.from_numpy(labels))
    loss.backward()
    assert abs(loss.item() - got["loss"]) <= 1e-12
    np.testing.assert_allclose(got["g_x"], xt.grad.numpy(), rtol=1e-9, atol=1e-12)
    for i in range(2):
        np.testing.assert_allclose(got["g_comb"][i], wt[i].grad.numpy(), rtol=1e-9, atol=1e-12)
        for k in range(3):
            np.testing.assert_allclose(got["g_cells"][i][k], ct[i][k].grad.numpy(), rtol=1e-9, atol=1e-12)
