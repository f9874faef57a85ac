"""Pins of the LSTM-aggregator oracle (oracle/lstm.py) against things other than itself: a closed
form with saturated gates, a library LSTM on single sequences, order dependence, and the
equivalence of naive and prefix-HAG execution (Theorem 2 with ordered covers, Section 3.1)."""
import numpy as np
import pytest

from oracle import lstm, sequential
from paper_1906_03707_amd import synth


def params(d, hidden, seed, scale=0.4):
    rng = np.random.default_rng(seed)
    return (rng.normal(0, scale, (4 * hidden, d)), rng.normal(0, scale, (4 * hidden, hidden)), rng.normal(0, scale, 4 * hidden))


def ordered_graph(n, deg, seed):
    """Ordered lists with many common prefixes: every list is a prefix of one of a few 'routes' plus a tail."""
    rng = np.random.default_rng(seed)
    routes = [rng.permutation(n)[:deg] for _ in range(4)]
    rowptr, col = [0], []
    for v in range(n):
        k = int(rng.integers(0, deg + 1))
        l = list(routes[int(rng.integers(0, 4))][:k]) + list(rng.integers(0, n, int(rng.integers(0, 3))))
        col += l
        rowptr.append(len(col))
    return np.asarray(rowptr, dtype=np.int64), np.asarray(col, dtype=np.int32)


def test_closed_form_with_saturated_gates():
    # input, forget and output gates held at exactly 1 by a large bias (sigmoid(60) rounds to 1.0 in
    # fp64), cell gate g = tanh(w x): then c_k = sum_t tanh(w x_t) and a = tanh(c_k)
    d, hidden = 1, 1
    w_ih = np.array([[0.0], [0.0], [0.7], [0.0]])
    w_hh = np.zeros((4, 1))
    b = np.array([60.0, 60.0, 0.0, 60.0])
    x = np.array([[0.3], [-1.2], [2.0], [0.5]])
    rowptr = np.array([0, 3, 3, 4, 6], dtype=np.int64)
    col = np.array([2, 0, 1, 3, 1, 1], dtype=np.int32)
    a, cells = lstm.naive_aggregate(rowptr, col, x, w_ih, w_hh, b)
    assert cells == 6
    want = [np.tanh(np.tanh(0.7 * 2.0) + np.tanh(0.7 * 0.3) + np.tanh(0.7 * -1.2)), 0.0, np.tanh(np.tanh(0.7 * 0.5)),
            np.tanh(2 * np.tanh(0.7 * -1.2))]
    np.testing.assert_allclose(a[:, 0], want, rtol=0, atol=1e-15)


def test_gate_order_and_recurrence_against_a_library_lstm():
    torch = pytest.importorskip("torch")
    d, hidden = 5, 3
    w_ih, w_hh, b = params(d, hidden, 7)
    rng = np.random.default_rng(8)
    x = rng.normal(size=(9, d))
    rowptr = np.array([0, 4, 4, 9, 10], dtype=np.int64)
    col = np.array([3, 1, 4, 1, 8, 7, 6, 5, 0, 2], dtype=np.int32)
    a, _ = lstm.naive_aggregate(rowptr, col, x, w_ih, w_hh, b)
    net = torch.nn.LSTM(d, hidden, batch_first=True).double()
    with torch.no_grad():
        net.weight_ih_l0.copy_(torch.from_numpy(w_ih))
        net.weight_hh_l0.copy_(torch.from_numpy(w_hh))
        net.bias_ih_l0.copy_(torch.from_numpy(b))
        net.bias_hh_l0.zero_()
        for v in range(4):
            ids = col[rowptr[v]:rowptr[v + 1]]
            if ids.size == 0:
                assert not a[v].any()
                continue
            _, (h, _) = net(torch.from_numpy(x[ids])[None])
            np.testing.assert_allclose(a[v], h[0, 0].numpy(), rtol=1e-12, atol=1e-14)


def test_the_aggregate_depends_on_the_order():
    d, hidden = 4, 4
    w_ih, w_hh, b = params(d, hidden, 11)
    x = np.random.default_rng(12).normal(size=(3, d))
    rowptr = np.array([0, 3, 6], dtype=np.int64)
    a, _ = lstm.naive_aggregate(rowptr, np.array([0, 1, 2, 2, 1, 0], dtype=np.int32), x, w_ih, w_hh, b)
    assert np.abs(a[0] - a[1]).max() > 1e-3


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_prefix_hag_execution_equals_naive_and_saves_cells(seed):
    n, d, hidden = 60, 6, 5
    rowptr, col = ordered_graph(n, 7, seed)
    w_ih, w_hh, b = params(d, hidden, seed + 20)
    x = np.random.default_rng(seed + 40).normal(size=(n, d))
    naive, cells_naive = lstm.naive_aggregate(rowptr, col, x, w_ih, w_hh, b)
    assert cells_naive == col.size
    for capacity in (0, 5, col.size):
        merges, lists = sequential.search(rowptr, col, capacity)
        assert sequential.cover_check(rowptr, col, merges, lists) == 0
        got, cells = lstm.hag_aggregate(n, merges, lists, x, w_ih, w_hh, b)
        assert np.array_equal(got, naive)            # same arithmetic in the same order
        # one cell per distinct non-empty prefix that is evaluated: never more than the naive walk
        assert cells <= cells_naive
        if capacity == col.size:
            # all sharing found (Theorem 3): one cell per distinct prefix of length >= 1
            prefixes = {tuple(col[rowptr[v]:rowptr[v] + k]) for v in range(n) for k in range(1, rowptr[v + 1] - rowptr[v] + 1)}
            assert cells == len(prefixes)


def test_a_planted_mistake_in_the_hag_is_seen():
    # a HAG whose merge has its pair reversed computes something else (the oracle is sensitive to order)
    n, d, hidden = 20, 4, 4
    rowptr, col = ordered_graph(n, 5, 9)
    w_ih, w_hh, b = params(d, hidden, 3)
    x = np.random.default_rng(4).normal(size=(n, d))
    merges, lists = sequential.search(rowptr, col, col.size)
    assert merges
    naive, _ = lstm.naive_aggregate(rowptr, col, x, w_ih, w_hh, b)
    bad = [(m[1], m[0], m[2]) if i == 0 else m for i, m in enumerate(merges)]
    got, _ = lstm.hag_aggregate(n, bad, lists, x, w_ih, w_hh, b)
    assert np.abs(got - naive).max() > 1e-6


def test_backward_against_autograd_of_a_library_lstm_and_finite_differences():
    torch = pytest.importorskip("torch")
    d, hidden, n = 4, 3, 7
    w_ih, w_hh, b = params(d, hidden, 31)
    rng = np.random.default_rng(32)
    x = rng.normal(size=(n, d))
    g_a = rng.normal(size=(n, hidden))
    rowptr = np.array([0, 3, 3, 5, 9, 10, 12, 12], dtype=np.int64)
    col = np.array([2, 0, 1, 4, 4, 6, 5, 0, 2, 3, 1, 1], dtype=np.int32)       # repeated nodes, empty lists
    g_x, g_wi, g_wh, g_b = lstm.naive_aggregate_backward(rowptr, col, x, w_ih, w_hh, b, g_a)
    # the library's LSTM run list by list, differentiated by the library
    xt = torch.from_numpy(x).requires_grad_(True)
    net = torch.nn.LSTM(d, hidden, batch_first=True).double()
    with torch.no_grad():
        net.weight_ih_l0.copy_(torch.from_numpy(w_ih)); net.weight_hh_l0.copy_(torch.from_numpy(w_hh))
        net.bias_ih_l0.copy_(torch.from_numpy(b)); net.bias_hh_l0.zero_()
    loss = 0.0
    for v in range(n):
        ids = col[rowptr[v]:rowptr[v + 1]]
        if ids.size:
            _, (h, _) = net(xt[torch.from_numpy(ids.astype(np.int64))][None])
            loss = loss + (h[0, 0] * torch.from_numpy(g_a[v])).sum()
    loss.backward()
    np.testing.assert_allclose(g_x, xt.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(g_wi, net.weight_ih_l0.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(g_wh, net.weight_hh_l0.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(g_b, net.bias_ih_l0.grad.numpy(), rtol=1e-10, atol=1e-12)
    # and a finite difference of the oracle's own forward pass in one direction of every argument
    def loss_of(x_, wi_, wh_, b_):
        a, _ = lstm.naive_aggregate(rowptr, col, x_, wi_, wh_, b_)
        return float((a * g_a).sum())
    eps = 1e-6
    for arg, grad in ((0, g_x), (1, g_wi), (2, g_wh), (3, g_b)):
        args = [x, w_ih, w_hh, b]
        direction = rng.normal(size=args[arg].shape)
        plus, minus = list(args), list(args)
        plus[arg] = args[arg] + eps * direction
        minus[arg] = args[arg] - eps * direction
        fd = (loss_of(*plus) - loss_of(*minus)) / (2 * eps)
        assert abs(fd - float((grad * direction).sum())) <= 1e-6 * max(1.0, abs(fd))
