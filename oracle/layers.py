"""Layer-level CPU oracle -- TEST INFRASTRUCTURE ONLY (numpy, fp64, plain definitions).

The two GNN layers of the paper's Table 1 written out from their definitions, forward and
backward, with the neighbourhood aggregation as an explicit loop over N(v).  Nothing here is
shared with the HIP library or with the C oracle; tests pin it against both and against a
hand-worked example.

  GCN row:      a_v = sum over N(v) of h_u;   h'_v = sigma(W . (a_v + h_v) / (|N(v)| + 1))
  pooling row:  a_v = max over N(v) of sigma(W1 h_u) (element-wise);   h'_v = sigma(W2 . [a_v, h_v])
sigma = ReLU.  Conventions where the paper is silent: an empty N(v) gives a_v = 0 (no gradient
through the max); a tie of the max goes to the smallest node id.
"""
from __future__ import annotations

import numpy as np


def gcn_aggregate(rowptr, col, z):
    """(sum over N(v) of z_u + z_v) / (|N(v)| + 1), fp64 (Table 1, GCN row, before the weights)."""
    n = rowptr.size - 1
    y = np.zeros((n, z.shape[1]), dtype=np.float64)
    for v in range(n):
        nb = col[rowptr[v]:rowptr[v + 1]]
        y[v] = (z[nb].sum(axis=0) + z[v]) / (nb.size + 1)
    return y


def gcn_aggregate_transposed(rowptr, col, g):
    """Vector-Jacobian product of gcn_aggregate: gz[u] = sum over v with u in N(v) or u = v of g[v] / (|N(v)| + 1)."""
    n = rowptr.size - 1
    gz = np.zeros((n, g.shape[1]), dtype=np.float64)
    for v in range(n):
        nb = col[rowptr[v]:rowptr[v + 1]]
        t = g[v] / (nb.size + 1)
        np.add.at(gz, nb, t)
        gz[v] += t
    return gz


def softmax_xent(logits, labels):
    """Mean SoftMax cross-entropy and its gradient w.r.t. the logits."""
    m = logits - logits.max(axis=1, keepdims=True)
    p = np.exp(m)
    p /= p.sum(axis=1, keepdims=True)
    n = logits.shape[0]
    loss = -np.log(p[np.arange(n), labels]).mean()
    g = p.copy()
    g[np.arange(n), labels] -= 1.0
    return loss, g / n


def gcn2(rowptr, col, x, w1, w2, labels):
    """Loss and weight gradients of the 2-layer GCN of Section 5.3: h1 = relu(agg(x W1)), logits = agg(h1 W2)."""
    x, w1, w2 = (np.asarray(a, dtype=np.float64) for a in (x, w1, w2))
    a1 = gcn_aggregate(rowptr, col, x @ w1)
    h1 = np.maximum(a1, 0.0)
    logits = gcn_aggregate(rowptr, col, h1 @ w2)
    loss, g_logits = softmax_xent(logits, labels)
    g_z2 = gcn_aggregate_transposed(rowptr, col, g_logits)
    g_w2 = h1.T @ g_z2
    g_a1 = (g_z2 @ w2.T) * (a1 > 0)
    g_z1 = gcn_aggregate_transposed(rowptr, col, g_a1)
    g_w1 = x.T @ g_z1
    return dict(loss=loss, logits=logits, h1=h1, g_w1=g_w1, g_w2=g_w2, g_x=g_z1 @ w1.T)


def max_pool_aggregate(rowptr, col, p):
    """a_v = element-wise max over N(v) of p_u, with the winning node id (smallest id on ties; -1 and 0 if N(v) is empty)."""
    n, d = rowptr.size - 1, p.shape[1]
    a = np.zeros((n, d), dtype=np.float64)
    arg = np.full((n, d), -1, dtype=np.int64)
    for v in range(n):
        for u in col[rowptr[v]:rowptr[v + 1]]:
            for f in range(d):
                if arg[v, f] < 0 or p[u, f] > a[v, f] or (p[u, f] == a[v, f] and u < arg[v, f]):
                    a[v, f] = p[u, f]
                    arg[v, f] = u
    return a, arg


def sage_pool_layer(rowptr, col, h, w1, w2, relu_out=True):
    """One GraphSAGE layer with the pooling aggregator (Table 1); returns the output and what backward needs."""
    h, w1, w2 = (np.asarray(a, dtype=np.float64) for a in (h, w1, w2))
    pre_p = h @ w1
    p = np.maximum(pre_p, 0.0)
    a, arg = max_pool_aggregate(rowptr, col, p)
    cat = np.concatenate([a, h], axis=1)
    pre = cat @ w2
    out = np.maximum(pre, 0.0) if relu_out else pre
    return out, dict(h=h, w1=w1, w2=w2, pre_p=pre_p, arg=arg, cat=cat, pre=pre, relu_out=relu_out)


def sage_pool_layer_backward(ctx, g_out):
    """Gradients of sage_pool_layer w.r.t. its input and both weight matrices."""
    g_pre = g_out * (ctx["pre"] > 0) if ctx["relu_out"] else g_out
    g_w2 = ctx["cat"].T @ g_pre
    g_cat = g_pre @ ctx["w2"].T
    k = ctx["w1"].shape[1]
    g_a, g_h = g_cat[:, :k], g_cat[:, k:].copy()
    g_p = np.zeros_like(ctx["pre_p"])
    n = g_a.shape[0]
    for v in range(n):
        for f in range(k):
            u = ctx["arg"][v, f]
            if u >= 0:
                g_p[u, f] += g_a[v, f]
    g_pre_p = g_p * (ctx["pre_p"] > 0)
    g_w1 = ctx["h"].T @ g_pre_p
    g_h += g_pre_p @ ctx["w1"].T
    return g_h, g_w1, g_w2


def sage_pool2(rowptr, col, x, pool, comb, labels):
    """Loss and weight gradients of a 2-layer GraphSAGE-P (second layer without the final ReLU: its output are the logits)."""
    o1, c1 = sage_pool_layer(rowptr, col, x, pool[0], comb[0], relu_out=True)
    o2, c2 = sage_pool_layer(rowptr, col, o1, pool[1], comb[1], relu_out=False)
    loss, g = softmax_xent(o2, labels)
    g_o1, g_p1, g_c1 = sage_pool_layer_backward(c2, g)
    g_x, g_p0, g_c0 = sage_pool_layer_backward(c1, g_o1)
    return dict(loss=loss, logits=o2, g_pool=[g_p0, g_p1], g_comb=[g_c0, g_c1], g_x=g_x)


def sage_lstm_layer(rowptr, col, h, w_ih, w_hh, b, w2, relu_out=True):
    """One GraphSAGE layer with an LSTM aggregator over the ORDERED lists N(v) (the sequential Aggregate of
    Section 3.1; Update as in Table 1's pooling row): a_v = the last hidden state of the LSTM run over
    (h_u : u in N(v)) from the zero state, h'_v = relu(W2 [a_v, h_v])."""
    from . import lstm
    h, w2 = np.asarray(h, dtype=np.float64), np.asarray(w2, dtype=np.float64)
    a, _ = lstm.naive_aggregate(rowptr, col, h, np.asarray(w_ih, dtype=np.float64), np.asarray(w_hh, dtype=np.float64),
                                np.asarray(b, dtype=np.float64))
    pre = np.concatenate([a, h], axis=1) @ w2
    return np.maximum(pre, 0.0) if relu_out else pre


def sage_lstm2_logits(rowptr, col, x, cells, comb):
    """Logits of a 2-layer GraphSAGE with LSTM aggregators (inference): cells[i] = (w_ih, w_hh, b) of layer i,
    comb[i] = W2 of layer i [hidden_i + d_i, d_{i+1}]; the second layer has no ReLU."""
    h1 = sage_lstm_layer(rowptr, col, x, *cells[0], comb[0], relu_out=True)
    return sage_lstm_layer(rowptr, col, h1, *cells[1], comb[1], relu_out=False)


def sage_lstm2(rowptr, col, x, cells, comb, labels):
    """Loss and gradients of the 2-layer GraphSAGE with LSTM aggregators above under a SoftMax cross-entropy loss (the
    chain rule through sage_lstm_layer, the aggregator's part being lstm.naive_aggregate_backward).
    Returns loss, logits, g_cells [(g_w_ih, g_w_hh, g_b)] and g_comb per layer, and g_x."""
    from . import lstm
    x = np.asarray(x, dtype=np.float64)
    cells = [tuple(np.asarray(a, dtype=np.float64) for a in c) for c in cells]
    comb = [np.asarray(w, dtype=np.float64) for w in comb]
    hs, cats, pres = [x], [], []
    for i in range(2):
        a, _ = lstm.naive_aggregate(rowptr, col, hs[i], *cells[i])
        cats.append(np.concatenate([a, hs[i]], axis=1))
        pres.append(cats[i] @ comb[i])
        hs.append(np.maximum(pres[i], 0.0) if i == 0 else pres[i])
    loss, g = softmax_xent(hs[2], labels)
    g_cells, g_comb = [None, None], [None, None]
    for i in (1, 0):
        g_pre = g * (pres[i] > 0) if i == 0 else g
        g_comb[i] = cats[i].T @ g_pre
        g_cat = g_pre @ comb[i].T
        hidden = cells[i][1].shape[1]
        g_x, g_wi, g_wh, g_b = lstm.naive_aggregate_backward(rowptr, col, hs[i], *cells[i], g_cat[:, :hidden])
        g_cells[i] = (g_wi, g_wh, g_b)
        g = g_cat[:, hidden:] + g_x
    return dict(loss=loss, logits=hs[2], g_cells=g_cells, g_comb=g_comb, g_x=g)
