"""CPU oracle for an LSTM neighbourhood aggregator run naively and over a prefix HAG -- TEST
INFRASTRUCTURE ONLY (numpy, fp64, explicit loops; small inputs).

A sequential Aggregate (Section 3.1) folds the ORDERED list N(v) = (u_1, ..., u_k) one element at a
time; here the fold is an LSTM cell, the aggregator the paper names for the sequential case:
    (h_0, c_0) = 0,   (h_t, c_t) = cell(x[u_t], h_{t-1}, c_{t-1}),   a_v = h_k   (a_v = 0 for an empty list).
A HAG for such an aggregate shares common prefixes: aggregation node w = (v1, v2) holds the state
after the ordered cover of v1 (Equation 2) followed by v2, and Algorithm 2 evaluates the
aggregation nodes in creation order before every v continues from the state of its list's head.
Equal results follow from Theorem 2 (equal ordered covers); the functions below compute both ways
with the same arithmetic in the same order, so they agree bit for bit.

The cell is the standard one: gates = W_ih x + W_hh h + b, split into input, forget, cell and output
gate (in this order), c' = sigmoid(f) c + sigmoid(i) tanh(g), h' = sigmoid(o) tanh(c').
Nothing here is shared with the library.
"""
from __future__ import annotations

import numpy as np


def sigmoid(z):
    return 1.0 / (1.0 + np.exp(-z))


def cell(x, h, c, w_ih, w_hh, b):
    """One LSTM step in fp64.  x [D], h, c [H], w_ih [4H, D], w_hh [4H, H], b [4H]."""
    hidden = h.size
    gates = w_ih @ x + w_hh @ h + b
    i, f, g, o = (gates[k * hidden:(k + 1) * hidden] for k in range(4))
    c_new = sigmoid(f) * c + sigmoid(i) * np.tanh(g)
    return sigmoid(o) * np.tanh(c_new), c_new


def naive_aggregate(rowptr, col, x, w_ih, w_hh, b):
    """a_v for every v by walking its list from the zero state.  Returns (a [n, H], cell evaluations)."""
    n = rowptr.size - 1
    hidden = w_hh.shape[1]
    x = np.asarray(x, dtype=np.float64)
    out = np.zeros((n, hidden))
    cells = 0
    for v in range(n):
        h, c = np.zeros(hidden), np.zeros(hidden)
        for u in col[rowptr[v]:rowptr[v + 1]]:
            h, c = cell(x[u], h, c, w_ih, w_hh, b)
            cells += 1
        out[v] = h
    return out, cells


def hag_aggregate(n, merges, lists, x, w_ih, w_hh, b):
    """The same over a prefix HAG: merges [(v1, v2, ...)] in creation order (node n + i), lists[v] the
    remaining ordered list of v (only its first entry may be an aggregation node).
    Returns (a [n, H], cell evaluations).  The state after a single original node u (the first step of a
    list that starts with u) is computed once per u and shared, like any other prefix."""
    hidden = w_hh.shape[1]
    x = np.asarray(x, dtype=np.float64)
    zero = np.zeros(hidden)
    first = {}            # u -> state after the one-element prefix (u)
    cells = 0

    def first_state(u):
        nonlocal cells
        if u not in first:
            first[u] = cell(x[u], zero, zero, w_ih, w_hh, b)
            cells += 1
        return first[u]

    agg = []              # states of the aggregation nodes, creation order (Algorithm 2's loop over V_A)
    for m in merges:
        v1, v2 = int(m[0]), int(m[1])
        h, c = first_state(v1) if v1 < n else agg[v1 - n]
        agg.append(cell(x[v2], h, c, w_ih, w_hh, b))
        cells += 1
    out = np.zeros((n, hidden))
    for v in range(n):
        l = lists[v]
        if not len(l):
            continue
        head = int(l[0])
        h, c = first_state(head) if head < n else agg[head - n]
        for u in l[1:]:
            h, c = cell(x[int(u)], h, c, w_ih, w_hh, b)
            cells += 1
        out[v] = h
    return out, cells


def naive_aggregate_backward(rowptr, col, x, w_ih, w_hh, b, g_a):
    """Gradients of L = sum_v <g_a[v], a_v> with respect to x, w_ih, w_hh and b, by backpropagation
    through time over every list (the chain rule applied to the definition above, list by list).
    Returns (g_x [n, D], g_w_ih, g_w_hh, g_b)."""
    n = rowptr.size - 1
    hidden = w_hh.shape[1]
    x = np.asarray(x, dtype=np.float64)
    g_x = np.zeros_like(x)
    g_w_ih, g_w_hh, g_b = np.zeros_like(w_ih), np.zeros_like(w_hh), np.zeros_like(b)
    for v in range(n):
        ids = [int(u) for u in col[rowptr[v]:rowptr[v + 1]]]
        if not ids:
            continue
        # forward, keeping what the backward pass needs
        h, c = np.zeros(hidden), np.zeros(hidden)
        tape = []
        for u in ids:
            gates = w_ih @ x[u] + w_hh @ h + b
            i, f, g, o = (gates[k * hidden:(k + 1) * hidden] for k in range(4))
            i, f, g, o = sigmoid(i), sigmoid(f), np.tanh(g), sigmoid(o)
            c_new = f * c + i * g
            tape.append((u, h, c, i, f, g, o, c_new))
            h, c = o * np.tanh(c_new), c_new
        d_h, d_c = np.asarray(g_a[v], dtype=np.float64).copy(), np.zeros(hidden)
        for u, h_prev, c_prev, i, f, g, o, c_new in reversed(tape):
            t = np.tanh(c_new)
            d_o = d_h * t
            d_c = d_c + d_h * o * (1.0 - t * t)
            d_gates = np.concatenate([d_c * g * i * (1.0 - i), d_c * c_prev * f * (1.0 - f), d_c * i * (1.0 - g * g),
                                      d_o * o * (1.0 - o)])
            g_w_ih += np.outer(d_gates, x[u])
            g_w_hh += np.outer(d_gates, h_prev)
            g_b += d_gates
            g_x[u] += w_ih.T @ d_gates
            d_h = w_hh.T @ d_gates
            d_c = d_c * f
    return g_x, g_w_ih, g_w_hh, g_b
