"""The two GNN layers of the paper's Table 1 around the library's aggregation calls.

Only the aggregation (and, for GCN, the normalisation fused into it) is this library's work; the
dense parts (weight matrices, ReLU, SoftMax loss) are plain torch and serve the end-to-end
measurements and the layer-level parity tests.  Each aggregation call can be recorded (its input and
output tensors), so that a test can hand exactly those inputs to the CPU oracle.

GCN (Table 1, GCN row; the model of Section 5.3):  h'_v = relu(W . (a_v + h_v) / (|N(v)| + 1)) with
a_v the sum over N(v).  W is linear, so the layer transforms first and aggregates at the narrow width:
h' = relu(gcn_agg(h W)), gcn_agg being op "gcn" of hag_forward.
GraphSAGE-P (Table 1, pooling row):  a_v = max over N(v) of relu(W1 h_u),  h'_v = relu(W2 [a_v, h_v]).
"""
from __future__ import annotations

import torch


def aggregation(h, op, naive=False, record=None):
    """torch.autograd.Function around hag_forward / hag_backward (or the naive-CSR kernels) for `op`.

    record: optional list; every call appends (kind, input tensor, output tensor[, argmax])."""
    fwd = h.naive_forward if naive else h.forward
    bwd = h.naive_backward if naive else h.backward

    class Agg(torch.autograd.Function):
        @staticmethod
        def forward(ctx, z):
            z = z.contiguous()
            if op == "max":
                y, am = fwd(z, "max")
                ctx.am = am
                if record is not None:
                    record.append(("forward", z.detach().clone(), y.detach().clone(), am.clone()))
                return y
            y = fwd(z, op)
            if record is not None:
                record.append(("forward", z.detach().clone(), y.detach().clone()))
            return y

        @staticmethod
        def backward(ctx, g):
            g = g.contiguous()
            gx = bwd(g, "max", argmax=ctx.am) if op == "max" else bwd(g, op)
            if record is not None:
                record.append(("backward", g.detach().clone(), gx.detach().clone()) + ((ctx.am.clone(),) if op == "max" else ()))
            return gx

    return Agg.apply


def gcn2_loss(h, x, w1, w2, labels, naive=False, record=None):
    """SoftMax cross-entropy of a 2-layer GCN (Section 5.3's model) on features x."""
    agg = aggregation(h, "gcn", naive, record)
    h1 = torch.relu(agg(x @ w1))
    logits = agg(h1 @ w2)
    return torch.nn.functional.cross_entropy(logits, labels)


def sage_pool2_loss(h, x, pool, comb, labels, naive=False, record=None):
    """SoftMax cross-entropy of a 2-layer GraphSAGE with the pooling aggregator of Table 1.

    pool[i]: [d_i, hidden] (W1 of layer i), comb[i]: [hidden + d_i, d_{i+1}] (W2 of layer i)."""
    agg = aggregation(h, "max", naive, record)
    hcur = x
    for i in range(2):
        a = agg(torch.relu(hcur @ pool[i]))
        hcur = torch.cat([a, hcur], dim=1) @ comb[i]
        if i == 0:
            hcur = torch.relu(hcur)
    return torch.nn.functional.cross_entropy(hcur, labels)


def sage_lstm2_logits(seq, x, cells, comb):
    """Logits of a 2-layer GraphSAGE with LSTM aggregators over ordered neighbour lists (inference; training would wrap
    SeqHag.lstm_forward_train / lstm_backward the way `aggregation` wraps the set aggregates).  seq: binding.SeqHag (a prefix HAG or the plain lists);
    cells[i] = (w_ih, w_hh, b) of layer i; comb[i] = W2 of layer i, [hidden_i + d_i, d_{i+1}].
    a_v = LSTM over (h_u : u in N(v)), h'_v = relu(W2 [a_v, h_v]); the second layer has no ReLU."""
    with torch.no_grad():
        h = x
        for i in range(2):
            a = seq.lstm_forward(h.contiguous(), *cells[i])
            h = torch.cat([a, h], dim=1) @ comb[i]
            if i == 0:
                h = torch.relu(h)
        return h


def lstm_aggregation(seq):
    """torch.autograd.Function around SeqHag.lstm_forward_train / lstm_backward: a = f(x, w_ih, w_hh, b)."""
    class Agg(torch.autograd.Function):
        @staticmethod
        def forward(ctx, x, w_ih, w_hh, b):
            x, w_ih, w_hh = x.contiguous(), w_ih.contiguous(), w_hh.contiguous()
            a, ws = seq.lstm_forward_train(x, w_ih, w_hh, b.contiguous())
            ctx.save_for_backward(x, w_ih, w_hh)
            ctx.ws = ws
            return a

        @staticmethod
        def backward(ctx, g):
            x, w_ih, w_hh = ctx.saved_tensors
            out = seq.lstm_backward(x, w_ih, w_hh, g.contiguous(), ctx.ws)
            ctx.ws = None
            return out

    return Agg.apply


def sage_lstm2_loss(seq, x, cells, comb, labels):
    """SoftMax cross-entropy of the 2-layer GraphSAGE with LSTM aggregators of sage_lstm2_logits, differentiable:
    the aggregator's forward and backward passes are the library's, the dense parts torch."""
    agg = lstm_aggregation(seq)
    h = x
    for i in range(2):
        a = agg(h, *cells[i])
        h = torch.cat([a, h], dim=1) @ comb[i]
        if i == 0:
            h = torch.relu(h)
    return torch.nn.functional.cross_entropy(h, labels)
