"""Layer-level GPU parity: the paper's two layers (Table 1) around hag_forward / hag_backward against the
layer oracle (oracle/layers.py, fp64, plain definitions).

Two bars.  (1) Every aggregation call the layer makes is compared with the C oracle ON THE INPUT THE
CALL RECEIVED, at the aggregation bars: |gpu - oracle| <= 1e-5 * sum|terms| for the fused GCN
aggregation, bit-exact values and argmax for max.  (2) Loss and weight gradients of the whole 2-layer
model against the fp64 layer oracle, as a norm-wise relative error: the dense parts run as fp32
library GEMMs, and a ReLU whose input rounds to the other side of zero changes single entries, so an
element-wise bar is not meaningful end to end."""
import numpy as np
import pytest

import oracle
from oracle import layers as OL
from paper_1906_03707_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 1e-5


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1906_03707_amd import binding
    binding.lib()
    return binding


def rel(a, ref):
    return float(np.linalg.norm(np.asarray(a, dtype=np.float64) - ref) / max(np.linalg.norm(ref), 1e-300))


def graphs(B):
    rowptr, col = synth.holme_kim(5000, 10, 0.5, seed=91)
    yield "power-law", rowptr, col, B.hag_search(rowptr, col, 1250).upload()
    rowptr, col, gp = synth.er_batch(n_graphs=80, size=30, p=0.6, seed=92)     # runs the component-local pass
    yield "graph batch", rowptr, col, B.hag_search_batched(rowptr, col, gp, 0.25).upload()


def check_recorded_calls(rowptr, col, record, op):
    for rec in record:
        kind, zin, zout = rec[0], rec[1].cpu().numpy(), rec[2].cpu().numpy()
        if op == "max":
            am = rec[3].cpu().numpy()
            if kind == "forward":
                y, _, am_ref = oracle.naive_forward(rowptr, col, zin, "max")
                assert np.array_equal(zout.astype(np.float64), y) and np.array_equal(am, am_ref)
            else:
                gx, gs = oracle.naive_backward(rowptr, col, zin, "max", am)
                assert np.all(np.abs(zout - gx) <= TOL * gs)
        else:
            ref, s = (oracle.naive_forward(rowptr, col, zin, op)[:2] if kind == "forward"
                      else oracle.naive_backward(rowptr, col, zin, op))
            assert np.all(np.abs(zout - ref) <= TOL * s), (kind, float(np.max(np.abs(zout - ref) / np.maximum(s, 1e-300))))


@pytest.mark.parametrize("naive", [False, True])
def test_two_layer_gcn_forward_and_backward(B, naive):
    from paper_1906_03707_amd import layers
    for name, rowptr, col, h in graphs(B):
        n, d, hidden, classes = rowptr.size - 1, 64, 16, 8
        rng = np.random.default_rng(93)
        x = synth.features_f32(n, d, 94)
        w1 = (rng.standard_normal((d, hidden)) / d ** 0.5).astype(np.float32)
        w2 = (rng.standard_normal((hidden, classes)) / hidden ** 0.5).astype(np.float32)
        labels = rng.integers(0, classes, n)
        xd = torch.from_numpy(x).cuda()
        w1d, w2d = torch.from_numpy(w1).cuda().requires_grad_(), torch.from_numpy(w2).cuda().requires_grad_()
        record = []
        loss = layers.gcn2_loss(h, xd, w1d, w2d, torch.from_numpy(labels).cuda(), naive=naive, record=record)
        loss.backward()
        torch.cuda.synchronize()
        assert len(record) == 4                                       # two aggregations forward, two backward
        check_recorded_calls(rowptr, col, record, "gcn")
        ref = OL.gcn2(rowptr, col, x, w1, w2, labels)
        assert abs(loss.item() - ref["loss"]) <= 1e-5 * abs(ref["loss"]), (name, loss.item(), ref["loss"])
        assert rel(w1d.grad.cpu().numpy(), ref["g_w1"]) <= 1e-4 and rel(w2d.grad.cpu().numpy(), ref["g_w2"]) <= 1e-4, name


@pytest.mark.parametrize("naive", [False, True])
def test_two_layer_graphsage_pool_forward_and_backward(B, naive):
    from paper_1906_03707_amd import layers
    for name, rowptr, col, h in graphs(B):
        n, d, hidden, classes = rowptr.size - 1, 32, 16, 5
        rng = np.random.default_rng(95)
        x = synth.features_f32(n, d, 96)
        dims = [d, hidden, classes]
        pool = [(rng.standard_normal((dims[i], hidden)) / dims[i] ** 0.5).astype(np.float32) for i in range(2)]
        comb = [(rng.standard_normal((hidden + dims[i], dims[i + 1])) / (hidden + dims[i]) ** 0.5).astype(np.float32) for i in range(2)]
        labels = rng.integers(0, classes, n)
        xd = torch.from_numpy(x).cuda()
        pd = [torch.from_numpy(w).cuda().requires_grad_() for w in pool]
        cd = [torch.from_numpy(w).cuda().requires_grad_() for w in comb]
        record = []
        loss = layers.sage_pool2_loss(h, xd, pd, cd, torch.from_numpy(labels).cuda(), naive=naive, record=record)
        loss.backward()
        torch.cuda.synchronize()
        assert len(record) == 4
        check_recorded_calls(rowptr, col, record, "max")
        ref = OL.sage_pool2(rowptr, col, x, pool, comb, labels)
        assert abs(loss.item() - ref["loss"]) <= 1e-5 * abs(ref["loss"]), (name, loss.item(), ref["loss"])
        for i in range(2):
            assert rel(pd[i].grad.cpu().numpy(), ref["g_pool"][i]) <= 1e-4, (name, i)
            assert rel(cd[i].grad.cpu().numpy(), ref["g_comb"][i]) <= 1e-4, (name, i)


@pytest.mark.parametrize("capacity", ["lists", "quarter", "unlimited"])
def test_two_layer_graphsage_lstm_inference(B, capacity):
    # 2-layer GraphSAGE with LSTM aggregators over ordered lists (first 12 neighbours of a power-law graph), inference:
    # the aggregation of each layer is the library's LSTM aggregator over the plain lists or a prefix HAG, the dense
    # Update is torch.  Against the fp64 layer oracle, norm-wise (fp32 GEMMs and ReLU around the aggregator).
    from paper_1906_03707_amd import layers, workloads
    rowptr, col = synth.holme_kim(1500, 8, 0.5, seed=93)
    rp, cl = workloads.first_neighbour_lists(rowptr, col, 12)
    n, d, hidden, classes = rp.size - 1, 24, 32, 8
    rng = np.random.default_rng(94)
    dims = [d, hidden, classes]
    cells = [(rng.normal(0, 0.3, (4 * hidden, dims[i])), rng.normal(0, 0.3, (4 * hidden, hidden)), rng.normal(0, 0.3, 4 * hidden))
             for i in range(2)]
    comb = [rng.normal(0, 1.0 / np.sqrt(hidden + dims[i]), (hidden + dims[i], dims[i + 1])) for i in range(2)]
    x = rng.normal(size=(n, d))
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    r64 = lambda a: dev(a).cpu().numpy().astype(np.float64)          # the oracle sees the fp32-rounded values
    want = OL.sage_lstm2_logits(rp, cl, r64(x), [tuple(r64(a) for a in c) for c in cells], [r64(w) for w in comb])
    cap = {"lists": 0, "quarter": n // 4, "unlimited": int(cl.size)}[capacity]
    seq = B.SeqHag(rp, cl, cap).upload()
    got = layers.sage_lstm2_logits(seq, dev(x), [tuple(dev(a) for a in c) for c in cells], [dev(w) for w in comb])
    seq.check()
    err = rel(got.cpu().numpy(), want)
    print(f"{capacity}: {seq.cells} cells, relative error of the logits {err:.2e}")
    assert err <= 1e-5


@pytest.mark.parametrize("capacity", ["lists", "unlimited"])
def test_two_layer_graphsage_lstm_training(B, capacity):
    # the same model trained: loss and every gradient (both LSTM cells, both dense maps) against the fp64 layer oracle,
    # norm-wise; the aggregator's forward and backward passes are the library's over the plain lists or a prefix HAG
    from paper_1906_03707_amd import layers, workloads
    rowptr, col = synth.holme_kim(600, 6, 0.5, seed=97)
    rp, cl = workloads.first_neighbour_lists(rowptr, col, 10)
    n, d, hidden, classes = rp.size - 1, 16, 24, 6
    rng = np.random.default_rng(98)
    dims = [d, hidden, classes]
    cells = [(rng.normal(0, 0.3, (4 * hidden, dims[i])), rng.normal(0, 0.3, (4 * hidden, hidden)), rng.normal(0, 0.3, 4 * hidden))
             for i in range(2)]
    comb = [rng.normal(0, 1.0 / np.sqrt(hidden + dims[i]), (hidden + dims[i], dims[i + 1])) for i in range(2)]
    x = rng.normal(size=(n, d))
    labels = rng.integers(0, classes, n)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    r64 = lambda a: dev(a).cpu().numpy().astype(np.float64)
    ref = OL.sage_lstm2(rp, cl, r64(x), [tuple(r64(a) for a in c) for c in cells], [r64(w) for w in comb], labels)
    seq = B.SeqHag(rp, cl, {"lists": 0, "unlimited": int(cl.size)}[capacity]).upload()
    xd = dev(x).requires_grad_()
    cd = [tuple(dev(a).requires_grad_() for a in c) for c in cells]
    wd = [dev(w).requires_grad_() for w in comb]
    loss = layers.sage_lstm2_loss(seq, xd, cd, wd, torch.from_numpy(labels).cuda())
    loss.backward()
    seq.check()
    assert abs(loss.item() - ref["loss"]) <= 1e-5 * abs(ref["loss"])
    assert rel(xd.grad.cpu().numpy(), ref["g_x"]) <= 1e-4
    for i in range(2):
        assert rel(wd[i].grad.cpu().numpy(), ref["g_comb"][i]) <= 1e-4, i
        for k in range(3):
            assert rel(cd[i][k].grad.cpu().numpy(), ref["g_cells"][i][k]) <= 1e-4, (i, k)
