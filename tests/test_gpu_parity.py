"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Bars: int32 and max (values and argmax) bit-exact; fp32 sum / mean within
|gpu - oracle| <= 1e-5 * sum|terms| per output element (the oracle accumulates in fp64).
"""
import numpy as np
import pytest

import oracle
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


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def assert_close(gpu, ref, s, what):
    gpu = gpu.cpu().numpy().astype(np.float64)
    err = np.abs(gpu - ref)
    bad = err > TOL * s
    assert not bad.any(), f"{what}: {bad.sum()} elements beyond 1e-5*sum|x|; worst ratio {np.max(err / np.maximum(s, 1e-300)):.3e}"


def assert_equal(gpu, ref, what):
    gpu = gpu.cpu().numpy()
    assert gpu.dtype == ref.dtype or gpu.dtype.kind == ref.dtype.kind, what
    assert np.array_equal(gpu, ref.astype(gpu.dtype)), f"{what}: {np.count_nonzero(gpu != ref.astype(gpu.dtype))} mismatches"


def run_all_ops(B, h, rowptr, col, d, seed, ops=("sum", "mean", "max", "gcn"), dtypes=("f32", "i32")):
    """Forward + backward of the HAG path and of the naive-CSR GPU baseline vs the oracle."""
    n = rowptr.size - 1
    h.upload()
    for dt in dtypes:
        if dt == "f32":
            x, gy = synth.features_f32(n, d, seed), synth.features_f32(n, d, seed + 1)
        else:
            x, gy = synth.features_i32(n, d, seed), synth.features_i32(n, d, seed + 1)
        xd, gyd = dev(x), dev(gy)
        for op in ops:
            if op in ("mean", "gcn") and dt == "i32":
                continue
            tag = f"n={n} d={d} {dt} {op}"
            y_ref, s, am_ref = oracle.naive_forward(rowptr, col, x, op)
            for name, fwd, bwd in (("hag", h.forward, h.backward), ("naive", h.naive_forward, h.naive_backward)):
                out = fwd(xd, op)
                torch.cuda.synchronize()
                if op == "max":
                    y, am = out
                    assert_equal(y, y_ref, f"{name} fwd values {tag}")
                    assert_equal(am, am_ref, f"{name} fwd argmax {tag}")
                    gx_ref, gs = oracle.naive_backward(rowptr, col, gy, op, am_ref)
                    gx = bwd(gyd, op, argmax=am)
                else:
                    if dt == "f32":
                        assert_close(out, y_ref, s, f"{name} fwd {tag}")
                    else:
                        assert_equal(out, y_ref, f"{name} fwd {tag}")
                    gx_ref, gs = oracle.naive_backward(rowptr, col, gy, op)
                    gx = bwd(gyd, op)
                torch.cuda.synchronize()
                if dt == "f32":
                    assert_close(gx, gx_ref, gs, f"{name} bwd {tag}")
                else:
                    assert_equal(gx, gx_ref, f"{name} bwd {tag}")


@pytest.mark.parametrize("n,p,d,directed", [
    (37, 0.3, 4, False), (200, 0.1, 8, True), (333, 0.15, 16, False), (500, 0.08, 32, True),
    (777, 0.05, 64, False), (1000, 0.04, 128, True), (301, 0.2, 100, False), (150, 0.3, 260, True),
    (260, 0.2, 512, False), (129, 0.25, 1028, False),
])
def test_random_graphs_all_ops(B, n, p, d, directed):
    rowptr, col = synth.random_graph(n, p, seed=n + d, directed=directed)
    h = B.hag_search(rowptr, col, n // 2)
    assert h.stats()["a"] > 0
    run_all_ops(B, h, rowptr, col, d, seed=7 * n + d)


def test_fused_and_unfused_stages(B, monkeypatch):
    # levels are fused into stages (one launch each) when that costs few extra row reads; both the
    # fused form and the one-launch-per-level form must match the oracle
    rowptr, col = synth.sbm(n_blocks=3, block=60, p_in=0.5, p_out=0.02, seed=31)
    n = rowptr.size - 1
    fused = B.hag_search(rowptr, col, n)
    assert fused.stats()["levels"] >= 3 and fused.stats()["stages"] < fused.stats()["levels"]
    run_all_ops(B, fused, rowptr, col, 32, seed=32)
    monkeypatch.setenv("HAG_STAGE_EXTRA_ROWS", "-1000000")
    unfused = B.hag_search(rowptr, col, n)
    assert unfused.stats()["stages"] == unfused.stats()["levels"]
    run_all_ops(B, unfused, rowptr, col, 32, seed=32)


@pytest.mark.parametrize("offset64", [False, True])
def test_source_partitioned_schedule(B, monkeypatch, offset64):
    # rows cut by source id into per-XCD segments with partial rows folded afterwards: forced on
    # for a small graph (by default only large graphs use it), incl. hubs that are also split;
    # once more with the 64-bit row addressing that matrices of 4 GiB and more take
    if offset64:
        monkeypatch.setenv("HAG_OFFSET64", "1")
    monkeypatch.setenv("HAG_PARTITION_MIN_ROWS", "0")
    monkeypatch.setenv("HAG_PART_MIN", "8")
    monkeypatch.setenv("HAG_PART_MEAN_MIN", "0")
    monkeypatch.setenv("HAG_PART_SHIFT", "3")           # workgroup b takes source class (b + 3) mod 8: same results
    monkeypatch.setenv("HAG_BLOCK_MAX", "40")
    rowptr, col = synth.holme_kim(1500, 9, 0.5, seed=41)
    n = rowptr.size - 1
    assert np.diff(rowptr).max() > 100
    h = B.hag_search(rowptr, col, n // 4)
    run_all_ops(B, h, rowptr, col, 64, seed=42)
    # the cut is really in effect: its partial rows make the workspace larger than without it
    monkeypatch.setenv("HAG_PARTITION", "0")
    h_plain = B.hag_search(rowptr, col, n // 4).upload()
    monkeypatch.delenv("HAG_PARTITION")
    assert h.workspace_bytes("sum", 0, 64) > h_plain.workspace_bytes("sum", 0, 64)
    run_all_ops(B, h, rowptr, col, 16, seed=43, ops=("sum", "max"), dtypes=("f32",))
    rowptr, col = synth.random_graph(300, 0.2, seed=44, directed=True)
    h = B.hag_search(rowptr, col, 150)
    run_all_ops(B, h, rowptr, col, 128, seed=45)


@pytest.mark.parametrize("parts", ["2", "4"])
def test_component_local_pass_with_feature_columns_cut_in_parts(B, parts, monkeypatch):
    # the component pass with each component handled by 2 or 4 workgroups, one per part of the feature
    # columns (chosen by occupancy in real runs, forced here), must agree with the oracle and, bit for
    # bit, with the uncut pass
    sizes = np.random.default_rng(64).integers(1, 41, size=150)
    rowptr, col, gp = ragged_batch(sizes, 0.6, seed=65)
    whole = B.hag_search_batched(rowptr, col, gp, 0.25).upload()
    monkeypatch.setenv("HAG_COMPONENT_PARTS", parts)
    cut = B.hag_search_batched(rowptr, col, gp, 0.25).upload()
    monkeypatch.delenv("HAG_COMPONENT_PARTS")
    assert cut.stats()["components"] >= 64
    for d in (32, 64, 128):
        run_all_ops(B, cut, rowptr, col, d, seed=66 + d, ops=("sum", "mean", "gcn"))
        x = dev(synth.features_f32(rowptr.size - 1, d, 67))
        for op in ("sum", "mean", "gcn"):
            assert torch.equal(cut.forward(x, op), whole.forward(x, op)), (d, op)
            assert torch.equal(cut.backward(x, op), whole.backward(x, op)), (d, op)
            assert torch.equal(cut.naive_forward(x, op), whole.naive_forward(x, op)), (d, op)


def ragged_batch(sizes, p, seed):
    """Disjoint G(size, p) graphs of the given sizes (size 1 = an isolated node), block-diagonal CSR."""
    rng = np.random.default_rng(seed)
    rows, cols, off = [], [], 0
    for sz in sizes:
        m = np.triu(rng.random((sz, sz)) < p, 1)
        m = m | m.T
        r, c = np.nonzero(m)
        rows.append(r + off)
        cols.append(c + off)
        off += sz
    rows, cols = np.concatenate(rows), np.concatenate(cols)
    rowptr = np.concatenate([[0], np.cumsum(np.bincount(rows, minlength=off))]).astype(np.int64)
    return rowptr, cols.astype(np.int32), np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)


@pytest.mark.parametrize("expand", ["0", "1"])
@pytest.mark.parametrize("d", [16, 64, 260])
def test_component_local_pass_on_graph_batches(B, d, expand, monkeypatch):
    # a batch of small graphs runs as one launch per pass out of LDS (one workgroup per graph):
    # ragged sizes incl. isolated nodes and graphs without aggregation nodes, all ops and dtypes;
    # aggregation rows stage by stage in two-input form ("0") or expanded to original rows ("1")
    monkeypatch.setenv("HAG_COMPONENT_EXPAND", expand)
    sizes = np.random.default_rng(61).integers(1, 41, size=150)
    rowptr, col, gp = ragged_batch(sizes, 0.6, seed=62)
    assert rowptr.size - 1 >= 1024
    h = B.hag_search_batched(rowptr, col, gp, 0.25)
    assert h.stats()["a"] > 100 and h.stats()["levels"] >= 2
    assert h.stats()["components"] >= 64            # the component-local pass is the one that runs
    run_all_ops(B, h, rowptr, col, d, seed=63 + d)
    # streaming stores of the output rows (a knob read when a handle is built) change nothing but
    # the cache policy
    xf = dev(synth.features_f32(rowptr.size - 1, d, 6))
    want_y, want_gx = h.forward(xf, "sum"), h.backward(xf, "mean")
    monkeypatch.setenv("HAG_STREAM_OUTPUT", "1")
    hs = B.hag_search_batched(rowptr, col, gp, 0.25).upload()
    assert torch.equal(hs.forward(xf, "sum"), want_y) and torch.equal(hs.backward(xf, "mean"), want_gx)
    monkeypatch.delenv("HAG_STREAM_OUTPUT")
    # the same handle through the generic kernels must agree bit for bit on int32
    monkeypatch.setenv("HAG_COMPONENT", "0")
    g = B.hag_search_batched(rowptr, col, gp, 0.25).upload()
    x = dev(synth.features_i32(rowptr.size - 1, d, 5))
    assert torch.equal(h.forward(x, "sum"), g.forward(x, "sum"))
    assert torch.equal(h.backward(x, "sum"), g.backward(x, "sum"))
    ya, aa = h.forward(x, "max")
    yb, ab = g.forward(x, "max")
    assert torch.equal(ya, yb) and torch.equal(aa, ab)


def test_capacity_zero_is_the_gnn_graph(B):
    # Section 3.1: the GNN-graph is the HAG with V_A empty -> identical kernels, identical bits
    rowptr, col = synth.random_graph(400, 0.1, seed=3)
    h = B.hag_search(rowptr, col, 0).upload()
    x = dev(synth.features_f32(400, 64, 4))
    assert torch.equal(h.forward(x, "sum"), h.naive_forward(x, "sum"))
    assert torch.equal(h.backward(x, "sum"), h.naive_backward(x, "sum"))


def test_split_rows_hubs_and_isolated_nodes(B):
    # a few hubs with thousands of neighbours (rows split across items and folded in a second
    # launch), many leaves, some isolated nodes; unsymmetric
    n, d = 6000, 64
    rng = np.random.default_rng(11)
    rows, cols = [], []
    for hub, deg in ((0, 5000), (1, 3100), (2, 1537), (3, 1536), (4, 2049)):
        nb = rng.choice(np.arange(10, n - 50), size=deg, replace=False)
        rows += [hub] * deg
        cols += nb.tolist()
        rows += nb[: deg // 2].tolist()          # half of them point back
        cols += [hub] * (deg // 2)
    extra_r = rng.integers(10, n - 50, 20000)
    extra_c = rng.integers(0, n - 50, 20000)
    keys = np.unique(np.concatenate([np.asarray(rows) * n + np.asarray(cols), extra_r * n + extra_c]))
    r, c = keys // n, keys % n
    keep = r != c
    r, c = r[keep], c[keep]
    rowptr = np.concatenate([[0], np.cumsum(np.bincount(r, minlength=n))]).astype(np.int64)
    col = c.astype(np.int32)
    assert np.diff(rowptr)[-50:].max() == 0 and np.diff(rowptr).max() == 5000
    h = B.hag_search(rowptr, col, n // 4)
    run_all_ops(B, h, rowptr, col, d, seed=12)
    run_all_ops(B, h, rowptr, col, 16, seed=13, ops=("sum", "max"), dtypes=("f32",))


def test_self_loops_and_dedup(B):
    # a node may be its own neighbour (source and destination roles are distinct); duplicates are
    # dropped on request
    n = 200
    rowptr, col = synth.random_graph(n, 0.08, seed=51, directed=True)
    rows = np.repeat(np.arange(n), np.diff(rowptr))
    rows = np.concatenate([rows, np.arange(0, n, 2), rows[:300]])          # self-loops on even nodes + duplicates
    cols = np.concatenate([col, np.arange(0, n, 2), col[:300]])
    order = np.argsort(rows, kind="stable")
    rows, cols = rows[order], cols[order].astype(np.int32)
    rp = np.concatenate([[0], np.cumsum(np.bincount(rows, minlength=n))]).astype(np.int64)
    with pytest.raises(B.HagError):
        B.hag_search(rp, cols, n // 2)
    h = B.hag_search(rp, cols, n // 2, flags=B.HAG_SEARCH_DEDUP)
    keys = np.unique(rows.astype(np.int64) * n + cols)
    r2, c2 = keys // n, (keys % n).astype(np.int32)
    rp2 = np.concatenate([[0], np.cumsum(np.bincount(r2, minlength=n))]).astype(np.int64)
    assert h.stats()["e"] == c2.size and np.any(r2 == c2)
    run_all_ops(B, h, rp2, c2, 32, seed=52)


@pytest.mark.parametrize("kind", ["power_law", "graph_batch"])
def test_forward_backward_inside_a_hip_graph(B, kind):
    # the device entry points allocate nothing, never synchronise and clear memory with kernels, so a
    # whole step can be captured once and replayed; every replay must reproduce the eager result
    # (graph_batch: sum / mean run as the one-launch component-local pass, max on the generic kernels)
    if kind == "power_law":
        rowptr, col = synth.holme_kim(3000, 8, 0.5, seed=71)
        n = rowptr.size - 1
        h = B.hag_search(rowptr, col, n // 4).upload()
    else:
        sizes = np.random.default_rng(74).integers(8, 41, size=120)
        rowptr, col, gp = ragged_batch(sizes, 0.6, seed=75)
        n = rowptr.size - 1
        h = B.hag_search_batched(rowptr, col, gp, 0.25).upload()
        assert h.stats()["components"] >= 64
    d = 64
    assert h.stats()["levels"] >= 2
    x = dev(synth.features_f32(n, d, 72))
    gy = dev(synth.features_f32(n, d, 73))
    y, gx = torch.empty_like(x), torch.empty_like(x)
    ym, am, gm = torch.empty_like(x), torch.empty((n, d), dtype=torch.int32, device="cuda"), torch.empty_like(x)
    ws = torch.empty(h.workspace_bytes("max", B.HAG_F32, d), dtype=torch.uint8, device="cuda")

    def step():
        h.forward(x, "sum", y=y, workspace=ws)
        h.backward(gy, "mean", gx=gx, workspace=ws)
        h.forward(x, "max", y=ym, argmax=am, workspace=ws)
        h.backward(gy, "max", argmax=am, gx=gm, workspace=ws)

    step()
    torch.cuda.synchronize()
    want = [t.clone() for t in (y, gx, ym, am)]
    want_gm = gm.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        for t in (y, gx, ym, gm):
            t.zero_()                            # eager work between replays
        am.fill_(-7)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip((y, gx, ym, am), want):
            assert torch.equal(got, ref), f"replay {rep} differs from the eager run"
        assert torch.allclose(gm, want_gm, rtol=1e-5, atol=1e-5)   # atomics: order not fixed


def test_max_ties_bit_exact(B):
    # few distinct values -> many exact ties; argmax must be the smallest original id
    n, d = 600, 32
    rowptr, col = synth.random_graph(n, 0.1, seed=21)
    h = B.hag_search(rowptr, col, n // 2).upload()
    x = np.random.default_rng(22).integers(0, 3, size=(n, d)).astype(np.float32)
    y_ref, _, am_ref = oracle.naive_forward(rowptr, col, x, "max")
    for fwd in (h.forward, h.naive_forward):
        y, am = fwd(dev(x), "max")
        assert_equal(y, y_ref, "tied max values")
        assert_equal(am, am_ref, "tied max argmax")


@pytest.mark.parametrize("knobs", [
    {},
    {"HAG_STAGE_EXTRA_ROWS": "-1000000"},                                                     # one launch per level
    {"HAG_PARTITION_MIN_ROWS": "0", "HAG_PART_MIN": "16", "HAG_PART_SHARE_PCT": "0", "HAG_PART_MEAN_MIN": "0"},   # rows cut by source id
    {"HAG_BLOCK_MAX": "48", "HAG_SUB_MAX": "24"},                                             # split rows, workgroup items
])
def test_max_ties_through_aggregation_rows(B, monkeypatch, knobs):
    # fp32 max looks up the winner stored beside an aggregation row only when a tie needs it: ties
    # between original rows and aggregation rows, and between aggregation rows, in every schedule
    for k, v in knobs.items():
        monkeypatch.setenv(k, v)
    rowptr, col = synth.holme_kim(2500, 12, 0.6, seed=23)
    n = rowptr.size - 1
    h = B.hag_search(rowptr, col, n // 2).upload()
    assert h.stats()["levels"] >= 2
    rng = np.random.default_rng(24)
    for d, levels_of_value in ((8, 2), (64, 4), (132, 50)):
        x = rng.integers(0, levels_of_value, size=(n, d)).astype(np.float32)
        y_ref, _, am_ref = oracle.naive_forward(rowptr, col, x, "max")
        y, am = h.forward(dev(x), "max")
        assert_equal(y, y_ref, f"values d={d}")
        assert_equal(am, am_ref, f"argmax d={d}")
        gy = synth.features_f32(n, d, 25)
        gx_ref, gs = oracle.naive_backward(rowptr, col, gy, "max", am_ref)
        assert_close(h.backward(dev(gy), "max", argmax=am), gx_ref, gs, f"backward d={d}")


def test_empty_graph_and_edgeless_graph(B):
    h = B.hag_search(np.zeros(1, dtype=np.int64), np.zeros(0, dtype=np.int32), 4).upload()
    y = h.forward(torch.empty((0, 8), device="cuda"), "sum")
    assert y.shape == (0, 8)
    n = 70
    h = B.hag_search(np.zeros(n + 1, dtype=np.int64), np.zeros(0, dtype=np.int32), 4).upload()
    x = dev(synth.features_f32(n, 8, 1))
    assert torch.count_nonzero(h.forward(x, "sum")) == 0
    y, am = h.forward(x, "max")
    assert torch.count_nonzero(y) == 0 and bool((am == -1).all())
    assert torch.count_nonzero(h.backward(x, "max", argmax=am)) == 0
    assert torch.count_nonzero(h.backward(x, "mean")) == 0


def test_device_argument_errors(B):
    rowptr, col = synth.random_graph(20, 0.3, seed=1)
    h = B.hag_search(rowptr, col, 4).upload()
    x = torch.zeros((20, 6), device="cuda")
    with pytest.raises(B.HagError) as e:
        h.forward(x, "sum")                      # d not a multiple of 4
    assert e.value.code == B.HAG_EINVAL
    xi = torch.zeros((20, 8), dtype=torch.int32, device="cuda")
    with pytest.raises(B.HagError):
        h.forward(xi, "mean")                    # integer mean is undefined
    x8 = torch.zeros((20, 8), device="cuda")
    with pytest.raises(B.HagError):
        h.forward(x8, "sum", y=x8)               # aliasing


def test_config1_sbm_sum_f32_and_i32(B):
    rowptr, col = synth.sbm()
    n = rowptr.size - 1
    h = B.hag_search(rowptr, col, n // 4)
    ref = oracle.search(rowptr, col, n // 4)     # canonical search parity at full config-1 size
    l, r, red = h.get_merges()
    assert np.array_equal(l, ref.left) and np.array_equal(r, ref.right) and np.array_equal(red, ref.red)
    run_all_ops(B, h, rowptr, col, 64, seed=synth.SEED_BASE + 1001, ops=("sum",))


# ------------------------------------------------------------------------------------------------
# the one-launch schedule: Algorithm 2's loop over V_A and its final loop (resp. their transposes)
# as a single kernel launch whose later phases wait inside the kernel for the earlier ones
# ------------------------------------------------------------------------------------------------
def one_launch_graphs(B, monkeypatch):
    """(name, rowptr, col, handle) of small HAGs with one stage and with several dependent stages, with the
    one-launch schedule (off by default) switched on."""
    monkeypatch.setenv("HAG_FUSE_MAX_ITEMS", "262144")
    out = []
    rowptr, col = synth.holme_kim(3000, 8, 0.5, seed=81)
    out.append(("power-law, fused levels", rowptr, col, B.hag_search(rowptr, col, 750)))
    monkeypatch.setenv("HAG_STAGE_EXTRA_ROWS", "-1000000")            # one stage per level: a chain of phases
    rowptr, col = synth.sbm(n_blocks=4, block=60, p_in=0.5, p_out=0.02, seed=82)
    h = B.hag_search(rowptr, col, rowptr.size - 1)
    assert 3 <= h.stats()["stages"] == h.stats()["levels"] <= 7
    out.append(("sbm, one phase per level", rowptr, col, h))
    monkeypatch.delenv("HAG_STAGE_EXTRA_ROWS")
    monkeypatch.delenv("HAG_FUSE_MAX_ITEMS")
    return out


def test_one_launch_pass_matches_oracle_and_per_stage_launches(B, monkeypatch):
    for name, rowptr, col, h in one_launch_graphs(B, monkeypatch):
        n = rowptr.size - 1
        for d in (16, 64, 256):
            run_all_ops(B, h, rowptr, col, d, seed=83 + d)
            h.check()                                                  # no wait gave up
            # the same handle with one launch per stage: the same additions in the same order
            x, xi = dev(synth.features_f32(n, d, 84)), dev(synth.features_i32(n, d, 85))
            one = [h.forward(x, "sum"), h.backward(x, "mean"), h.forward(x, "gcn"), h.backward(xi, "sum"), *h.forward(x, "max"),
                   *h.forward(xi, "max")]
            h.set_option(B.HAG_OPT_ONE_LAUNCH_MAX_ITEMS, 0)
            per = [h.forward(x, "sum"), h.backward(x, "mean"), h.forward(x, "gcn"), h.backward(xi, "sum"), *h.forward(x, "max"),
                   *h.forward(xi, "max")]
            h.set_option(B.HAG_OPT_ONE_LAUNCH_MAX_ITEMS, 262144)
            for k, (a, b) in enumerate(zip(one, per)):
                assert torch.equal(a, b), (name, d, k)


def test_one_launch_pass_replayed_from_a_hip_graph(B, monkeypatch):
    # the pass resets its own ticket and count (no memset node): replays, with eager work and
    # synchronisations in between, must all give the eager result
    name, rowptr, col, h = one_launch_graphs(B, monkeypatch)[1]
    n, d = rowptr.size - 1, 64
    h.upload()
    x, gy = dev(synth.features_f32(n, d, 86)), dev(synth.features_f32(n, d, 87))
    y, gx = torch.empty_like(x), torch.empty_like(x)
    want_y, want_gx = h.forward(x, "sum").clone(), h.backward(gy, "sum").clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        h.forward(x, "sum", y=y)
        h.backward(gy, "sum", gx=gx)
    torch.cuda.current_stream().wait_stream(side)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        h.forward(x, "sum", y=y)
        h.backward(gy, "sum", gx=gx)
    for rep in range(4):
        y.fill_(-1.0)
        gx.fill_(-1.0)
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, want_y) and torch.equal(gx, want_gx), rep
        assert torch.equal(h.forward(x, "sum"), want_y)               # eager work between the replays
        torch.cuda.synchronize()
    h.check()


def test_one_launch_pass_bounded_wait_gives_up_and_reports(B, monkeypatch):
    # forced from the host: the awaited count is made unreachable and the spin limit tiny, so every
    # wait ends by giving up; the kernel still runs to its end and hag_check reports it
    name, rowptr, col, h = one_launch_graphs(B, monkeypatch)[0]
    n, d = rowptr.size - 1, 32
    h.upload()
    x = dev(synth.features_f32(n, d, 88))
    want = h.forward(x, "sum").clone()
    h.check()
    h.set_option(B.HAG_OPT_TEST_WAIT_UNREACHABLE, 1).set_option(B.HAG_OPT_SPIN_LIMIT, 4)
    h.forward(x, "sum")
    h.backward(x, "sum")
    with pytest.raises(B.HagError) as ei:
        h.check()
    assert ei.value.code == B.HAG_ETIMEOUT
    h.set_option(B.HAG_OPT_TEST_WAIT_UNREACHABLE, 0).set_option(B.HAG_OPT_SPIN_LIMIT, 1 << 18)
    assert torch.equal(h.forward(x, "sum"), want)                      # the next pass is sound again
    h.check()


def test_deterministic_max_backward_is_bit_reproducible_and_matches_oracle(B, monkeypatch):
    # the backward pass of max as a gather over the transposed input graph filtered by argmax (no atomics):
    # int32 bit-exact, fp32 within tolerance and identical from run to run; also with rows cut into pieces
    for env in ({}, {"HAG_PARTITION_MIN_ROWS": "0", "HAG_PART_MIN": "8", "HAG_PART_MEAN_MIN": "0", "HAG_BLOCK_MAX": "40"}):
        for k, v in env.items():
            monkeypatch.setenv(k, v)
        rowptr, col = synth.holme_kim(2500, 9, 0.5, seed=97)
        n = rowptr.size - 1
        h = B.hag_search(rowptr, col, n // 4).upload()
        for k in env:
            monkeypatch.delenv(k)
        for d in (16, 64, 260):
            x, gy = synth.features_f32(n, d, 98), synth.features_f32(n, d, 99)
            xi, gi = synth.features_i32(n, d, 98, lo=-5, hi=5), synth.features_i32(n, d, 99)
            for feats, grads in ((x, gy), (xi, gi)):
                y, am = h.forward(dev(feats), "max")
                _, _, am_ref = oracle.naive_forward(rowptr, col, feats, "max")
                assert_equal(am, am_ref, "argmax")
                gx_ref, gs = oracle.naive_backward(rowptr, col, grads, "max", am_ref)
                atomic = h.backward(dev(grads), "max", argmax=am)
                h.set_option(B.HAG_OPT_DETERMINISTIC_MAX_BACKWARD, 1)
                det = [h.backward(dev(grads), "max", argmax=am).clone() for _ in range(3)]
                det_naive = h.naive_backward(dev(grads), "max", argmax=am)
                h.set_option(B.HAG_OPT_DETERMINISTIC_MAX_BACKWARD, 0)
                torch.cuda.synchronize()
                assert torch.equal(det[0], det[1]) and torch.equal(det[0], det[2]) and torch.equal(det[0], det_naive)
                if feats.dtype == np.int32:
                    assert_equal(det[0], gx_ref, f"deterministic i32 d={d}")
                    assert_equal(atomic, gx_ref, f"atomic i32 d={d}")
                else:
                    assert_close(det[0], gx_ref, gs, f"deterministic f32 d={d}")
                    assert_close(atomic, gx_ref, gs, f"atomic f32 d={d}")
