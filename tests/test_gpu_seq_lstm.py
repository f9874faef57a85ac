"""GPU parity of the LSTM aggregator over ordered lists (hag_seq_create / hag_seq_lstm_forward) with
the fp64 oracle (oracle/lstm.py): naive lists and prefix HAGs of several capacities, widths that take
every kernel variant, empty lists, repeated nodes, a ragged last tile of jobs.

Tolerance: the kernel computes every cell in fp32 (fp32 matrix-core products, fp32 exp/tanh); one cell's
pre-activations carry a rounding error of at most about (d + H) * 2^-24 * sum|terms| (a few 1e-6 here), the
gate functions do not amplify it (slopes <= 1) and the state passes it on through the forget gate (< 1), so
over the chains here (<= 40 cells) the outputs, which lie in (-1, 1), stay within 1e-5 of the oracle (observed: 1e-6;
with d + H = 256, twice the terms, 2e-6)."""
import numpy as np
import pytest

from oracle import lstm, sequential
from paper_1906_03707_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

ATOL = 1e-5


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1906_03707_amd import binding
    binding.lib()
    return binding


def params(d, hidden, seed, scale=0.4):
    rng = np.random.default_rng(seed)
    return (rng.normal(0, scale, (4 * hidden, d)), rng.normal(0, scale, (4 * hidden, hidden)), rng.normal(0, scale, 4 * hidden))


def route_graph(n, deg, seed):
    """Ordered lists with common prefixes, empty lists and repeated nodes."""
    rng = np.random.default_rng(seed)
    routes = [rng.permutation(n)[:deg] for _ in range(5)]
    rowptr, col = [0], []
    for v in range(n):
        k = int(rng.integers(0, deg + 1))
        col += list(routes[int(rng.integers(0, 5))][:k]) + list(rng.integers(0, n, int(rng.integers(0, 4))))
        rowptr.append(len(col))
    return np.asarray(rowptr, dtype=np.int64), np.asarray(col, dtype=np.int32)


def first_neighbours(rowptr, col, k):
    """Every list cut to its first k entries (ascending ids: hubs first, so prefixes are shared)."""
    n = rowptr.size - 1
    keep = [col[rowptr[v]:min(rowptr[v + 1], rowptr[v] + k)] for v in range(n)]
    return np.concatenate([[0], np.cumsum([len(x) for x in keep])]).astype(np.int64), np.concatenate(keep).astype(np.int32)


def check(B, rowptr, col, d, hidden, seed, capacities):
    n = rowptr.size - 1
    w_ih, w_hh, b = params(d, hidden, seed)
    x = np.random.default_rng(seed + 1).normal(size=(n, d))
    want, cells_naive = lstm.naive_aggregate(rowptr, col, x, w_ih, w_hh, b)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    xd, wid, whd, bd = dev(x), dev(w_ih), dev(w_hh), dev(b)
    # the oracle sees the same fp32-rounded inputs
    want, _ = lstm.naive_aggregate(rowptr, col, xd.cpu().numpy().astype(np.float64), wid.cpu().numpy().astype(np.float64),
                                   whd.cpu().numpy().astype(np.float64), bd.cpu().numpy().astype(np.float64))
    worst = 0.0
    for cap in capacities:
        h = B.SeqHag(rowptr, col, cap).upload()
        merges, lists = sequential.search(rowptr, col, cap)
        if cap == 0:
            assert h.cells == cells_naive and h.merges == 0
        else:
            _, cells = lstm.hag_aggregate(n, merges, lists, x, w_ih, w_hh, b)
            assert h.merges == len(merges)
            assert h.cells == cells
        per_mode = []
        for one_launch in (1, 0):       # all levels in one launch (paths wait for their start states) / one launch per level
            h.set_option(B.HAG_OPT_SEQ_ONE_LAUNCH, one_launch)
            for rep in range(2):        # the second call reuses the state rows and flags of the first
                got_t = h.lstm_forward(xd, wid, whd, bd)
                h.check()
                got = got_t.cpu().numpy().astype(np.float64)
                err = np.abs(got - want).max() if got.size else 0.0
                worst = max(worst, err)
                assert err <= ATOL, f"cap {cap} d {d} H {hidden} one_launch {one_launch}: max |gpu - oracle| = {err}"
                empty = np.diff(rowptr) == 0
                assert not got[empty].any()
            per_mode.append(got)
        assert np.array_equal(per_mode[0], per_mode[1])      # the same arithmetic either way
    return worst


@pytest.mark.parametrize("d,hidden", [(8, 8), (16, 32), (4, 16), (64, 64), (24, 40), (96, 32),
                                      # the variants that stream the weights: hidden > 64 or d + hidden > 128
                                      (64, 128), (128, 128), (32, 96), (128, 64), (120, 72), (4, 72)])
def test_route_graph_all_kernel_variants(B, d, hidden):
    rowptr, col = route_graph(150, 9, seed=d + hidden)
    check(B, rowptr, col, d, hidden, seed=5, capacities=(0, 7, col.size))


def test_power_law_graph_first_neighbours(B):
    # a Holme-Kim graph, every list cut to its 16 smallest ids: thousands of jobs per rank (several tiles per
    # workgroup, ragged last tile), deep prefix sharing
    rowptr, col = synth.holme_kim(3000, 8, 0.5, seed=77)
    rowptr, col = first_neighbours(rowptr, col, 16)
    n = rowptr.size - 1
    worst = check(B, rowptr, col, 32, 32, seed=9, capacities=(0, n // 4, col.size))
    h0, h1 = B.SeqHag(rowptr, col, 0), B.SeqHag(rowptr, col, col.size)
    print(f"cells naive {h0.cells} prefix HAG {h1.cells} ({h0.cells / h1.cells:.2f}x fewer), ranks {h0.ranks}/{h1.ranks}, max error {worst:.2e}")
    assert h1.cells < h0.cells


@pytest.mark.timeout(600)
@pytest.mark.parametrize("width", [64, 128])                 # weights in registers / streamed
def test_bench_workload_sampled_nodes(B, width):
    # the workload bench.py --seq-lstm times, at its full size and in its launch configuration (config 4's graphs,
    # first 16 neighbours, d = H = 64, and d = H = 128 as with --d 128; plain lists, capacity |V|/4, unlimited): the oracle walks the lists of sampled
    # nodes one by one
    from paper_1906_03707_amd import workloads
    cfg, d, hidden = 4, width, width
    rowptr, col, _ = synth.graph_for_config(cfg)
    n = rowptr.size - 1
    rp, cl = workloads.first_neighbour_lists(rowptr, col, 16)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    xd, wid, whd, bd = (dev(a) for a in workloads.lstm_inputs(cfg, n, d, hidden))
    x64, wi64, wh64, b64 = (t.cpu().numpy().astype(np.float64) for t in (xd, wid, whd, bd))
    sample = np.unique(np.concatenate([np.random.default_rng(5).integers(0, n, 400), [0, n - 1]]))
    s_rp = np.concatenate([[0], np.cumsum(rp[sample + 1] - rp[sample])]).astype(np.int64)
    s_cl = np.concatenate([cl[rp[v]:rp[v + 1]] for v in sample]).astype(np.int32)
    want, _ = lstm.naive_aggregate(s_rp, s_cl, x64, wi64, wh64, b64)
    results = []
    for cap in (0, n // 4, int(cl.size)):
        h = B.SeqHag(rp, cl, cap).upload()
        got = h.lstm_forward(xd, wid, whd, bd)
        h.check()
        err = np.abs(got[torch.from_numpy(sample).cuda()].cpu().numpy().astype(np.float64) - want).max()
        print(f"capacity {cap}: {h.cells} cells, {h.plan()[4].size - 1} levels, max |gpu - oracle| on {sample.size} nodes = {err:.2e}", flush=True)
        assert err <= ATOL
        results.append(got)
    # the three plans evaluate the same cells in the same order along every list
    assert torch.equal(results[0], results[1]) and torch.equal(results[0], results[2])


def test_degenerate_shapes(B):
    # no nodes; nodes without any list; one-entry lists only (every a_v is a shared one-element prefix); one list much
    # longer than a tile is wide, next to short ones (a tile whose paths end far apart); a list that repeats one node
    d, hidden = 8, 16
    w_ih, w_hh, b = params(d, hidden, 2)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    wid, whd, bd = dev(w_ih), dev(w_hh), dev(b)
    h = B.SeqHag(np.zeros(1, dtype=np.int64), np.zeros(0, dtype=np.int32), 4).upload()
    assert h.cells == 0 and h.launches == 0
    assert h.lstm_forward(torch.zeros((0, d), device="cuda"), wid, whd, bd).shape == (0, hidden)
    rng = np.random.default_rng(3)
    cases = {
        "all empty": (np.zeros(6, dtype=np.int64), np.zeros(0, dtype=np.int32)),
        "one entry each": (np.arange(0, 41, dtype=np.int64), rng.integers(0, 5, 40).astype(np.int32)),
        "one long list": (np.concatenate([[0], np.cumsum([300] + [2] * 99)]).astype(np.int64),
                          np.concatenate([rng.integers(0, 100, 300), np.tile([7, 9], 99)]).astype(np.int32)),
        "one node repeated": (np.array([0, 50, 75, 75], dtype=np.int64), np.full(75, 2, dtype=np.int32)),
    }
    for name, (rowptr, col) in cases.items():
        n = rowptr.size - 1
        x = np.random.default_rng(4).normal(size=(n, d))
        xd = dev(x)
        want, _ = lstm.naive_aggregate(rowptr, col, xd.cpu().numpy().astype(np.float64), wid.cpu().numpy().astype(np.float64),
                                       whd.cpu().numpy().astype(np.float64), bd.cpu().numpy().astype(np.float64))
        for cap in (0, max(n // 4, 1), max(int(col.size), 1)):
            h = B.SeqHag(rowptr, col, cap).upload()
            for one_launch in (1, 0):
                h.set_option(B.HAG_OPT_SEQ_ONE_LAUNCH, one_launch)
                got = h.lstm_forward(xd, wid, whd, bd)
                h.check()
                err = np.abs(got.cpu().numpy().astype(np.float64) - want).max() if n else 0.0
                # 300 steps: the forget gate keeps the accumulated rounding error bounded, the tolerance of the short chains holds
                assert err <= ATOL, f"{name}, capacity {cap}, one_launch {one_launch}: {err}"


def test_rejections(B):
    rowptr, col = route_graph(20, 4, seed=3)
    h = B.SeqHag(rowptr, col, 3)
    x = torch.zeros((20, 8), device="cuda")
    w_ih, w_hh, b = torch.zeros((32, 8), device="cuda"), torch.zeros((32, 8), device="cuda"), torch.zeros(32, device="cuda")
    with pytest.raises(B.HagError):       # before upload
        h.lstm_forward(x, w_ih, w_hh, b)
    h.upload()
    h.lstm_forward(x, w_ih, w_hh, b)
    with pytest.raises(ValueError):       # wrong shape
        h.lstm_forward(x[:10].contiguous(), w_ih, w_hh, b)
    with pytest.raises(B.HagError):       # hidden not a multiple of 8
        h.lstm_forward(x, torch.zeros((16, 8), device="cuda"), torch.zeros((16, 4), device="cuda"), torch.zeros(16, device="cuda"))
    with pytest.raises(B.HagError):       # hidden above the kernel's limit
        h.lstm_forward(x, torch.zeros((544, 8), device="cuda"), torch.zeros((544, 136), device="cuda"), torch.zeros(544, device="cuda"))
    with pytest.raises(B.HagError):       # d + hidden above the kernel's limit
        h.lstm_forward(torch.zeros((20, 192), device="cuda"), torch.zeros((320, 192), device="cuda"), torch.zeros((320, 80), device="cuda"),
                       torch.zeros(320, device="cuda"))


def test_bounded_wait_gives_up_and_reports(B):
    # forced from the host: no "state is written" flag is ever set and the spin limit is tiny, so every wait of the
    # one-launch pass ends by giving up; the kernel still runs to its end and hag_seq_check reports it
    rowptr, col = route_graph(300, 9, seed=31)
    d = hidden = 16
    w_ih, w_hh, b = (torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda() for a in params(d, hidden, 3))
    h = B.SeqHag(rowptr, col, col.size).upload()
    assert h.plan()[4].size - 1 > 1                          # more than one level: there are waits
    x = torch.randn((300, d), device="cuda")
    want = h.lstm_forward(x, w_ih, w_hh, b).clone()
    h.check()
    h.set_option(B.HAG_OPT_TEST_WAIT_UNREACHABLE, 1).set_option(B.HAG_OPT_SPIN_LIMIT, 4)
    h.lstm_forward(x, w_ih, w_hh, b)
    with pytest.raises(B.HagError) as ei:
        h.check()
    assert ei.value.code == B.HAG_ETIMEOUT
    h.set_option(B.HAG_OPT_TEST_WAIT_UNREACHABLE, 0).set_option(B.HAG_OPT_SPIN_LIMIT, 1 << 21)
    assert torch.equal(h.lstm_forward(x, w_ih, w_hh, b), want)           # the next pass is sound again
    h.check()


def test_replay_from_a_hip_graph(B):
    # the pass allocates nothing and records no memset: captured once, replayed with eager work in between, every
    # replay against the eager result (new inputs each time)
    rowptr, col = route_graph(400, 9, seed=21)
    d = hidden = 32
    w_ih, w_hh, b = (torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda() for a in params(d, hidden, 13))
    h = B.SeqHag(rowptr, col, col.size).upload()
    x = torch.randn((400, d), device="cuda")
    out = torch.empty((400, hidden), device="cuda")
    ws = torch.empty(h.workspace_bytes(d, hidden), dtype=torch.uint8, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        h.lstm_forward(x, w_ih, w_hh, b, out=out, workspace=ws)
    torch.cuda.current_stream().wait_stream(side)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        h.lstm_forward(x, w_ih, w_hh, b, out=out, workspace=ws)
    for rep in range(3):
        x.copy_(torch.randn((400, d), device="cuda"))
        want = h.lstm_forward(x, w_ih, w_hh, b).clone()      # eager, its own workspace
        torch.cuda.synchronize()
        out.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want), f"replay {rep}"
