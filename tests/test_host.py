"""Host logic of libhag (no GPU): exports, validation, search vs the oracle's brute-force
Algorithm 3, replay of merge lists, level ordering, statistics."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from paper_1906_03707_amd import binding as B
from paper_1906_03707_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def oracle_view(h: B.Hag) -> oracle.Hag:
    """The library's level-ordered forward form as an oracle HAG (level order is topological)."""
    f = h.get_forward()
    return oracle.Hag(h.stats()["n"], f["agg_left"], f["agg_right"], f["hrowptr"], f["hcol"])


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "hag.h")).read()
    declared = set(re.findall(r"\b(hag_[a-z0-9_]+)\s*\(", header))
    declared -= {"hag_handle"}
    assert declared == set(B.EXPORTS)
    L = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(L, name), name


@pytest.mark.parametrize("seed", range(8))
def test_search_matches_oracle_on_small_graphs(seed):
    n = 24 + 3 * seed
    rowptr, col = synth.random_graph(n, 0.3 + 0.05 * (seed % 3), seed=900 + seed, directed=(seed % 2 == 1))
    for cap in (0, 1, n // 4, n):
        ref = oracle.search(rowptr, col, cap)
        h = B.hag_search(rowptr, col, cap)
        l, r, red = h.get_merges()
        assert np.array_equal(l, ref.left) and np.array_equal(r, ref.right) and np.array_equal(red, ref.red)
        ov = oracle_view(h)
        assert oracle.cover_check(rowptr, col, ov) == 0
        st = h.stats()
        assert st["a"] == ref.a and st["aggr_hag"] == ref.aggregations() and st["e_hag"] == ref.edges()
        assert st["aggr_naive"] == int(np.maximum(np.diff(rowptr) - 1, 0).sum()) and st["e"] == col.size


def test_search_matches_oracle_on_sbm_blocks():
    rowptr, col = synth.sbm(n_blocks=6, block=48, p_in=0.3, p_out=0.01, seed=77)
    n = rowptr.size - 1
    ref = oracle.search(rowptr, col, n // 4)
    h = B.hag_search(rowptr, col, n // 4)
    l, r, red = h.get_merges()
    assert np.array_equal(l, ref.left) and np.array_equal(r, ref.right) and np.array_equal(red, ref.red)


@pytest.mark.parametrize("n,n_blocks,mean_degree,seed", [(1500, 6, 8.5, 102), (1800, 8, 10.0, 100)])
def test_search_to_exhaustion_matches_oracle(n, n_blocks, mean_degree, seed):
    # Capacity beyond what the graph can use: the search runs until no pair is shared twice, through long
    # chains of aggregation nodes built on aggregation nodes.  Graphs on which a bound that pruned the
    # descendants of a partner by that partner's current count (its rows had moved on to them) lost a pair.
    rowptr, col = synth.dcsbm(n=n, n_blocks=n_blocks, mean_degree=mean_degree, seed=seed)
    ref = oracle.search(rowptr, col, 2 * n)
    h = B.hag_search(rowptr, col, 2 * n)
    l, r, red = h.get_merges()
    assert ref.a == l.size < 2 * n and ref.red[-1] == 2
    assert np.array_equal(l, ref.left) and np.array_equal(r, ref.right) and np.array_equal(red, ref.red)


def test_level_order_and_forward_form():
    rowptr, col = synth.sbm(n_blocks=3, block=40, p_in=0.5, p_out=0.02, seed=78)
    n = rowptr.size - 1
    h = B.hag_search(rowptr, col, n)
    f = h.get_forward()
    st = h.stats()
    a, L = st["a"], st["levels"]
    assert L == f["n_levels"] and f["level_ptr"][0] == 0 and f["level_ptr"][-1] == a and L >= 2
    depth = np.zeros(n + a, dtype=np.int64)
    for i in range(a):
        l, r = f["agg_left"][i], f["agg_right"][i]
        assert l < r < n + i
        depth[n + i] = 1 + max(depth[l], depth[r])
    for lv in range(1, L + 1):
        assert np.all(depth[n + f["level_ptr"][lv - 1]: n + f["level_ptr"][lv]] == lv)
    for v in range(n):
        assert np.all(np.diff(f["hcol"][f["hrowptr"][v]:f["hrowptr"][v + 1]]) > 0)
    # every aggregation node is consumed at least twice in total (Algorithm 3 merges only when > 1)
    uses = np.bincount(np.concatenate([f["hcol"], f["agg_left"], f["agg_right"]]), minlength=n + a)
    assert uses[n:].min() >= 1
    # oracle agrees that HAG forward == naive on the level-ordered form
    x = synth.features_i32(n, 4, 1)
    ov = oracle_view(h)
    assert np.array_equal(oracle.hag_forward(ov, np.diff(rowptr), x, "sum")[0], oracle.naive_forward(rowptr, col, x, "sum")[0])


def test_from_merges_and_prefix_replay():
    rowptr, col = synth.random_graph(40, 0.4, seed=5)
    h = B.hag_search(rowptr, col, 20)
    l, r, red = h.get_merges()
    h2 = B.hag_from_merges(rowptr, col, l, r)
    assert h2.stats() == h.stats()
    f1, f2 = h.get_forward(), h2.get_forward()
    for k in f1:
        assert np.array_equal(f1[k], f2[k])
    for k in (0, 1, len(l) // 2, len(l)):
        hp = h.prefix(k)
        hk = B.hag_search(rowptr, col, k)
        assert hp.stats() == hk.stats()
        assert np.array_equal(hp.get_forward()["hcol"], hk.get_forward()["hcol"])
    aggr = [h.prefix(k).stats()["aggr_hag"] for k in range(len(l) + 1)]
    assert all(x > y for x, y in zip(aggr, aggr[1:]))          # every merge saves r-1 >= 1
    assert [x - y for x, y in zip(aggr, aggr[1:])] == (red - 1).tolist()


def test_max_depth_limits_levels():
    rowptr, col = synth.sbm(n_blocks=2, block=48, p_in=0.6, p_out=0.05, seed=79)
    n = rowptr.size - 1
    free = B.hag_search(rowptr, col, n)
    assert free.stats()["levels"] > 2
    for md in (1, 2):
        h = B.hag_search(rowptr, col, n, max_depth=md)
        assert 0 < h.stats()["levels"] <= md
        assert oracle.cover_check(rowptr, col, oracle_view(h)) == 0


def test_batched_search_equals_per_graph_search():
    rowptr, col, gp = synth.er_batch(6, 20, 0.8, seed=9)
    h = B.hag_search_batched(rowptr, col, gp, 0.25)
    st = h.stats()
    assert st["a"] == 6 * 5
    assert oracle.cover_check(rowptr, col, oracle_view(h)) == 0
    l, r, _ = h.get_merges()
    n = rowptr.size - 1
    off = 0
    for g in range(6):
        v0, v1 = gp[g], gp[g + 1]
        sub_ptr = rowptr[v0:v1 + 1] - rowptr[v0]
        sub_col = col[rowptr[v0]:rowptr[v1]] - v0
        ref = oracle.search(sub_ptr, sub_col, 5)
        nv = v1 - v0
        mp = lambda t: np.where(t < nv, t + v0, n + off + (t - nv))
        assert np.array_equal(l[off:off + ref.a], mp(ref.left)) and np.array_equal(r[off:off + ref.a], mp(ref.right))
        off += ref.a


def test_validation_errors():
    rowptr = np.array([0, 2, 3], dtype=np.int64)
    col = np.array([1, 1, 0], dtype=np.int32)
    with pytest.raises(B.HagError) as e:
        B.hag_search(rowptr, col, 1)
    assert e.value.code == B.HAG_EINVAL and "duplicate" in str(e.value)
    h = B.hag_search(rowptr, col, 1, flags=B.HAG_SEARCH_DEDUP)
    assert h.stats()["e"] == 2
    for bad_ptr, bad_col in (([0, 2, 1], [1, 0]), ([0, 1, 2], [1, 5]), ([1, 1, 2], [0, 1])):
        with pytest.raises(B.HagError) as e:
            B.hag_search(np.array(bad_ptr, dtype=np.int64), np.array(bad_col, dtype=np.int32), 1)
        assert e.value.code == B.HAG_EINVAL
    good_ptr, good_col = np.array([0, 1, 2], dtype=np.int64), np.array([1, 0], dtype=np.int32)
    with pytest.raises(B.HagError):
        B.hag_search(good_ptr, good_col, -1)
    with pytest.raises(B.HagError):
        B.hag_from_merges(good_ptr, good_col, [0], [0])      # equal inputs
    with pytest.raises(B.HagError):
        B.hag_from_merges(good_ptr, good_col, [0], [5])      # unknown node
    with pytest.raises(B.HagError):
        B.hag_from_merges(good_ptr, good_col, [0], [1])      # used by no list
    # device entry point before upload -> HAG_ESTATE (no GPU needed: the check precedes any HIP call)
    h = B.hag_search(good_ptr, good_col, 0)
    rc = B.lib().hag_forward(h._h, B.HAG_SUM, B.HAG_F32, 4, 16, 32, None, None, None)
    assert rc == B.HAG_ESTATE and b"hag_upload" in B.lib().hag_last_error()


def test_device_counted_search_needs_a_device():
    # without a GPU the flag must fail loudly, not fall back to the host threads
    torch = pytest.importorskip("torch")
    if torch.cuda.is_available():
        pytest.skip("a GPU is visible: the flag works (covered by the gpu tests)")
    rowptr, col = synth.random_graph(30, 0.4, seed=6)
    with pytest.raises(B.HagError) as e:
        B.hag_search(rowptr, col, 10, flags=B.HAG_SEARCH_DEVICE)
    assert e.value.code == B.HAG_EHIP
    # capacity 0 needs no counting at all
    assert B.hag_search(rowptr, col, 0, flags=B.HAG_SEARCH_DEVICE).stats()["a"] == 0


def test_search_checkpoint_holds_a_prefix_of_the_merge_list(tmp_path, monkeypatch, capfd):
    # HAG_SEARCH_PROGRESS=<every> prints a line and, with HAG_SEARCH_CHECKPOINT=<file>, dumps the merges so
    # far (int64 count, then left[], right[] as int32), so that a long search can be resumed by replay
    rowptr, col = synth.sbm(n_blocks=4, block=40, p_in=0.4, p_out=0.02, seed=81)
    n = rowptr.size - 1
    path = tmp_path / "merges.bin"
    monkeypatch.setenv("HAG_SEARCH_PROGRESS", "7")
    monkeypatch.setenv("HAG_SEARCH_CHECKPOINT", str(path))
    h = B.hag_search(rowptr, col, n // 2)
    assert "[hag_search]" in capfd.readouterr().err
    left, right, _ = h.get_merges()
    raw = path.read_bytes()
    k = int(np.frombuffer(raw[:8], dtype=np.int64)[0])
    assert k > 0 and k % 7 == 0 and k <= left.size and len(raw) == 8 + 8 * k
    assert np.array_equal(np.frombuffer(raw[8:8 + 4 * k], dtype=np.int32), left[:k])
    assert np.array_equal(np.frombuffer(raw[8 + 4 * k:], dtype=np.int32), right[:k])
    monkeypatch.delenv("HAG_SEARCH_PROGRESS")
    monkeypatch.delenv("HAG_SEARCH_CHECKPOINT")
    resumed = B.hag_from_merges(rowptr, col, left[:k], right[:k])
    assert resumed.stats() == h.prefix(k).stats()


def test_empty_and_isolated():
    h = B.hag_search(np.zeros(1, dtype=np.int64), np.zeros(0, dtype=np.int32), 4)
    assert h.stats()["n"] == 0 and h.stats()["a"] == 0
    rowptr = np.array([0, 0, 0, 0], dtype=np.int64)
    h = B.hag_search(rowptr, np.zeros(0, dtype=np.int32), 2)
    assert h.stats()["a"] == 0 and h.stats()["aggr_naive"] == 0


def test_config1_search_invariants():
    rowptr, col = synth.sbm()
    n = rowptr.size - 1
    h = B.hag_search(rowptr, col, n // 4)
    st = h.stats()
    l, r, red = h.get_merges()
    assert st["a"] == n // 4 and np.all(np.diff(red) <= 0) and red.min() >= 2
    assert oracle.cover_check(rowptr, col, oracle_view(h)) == 0
    assert st["aggr_naive"] - st["aggr_hag"] == int((red - 1).sum())
    assert st["e"] - st["e_hag"] == int((red - 2).sum())


def test_stage_fusion_and_component_detection(monkeypatch):
    # levels are fused into stages when that is cheap; a batch of small graphs with contiguous ids is
    # recognised as such (one workgroup per component on the device), anything else is not
    rowptr, col, gp = synth.er_batch(100, 16, 0.7, seed=12)
    h = B.hag_search_batched(rowptr, col, gp, 0.25)
    st = h.stats()
    assert 1 <= st["stages"] <= st["levels"] and st["components"] == 100
    assert oracle.cover_check(rowptr, col, oracle_view(h)) == 0
    # graphs that are not connected still give contiguous ranges: at most one range per component
    rp, cl, gq = synth.er_batch(200, 9, 0.25, seed=15)
    hb = B.hag_search_batched(rp, cl, gq, 0.25)
    assert 200 <= hb.stats()["components"] < rp.size - 1
    monkeypatch.setenv("HAG_STAGE_EXTRA_ROWS", "-1000000")
    assert B.hag_search_batched(rowptr, col, gp, 0.25).stats()["stages"] == st["levels"]
    monkeypatch.delenv("HAG_STAGE_EXTRA_ROWS")
    # the same graphs with node ids shuffled: components are no longer contiguous ranges
    n = rowptr.size - 1
    perm = np.random.default_rng(13).permutation(n)
    rows = perm[np.repeat(np.arange(n), np.diff(rowptr))]
    cols = perm[col]
    order = np.lexsort((cols, rows))
    rp2 = np.concatenate([[0], np.cumsum(np.bincount(rows, minlength=n))]).astype(np.int64)
    h2 = B.hag_search(rp2, cols[order].astype(np.int32), n // 4)
    assert h2.stats()["components"] == 0
    # one connected graph: no components either
    rowptr, col = synth.sbm(n_blocks=8, block=160, p_in=0.1, p_out=0.01, seed=14)
    assert B.hag_search(rowptr, col, 64).stats()["components"] == 0
    # workspace grows with d and covers the aggregation rows
    h3 = B.hag_search(rowptr, col, 64)
    a = h3.stats()["a"]
    assert h3.workspace_bytes("sum", B.HAG_F32, 64) >= a * 64 * 4
    assert h3.workspace_bytes("max", B.HAG_F32, 64) >= 2 * a * 64 * 4
    assert h3.workspace_bytes("sum", B.HAG_F32, 128) > h3.workspace_bytes("sum", B.HAG_F32, 64)


def test_build_rejects_kernels_that_use_scratch_memory():
    # build.py reads the compiler's per-kernel resource remarks: a kernel whose arguments or
    # registers end up in scratch memory still passes every parity test, only several times slower
    from paper_1906_03707_amd.build import check_resource_usage

    def remarks(scratch):
        rows = ["Function Name: _ZN3hag13gather_kernelIfLi1ELi32ELi0EEEvNS_10GatherArgsIT_EE", "    VGPRs: 62",
                f"    ScratchSize [bytes/lane]: {scratch}", "    LDS Size [bytes/block]: 8192"]
        return "\n".join(f"x.hip:271:1: remark: {r} [-Rpass-analysis=kernel-resource-usage]" for r in rows)

    usage = check_resource_usage(remarks(0))
    (name, u), = usage.items()
    assert name.startswith("_ZN3hag13gather_kernel") and u["VGPRs"] == "62" and u["LDS Size [bytes/block]"] == "8192"
    with pytest.raises(RuntimeError, match="scratch"):
        check_resource_usage(remarks(344))


def test_binding_rejects_misshaped_tensors_before_the_call():
    # the C ABI takes raw pointers and no row count: the binding must refuse anything that would
    # make a kernel run out of bounds (checked on CPU tensors: the refusal comes before any launch)
    import torch

    rowptr, col = synth.random_graph(40, 0.2, seed=3)
    h = B.hag_search(rowptr, col, 10)
    n = 40
    ok = torch.zeros((n, 8), dtype=torch.float32)
    with pytest.raises(ValueError, match="shape"):
        h.forward(torch.zeros((n - 1, 8), dtype=torch.float32))
    with pytest.raises(ValueError, match="shape"):
        h.backward(torch.zeros((n + 5, 8), dtype=torch.float32))
    with pytest.raises(ValueError, match="output"):
        h.forward(ok, y=torch.zeros((n, 8), dtype=torch.float16))
    with pytest.raises(ValueError, match="output"):
        h.forward(ok, y=torch.zeros((n, 4), dtype=torch.float32))
    with pytest.raises(ValueError, match="argmax"):
        h.forward(ok, "max", argmax=torch.zeros((n, 8), dtype=torch.int64))
    with pytest.raises(ValueError, match="argmax"):
        h.backward(ok, "max")
    with pytest.raises(ValueError, match="workspace"):
        h.forward(ok, workspace=torch.zeros(16, dtype=torch.uint8))
    with pytest.raises(ValueError, match="unknown op"):
        h.forward(ok, "prod")
    with pytest.raises(TypeError):
        h.forward(torch.zeros((n, 8), dtype=torch.float64))
    # a well-formed call on CPU tensors still never reaches the library
    with pytest.raises(ValueError, match="GPU"):
        h.forward(ok, workspace=torch.zeros(1 << 20, dtype=torch.uint8))
