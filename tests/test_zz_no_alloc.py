"""hag_forward_static_scratch: the forward pass with the library's fixed scratch array as workspace, for
callers that cannot allocate.  Checked against hag_forward (same kernels, caller-owned workspace) and the
oracle, on two calls in a row, the second on a smaller input; sizes beyond the array are refused."""
import ctypes

import numpy as np
import pytest

import oracle
from paper_1906_03707_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1906_03707_amd import binding
    binding.lib()
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def test_static_scratch_forward_matches_forward_on_two_calls_in_a_row(B, monkeypatch):
    # rows cut into pieces and by source id, so that partial rows go through the scratch array as well
    # as the aggregation rows
    monkeypatch.setenv("HAG_PARTITION_MIN_ROWS", "0")
    monkeypatch.setenv("HAG_PART_MIN", "8")
    monkeypatch.setenv("HAG_PART_MEAN_MIN", "0")
    monkeypatch.setenv("HAG_BLOCK_MAX", "40")
    cases = []
    for n, m, d, seed in ((3000, 9, 64, 71), (700, 6, 32, 72)):          # the second input is the smaller one
        rowptr, col = synth.holme_kim(n, m, 0.5, seed=seed)
        h = B.hag_search(rowptr, col, n // 4).upload()
        assert h.stats()["a"] > 0 and 0 < h.workspace_bytes("max", B.HAG_F32, d) <= B.HAG_STATIC_SCRATCH_BYTES
        cases.append((rowptr, col, h, d, seed))
    for rowptr, col, h, d, seed in cases:
        n = rowptr.size - 1
        x, xi = synth.features_f32(n, d, seed + 100), synth.features_i32(n, d, seed + 200)
        for op in ("sum", "mean", "gcn"):
            want = h.forward(dev(x), op)
            got = h.forward_static_scratch(dev(x), op)
            torch.cuda.synchronize()
            y_ref, s, _ = oracle.naive_forward(rowptr, col, x, op)
            assert np.all(np.abs(got.cpu().numpy() - y_ref) <= 1e-5 * s), (n, op)
            assert torch.equal(got, want), (n, op)                         # same kernels, same order of additions
        want = h.forward(dev(xi), "sum")
        got = h.forward_static_scratch(dev(xi), "sum")
        y_ref, _, _ = oracle.naive_forward(rowptr, col, xi, "sum")
        assert np.array_equal(got.cpu().numpy(), y_ref) and torch.equal(got, want)
        for feats in (x, xi):
            wy, wa = h.forward(dev(feats), "max")
            gy_, ga = h.forward_static_scratch(dev(feats), "max")
            y_ref, _, am_ref = oracle.naive_forward(rowptr, col, feats, "max")
            assert np.array_equal(gy_.cpu().numpy().astype(np.float64), y_ref.astype(np.float64))
            assert np.array_equal(ga.cpu().numpy(), am_ref)
            assert torch.equal(gy_, wy) and torch.equal(ga, wa)


def test_static_scratch_refuses_what_does_not_fit_and_what_is_not_uploaded(B):
    rowptr, col = synth.holme_kim(2000, 8, 0.5, seed=73)
    n = rowptr.size - 1
    h = B.hag_search(rowptr, col, n // 4)
    small = torch.zeros((n, 8), dtype=torch.float32, device="cuda")
    with pytest.raises(B.HagError) as ei:
        h.forward_static_scratch(small, "sum")
    assert ei.value.code == B.HAG_ESTATE
    h.upload()
    # a width whose aggregation rows alone exceed the array: refused before anything is launched, so the
    # small buffers handed over are never touched (raw call: the binding would refuse the shapes first)
    d_big = 65536
    assert h.workspace_bytes("sum", B.HAG_F32, d_big) > B.HAG_STATIC_SCRATCH_BYTES
    out = torch.full((n, 8), 7.0, dtype=torch.float32, device="cuda")
    rc = B.lib().hag_forward_static_scratch(h._h, B.HAG_SUM, B.HAG_F32, d_big, ctypes.c_void_p(small.data_ptr()),
                                            ctypes.c_void_p(out.data_ptr()), None, None)
    assert rc == B.HAG_EINVAL and b"static array" in B.lib().hag_last_error()
    torch.cuda.synchronize()
    assert torch.all(out == 7.0)
    # and the handle still works
    y = h.forward_static_scratch(small + 1.0, "sum")
    assert torch.equal(y, h.forward(small + 1.0, "sum"))
