"""GPU parity for the thresholded sparse proximity (strict upper triangle as coordinate triplets).
The order of the triplets is unspecified, so both sides are compared as sorted lists."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch


def _dev(torch, leaf):
    return torch.from_numpy(np.ascontiguousarray(leaf).view(np.int32)).cuda()


def _sorted_triplets(rows, cols, counts, prox=None):
    r = rows.cpu().numpy().astype(np.int64)
    c = cols.cpu().numpy().astype(np.int64)
    v = counts.cpu().numpy()
    v = v.view(np.uint16) if v.dtype == np.int16 else v.view(np.uint32)
    order = np.lexsort((c, r))
    p = prox.cpu().numpy()[order] if prox is not None else None
    return r[order], c[order], v[order].astype(np.uint32), p


def _compare(torch, rfx, oracle, leaf, bound, min_count, dtype):
    """Both ways the library computes the list (pair tests on bit planes: "auto" on these shallow cases; row by row from
    the samples grouped by leaf: "rows") against the oracle's."""
    B, N = leaf.shape
    rr, rc, rv = oracle.sparse_upper(leaf, min_count)
    for method in ("auto", "rows"):
        assert rfx.prox_sparse_count(_dev(torch, leaf), bound, min_count, method) == rr.size, method
        rows, cols, counts, prox = rfx.prox_sparse(_dev(torch, leaf), bound, min_count, count_dtype=dtype, want_prox=True,
                                                   method=method)
        r, c, v, p = _sorted_triplets(rows, cols, counts, prox)
        np.testing.assert_array_equal(r, rr, err_msg=method)
        np.testing.assert_array_equal(c, rc, err_msg=method)
        np.testing.assert_array_equal(v, rv, err_msg=method)
        np.testing.assert_array_equal(p, (rv.astype(np.float32) / np.float32(B)).astype(np.float32), err_msg=method)


@pytest.mark.parametrize("N,B,bound", [(1, 3, 5), (2, 1, 2), (255, 31, 40), (256, 32, 40), (257, 33, 40), (515, 65, 2),
                                       (300, 97, 1), (1100, 40, 3000), (70000, 5, 9000), (32769, 3, 600), (65536, 2, 40000)])
# (a dense case with N > 32768, where a chunk of the row pass keeps more pairs than it has counter words, is
# test_row_pass_on_a_nearly_dense_matrix below: the oracle's list would be too long there)
def test_sparse_on_boundary_shapes(torch_cuda, N, B, bound):
    import oracle
    import paper_2511_19493_amd as rfx
    print(f"sparse boundary shapes N={N} B={B} bound={bound}", flush=True)
    rng = np.random.default_rng(7000 * N + B)
    leaf = rng.integers(0, bound, size=(B, N)).astype(np.uint32)
    if N > 20000:            # several column chunks of the row pass; the oracle needs seconds per list here
        leaf[:, N - 3:] = leaf[:, :1]       # pairs across the first and the last chunk
        _compare(torch_cuda, rfx, oracle, leaf, bound, 1, rfx.U32)
        _compare(torch_cuda, rfx, oracle, leaf, bound, 2, rfx.U16)
        return
    for min_count in sorted({1, 2, max(1, B // 4), B}):
        _compare(torch_cuda, rfx, oracle, leaf, bound, min_count, rfx.U32)
    if B <= 65535:
        _compare(torch_cuda, rfx, oracle, leaf, bound, 1, rfx.U16)


def test_sparse_on_grown_forests(torch_cuda, cfg1, small2):
    import oracle
    import paper_2511_19493_amd as rfx
    for name, w in (("cfg1", cfg1), ("small2", small2)):
        leaf = w["leaf"]
        B, N = leaf.shape
        bound = int(leaf.max()) + 1
        print(f"sparse {name} N={N} B={B}", flush=True)
        for min_count in (1, 3, B // 2):
            _compare(torch_cuda, rfx, oracle, leaf, bound, min_count, rfx.U16)
        # the list with min_count 1 is an exact representation: it rebuilds the dense counts
        rows, cols, counts, _ = rfx.prox_sparse(_dev(torch_cuda, leaf), bound, 1)
        dense = np.zeros((N, N), np.uint32)
        r, c, v, _ = _sorted_triplets(rows, cols, counts)
        dense[r, c] = v
        dense = dense + dense.T
        np.fill_diagonal(dense, B)
        np.testing.assert_array_equal(dense, oracle.counts_full(leaf))


def test_sparse_capacity_and_argument_errors(torch_cuda, cfg1):
    import oracle
    import paper_2511_19493_amd as rfx
    torch = torch_cuda
    leaf = cfg1["leaf"]
    B, N = leaf.shape
    bound = int(leaf.max()) + 1
    d = _dev(torch, leaf)
    need = oracle.sparse_upper(leaf, 1)[0].size
    assert need > 10
    with pytest.raises(rfx.RfxError) as e:
        rfx.prox_sparse(d, bound, 1, capacity=need - 1)
    assert e.value.code == rfx.ERR_CAPACITY and str(need) in str(e.value)
    rows, cols, counts, _ = rfx.prox_sparse(d, bound, 1, capacity=need)         # exactly enough
    assert rows.numel() == need
    rows, cols, counts, _ = rfx.prox_sparse(d, bound, 1, capacity=need + 1000)  # more than enough: trimmed
    assert rows.numel() == need
    with pytest.raises(rfx.RfxError) as e:
        rfx.prox_sparse(d, bound, 0)
    assert e.value.code == rfx.ERR_INVALID_ARG
    # nothing qualifies: empty list, no error
    rows, cols, counts, _ = rfx.prox_sparse(d, bound, B + 1, capacity=16)
    assert rows.numel() == 0
    # two calls in a row give the same set (the order may differ)
    a = _sorted_triplets(*rfx.prox_sparse(d, bound, 2)[:3])
    b = _sorted_triplets(*rfx.prox_sparse(d, bound, 2)[:3])
    for x, y in zip(a[:3], b[:3]):
        np.testing.assert_array_equal(x, y)


def test_row_pass_from_an_existing_plan(torch_cuda, small2):
    """rfx_prox_sparse_plan: the list from the plan of the implicit product, asynchronous, nothing allocated inside; the
    triplets against the oracle's, and the plan serves the implicit product afterwards exactly as a fresh one does
    (the marks the row pass leaves in its member lists are taken out again)."""
    import oracle
    import paper_2511_19493_amd as rfx
    import rfx_inputs as ri
    torch = torch_cuda
    cases = [("small2", small2["leaf"][:48], int(small2["leaf"][:48].max()) + 1)]
    rng = np.random.default_rng(31)
    cases.append(("random ids, three column chunks", rng.integers(0, 7000, size=(4, 70001)).astype(np.uint32), 7000))
    for name, leaf, bound in cases:
        B, N = leaf.shape
        print(f"row pass from a plan: {name} N={N} B={B}", flush=True)
        d = _dev(torch, leaf)
        plan = rfx.PvPlan(d, bound)
        V = torch.from_numpy(ri.start_block(N, 24)).cuda()
        y_before = plan.apply(V).clone()
        ws = rfx.new_workspace(rfx.prox_sparse_plan_workspace_bytes(plan))
        nnz = torch.full((1,), -1, dtype=torch.int64, device="cuda")
        for min_count, dtype in ((1, rfx.U32), (2, rfx.U16)):
            rr, rc, rv = oracle.sparse_upper(leaf, min_count)
            rfx.prox_sparse_plan(plan, ws, nnz, min_count=min_count, count_dtype=dtype)          # count only
            assert int(nnz.item()) == rr.size
            cap = rr.size + 5
            rows = torch.full((cap,), -1, dtype=torch.int32, device="cuda")
            cols = torch.full((cap,), -1, dtype=torch.int32, device="cuda")
            counts = torch.zeros(cap, dtype=torch.int16 if dtype == rfx.U16 else torch.int32, device="cuda")
            prox = torch.zeros(cap, dtype=torch.float32, device="cuda")
            rfx.prox_sparse_plan(plan, ws, nnz, rows, cols, counts, prox, min_count=min_count, count_dtype=dtype)
            y_after = plan.apply(V)                                  # queued right behind it on the same stream
            torch.cuda.synchronize()
            n = int(nnz.item())
            assert n == rr.size
            assert bool((rows[n:] == -1).all())                      # nothing beyond the list
            r, c, v, pq = _sorted_triplets(rows[:n], cols[:n], counts[:n], prox[:n])
            np.testing.assert_array_equal(r, rr)
            np.testing.assert_array_equal(c, rc)
            np.testing.assert_array_equal(v, rv)
            np.testing.assert_array_equal(pq, (rv.astype(np.float32) / np.float32(B)).astype(np.float32))
            assert torch.equal(y_after, y_before)
        # too small a list: the count is still complete and nothing is written past the capacity
        small = torch.full((3,), -1, dtype=torch.int32, device="cuda")
        guard = torch.full((3,), -1, dtype=torch.int32, device="cuda")
        rfx.prox_sparse_plan(plan, ws, nnz, small, guard.clone(), min_count=1)
        torch.cuda.synchronize()
        assert int(nnz.item()) == oracle.sparse_upper(leaf, 1)[0].size
        fresh = rfx.PvPlan(d, bound)
        assert torch.equal(plan.apply(V), fresh.apply(V))
        plan.close()
        fresh.close()
    # host-side checks
    lib = rfx.load()
    import ctypes
    plan = rfx.PvPlan(_dev(torch, cases[0][1]), cases[0][2])
    ws = rfx.new_workspace(rfx.prox_sparse_plan_workspace_bytes(plan))
    nnz = torch.zeros(1, dtype=torch.int64, device="cuda")
    wp, wb = rfx._ws_ptr(ws)
    assert lib.rfx_prox_sparse_plan(plan._h, 1, rfx.U32, 0, None, None, None, None, nnz.data_ptr(), wp, wb - 256, None) == rfx.ERR_CAPACITY
    assert lib.rfx_prox_sparse_plan(plan._h, 0, rfx.U32, 0, None, None, None, None, nnz.data_ptr(), wp, wb, None) == rfx.ERR_INVALID_ARG
    assert lib.rfx_prox_sparse_plan(plan._h, 1, rfx.U32, 4, None, None, None, None, nnz.data_ptr(), wp, wb, None) == rfx.ERR_NULL
    assert lib.rfx_prox_sparse_plan(None, 1, rfx.U32, 0, None, None, None, None, nnz.data_ptr(), wp, wb, None) == rfx.ERR_NULL
    plan.close()


def test_row_pass_rejects_what_it_cannot_hold(torch_cuda):
    import paper_2511_19493_amd as rfx
    import ctypes
    lib = rfx.load()
    fake = ctypes.c_void_p(0x1000)
    nnz = ctypes.c_int64(0)
    assert lib.rfx_prox_sparse_rows(fake, 100, 5000, 8, 1, rfx.U32, 0, None, None, None, None, ctypes.byref(nnz), None) == rfx.ERR_UNSUPPORTED
    assert lib.rfx_prox_sparse_rows(fake, 100, 50, 8, 0, rfx.U32, 0, None, None, None, None, ctypes.byref(nnz), None) == rfx.ERR_INVALID_ARG
    assert lib.rfx_prox_sparse_rows(fake, 100, 50, 8, 1, rfx.U32, 4, None, None, None, None, ctypes.byref(nnz), None) == rfx.ERR_NULL
    assert lib.rfx_prox_sparse_rows(None, 100, 50, 8, 1, rfx.U32, 0, None, None, None, None, ctypes.byref(nnz), None) == rfx.ERR_NULL


def test_row_pass_on_a_nearly_dense_matrix(torch_cuda):
    """Two leaves per tree: three quarters of all pairs are non-zero, so a 32,768-column chunk of the row pass keeps more
    pairs than its counter array has words and every thread writes its own run.  The list is too long for the oracle's
    triplet form (3e8 entries), so it is checked through what fixes it: the pair count and the sum of the counts from the
    leaf sizes (sum over trees and leaves of s (s - 1) / 2), i < j, every count in range, no pair twice (the tile pass,
    itself checked against the oracle on every other case, gives the same number of pairs), and sampled rows against
    the oracle's dense rows."""
    import oracle
    import paper_2511_19493_amd as rfx
    torch = torch_cuda
    N, B, bound = 33000, 3, 2
    rng = np.random.default_rng(99)
    leaf = rng.integers(0, bound, size=(B, N)).astype(np.uint32)
    d = _dev(torch, leaf)
    rows, cols, counts, _ = rfx.prox_sparse(d, bound, 1, method="rows")
    n = rows.numel()
    assert n == rfx.prox_sparse_count(d, bound, 1)                      # tile pass ("auto" picks it here: few visits saved)
    expect = sum(int((np.bincount(leaf[b]).astype(np.int64) * (np.bincount(leaf[b]).astype(np.int64) - 1) // 2).sum()) for b in range(B))
    assert int(counts.sum(dtype=torch.int64)) == expect
    assert bool((rows < cols).all()) and int(cols.max()) < N and int(counts.min()) >= 1 and int(counts.max()) <= B
    key = rows.long() * N + cols.long()
    assert int(torch.unique(key).numel()) == n
    for i in (0, 1, 12345, 32767, 32768, N - 2):
        ref = oracle.counts_rows(leaf, i, i + 1)[0]
        m = rows == i
        j = cols[m].cpu().numpy().astype(np.int64)
        v = counts[m].cpu().numpy().view(np.uint32)
        order = np.argsort(j)
        want = np.nonzero(ref[i + 1:] >= 1)[0] + i + 1
        np.testing.assert_array_equal(j[order], want)
        np.testing.assert_array_equal(v[order], ref[want])
