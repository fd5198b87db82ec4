"""The entry point that allocates nothing: rfx_prox_dense_noalloc against rfx_prox_dense.

Two calls in a row through the C ABI, the second on a smaller input (fewer samples, fewer trees, a smaller
leaf bound, so stale contents of the built-in scratch from the first call lie beyond and between what the
second one writes); both must equal what rfx_prox_dense returns bit for bit (integer counts; the float32
proximities are the same IEEE quotients).  Then the size limit."""
import ctypes

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def test_noalloc_equals_prox_dense_on_two_calls_in_a_row(small2, cfg1):
    import torch
    import paper_2511_19493_amd as rfx
    assert torch.cuda.is_available(), "this test needs the MI355X"
    lib = rfx.load()
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream().cuda_stream
    first = True
    for d, cdt, layout in ((small2, rfx.U32, rfx.FULL), (cfg1, rfx.U16, rfx.UPPER_PACKED), (cfg1, rfx.U32, rfx.FULL)):
        leaf_h = d["leaf"]
        B, N = leaf_h.shape
        Lb = int(d["F"].n_leaves.max())
        print(f"no-alloc dense N={N} B={B} leaf_bound={Lb} dtype={cdt} layout={layout}", flush=True)
        leaf = torch.from_numpy(leaf_h.view(np.int32)).to(dev)
        n_out = N * N if layout == rfx.FULL else N * (N - 1) // 2
        tdt = torch.int16 if cdt == rfx.U16 else torch.int32
        want_c = torch.empty(n_out, dtype=tdt, device=dev)
        want_p = torch.empty(n_out, dtype=torch.float32, device=dev)
        got_c = torch.full((n_out,), -1, dtype=tdt, device=dev)
        got_p = torch.full((n_out,), -1.0, dtype=torch.float32, device=dev)
        assert lib.rfx_prox_dense(leaf.data_ptr(), N, B, Lb, cdt, layout, want_c.data_ptr(), want_p.data_ptr(), stream) == 0
        torch.cuda.synchronize()
        rc = lib.rfx_prox_dense_noalloc(leaf.data_ptr(), N, B, Lb, cdt, layout, got_c.data_ptr(), got_p.data_ptr(), stream)
        assert rc == 0, lib.rfx_last_error()
        torch.cuda.synchronize()
        assert torch.equal(got_c, want_c), f"counts differ (first call: {first})"
        assert torch.equal(got_p, want_p), f"proximities differ (first call: {first})"
        first = False


def test_noalloc_rejects_what_its_scratch_cannot_hold():
    import paper_2511_19493_amd as rfx
    lib = rfx.load()
    fake = ctypes.c_void_p(0x1000)
    # 32 tree groups x 102,400 padded samples x 16 words x 4 bytes = 210 MB of bit planes
    assert lib.rfx_prox_dense_noalloc(fake, 100_000, 1000, 4021, rfx.U32, rfx.FULL, fake, None, None) == rfx.ERR_CAPACITY
    assert b"16777216" in lib.rfx_last_error()
    assert lib.rfx_prox_dense_noalloc(None, 100, 10, 8, rfx.U32, rfx.FULL, fake, None, None) == rfx.ERR_NULL
    assert lib.rfx_prox_dense_noalloc(fake, 100, 10, 8, rfx.U32, rfx.FULL, None, None, None) == rfx.ERR_NULL
