"""The C-ABI library loads and exports every symbol include/rfx.h declares (no GPU needed)."""
import ctypes
import re
from pathlib import Path

import pytest

import paper_2511_19493_amd as rfx

ROOT = Path(__file__).resolve().parents[1]


def _declared():
    text = (ROOT / "include" / "rfx.h").read_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rfx_[a-z0-9_]+)\s*\(", text)))


def test_header_and_binding_agree():
    assert _declared() == sorted(rfx.EXPORTS)


def test_library_exports_every_declared_symbol():
    if not rfx.lib_path().exists():
        pytest.fail("librfx.so is not built: run `python -m paper_2511_19493_amd.build`")
    lib = ctypes.CDLL(str(rfx.lib_path()))
    for name in _declared():
        assert hasattr(lib, name), name
    rfx.load()


def test_host_side_argument_checks():
    """Validation happens before any device work, so these run without a GPU."""
    lib = rfx.load()
    assert lib.rfx_prox_dense(None, 10, 4, 8, rfx.U32, rfx.FULL, None, None, None) == -2
    assert b"leaf is null" in lib.rfx_last_error()
    fake = ctypes.c_void_p(0x1000)
    assert lib.rfx_prox_dense(fake, 10, 70000, 8, rfx.U16, rfx.FULL, fake, None, None) == -3   # overflow of u16
    assert lib.rfx_prox_dense(fake, 10, 4, 8, 7, rfx.FULL, fake, None, None) == -1
    assert lib.rfx_prox_dense(fake, 10, 4, 8, rfx.U32, rfx.FULL, None, None, None) == -2
    assert lib.rfx_prox_oob(fake, None, 10, 4, 8, rfx.U32, rfx.FULL, fake, fake, None, None) == -2
    assert lib.rfx_pv_apply(None, fake, 4, fake, None) == -2
    nnz = ctypes.c_int64(0)
    assert lib.rfx_prox_sparse(fake, 10, 4, 8, 0, rfx.U32, 0, None, None, None, None, ctypes.byref(nnz), None) == rfx.ERR_INVALID_ARG
    assert lib.rfx_prox_sparse(fake, 10, 4, 8, 1, rfx.U32, 5, None, None, None, None, ctypes.byref(nnz), None) == rfx.ERR_NULL
    assert lib.rfx_prox_sparse(fake, 10, 4, 8, 1, rfx.U32, 0, None, None, None, None, None, None) == rfx.ERR_NULL
    assert lib.rfx_prox_sparse(fake, 10, 1 << 20, 8, 1, rfx.U32, 0, None, None, None, None, ctypes.byref(nnz), None) == rfx.ERR_UNSUPPORTED
    assert lib.rfx_prox_lowrank(fake, 10, 4, 8, 300, 5, fake, fake, fake, None, None, None) == -1
    assert lib.rfx_prox_lowrank(fake, 10, 4, 8, 4, 0, fake, fake, fake, None, None, None) == -1
    assert lib.rfx_forest_create(None, None) == -2
    # fused pass, consumers, growth
    assert lib.rfx_prox_dense_oob(fake, fake, 10, 1024, 8, rfx.U32, rfx.FULL, fake, None, rfx.FULL, fake, None, None, None) == rfx.ERR_UNSUPPORTED
    assert lib.rfx_prox_dense_oob(fake, fake, 10, 4, 8, rfx.U32, rfx.FULL, fake, None, rfx.FULL, None, None, None, None) == rfx.ERR_NULL
    assert lib.rfx_prox_dense_oob(fake, fake, 10, 4, 8, rfx.U32, rfx.FULL, fake, None, 9, fake, None, None, None) == rfx.ERR_INVALID_ARG
    assert lib.rfx_prox_outlier(fake, 1, 4, 8, None, fake, None, None) == rfx.ERR_INVALID_ARG
    assert lib.rfx_prox_outlier(fake, 10, 4, 8, None, None, None, None) == rfx.ERR_NULL
    assert lib.rfx_oob_vote(fake, fake, fake, 10, 4, 8, 200, None, None, fake, None, None, None) == rfx.ERR_INVALID_ARG
    assert lib.rfx_oob_vote(fake, fake, fake, 10, 4, 8, 3, None, None, fake, ctypes.byref(nnz), None, None) == rfx.ERR_NULL
    h = ctypes.c_void_p()
    assert lib.rfx_forest_grow(fake, fake, 1 << 20, 4, 2, 0, 1, 2, 7, ctypes.byref(h), None) == rfx.ERR_INVALID_ARG
    assert lib.rfx_forest_grow(fake, fake, 100, 4, 2, 0, 1, 5, 7, ctypes.byref(h), None) == rfx.ERR_INVALID_ARG
    assert lib.rfx_forest_grow(fake, fake, 100, 4, 65, 0, 1, 2, 7, ctypes.byref(h), None) == rfx.ERR_INVALID_ARG
    assert lib.rfx_forest_grow(fake, None, 100, 4, 2, 0, 1, 2, 7, ctypes.byref(h), None) == rfx.ERR_NULL
    assert lib.rfx_grown_sizes(None, None, None, None, None) == rfx.ERR_NULL
    # asynchronous forms: workspace size queries and their argument checks run without a device
    nb = ctypes.c_int64(0)
    assert lib.rfx_prox_workspace_bytes(1000, 100, 300, ctypes.byref(nb)) == 0
    planes = 4 * 4 * 1024 * 12                                  # 4 tree groups x 1024 padded samples x 12 words
    assert nb.value == planes + 16128 + 256                     # + per-sample sums (16 N, padded) + counter
    assert lib.rfx_prox_workspace_bytes(0, 100, 300, ctypes.byref(nb)) == rfx.ERR_INVALID_ARG
    assert lib.rfx_prox_workspace_bytes(1000, 100, 300, None) == rfx.ERR_NULL
    assert lib.rfx_prox_dense_ws(fake, 10, 4, 8, rfx.U32, rfx.FULL, fake, None, None, 1 << 20, None) == rfx.ERR_NULL
    assert lib.rfx_prox_dense_ws(fake, 10, 4, 8, rfx.U32, rfx.FULL, fake, None, fake, 100, None) == rfx.ERR_CAPACITY
    assert lib.rfx_prox_dense_ws(fake, 10, 4, 8, rfx.U32, rfx.FULL, fake, None, ctypes.c_void_p(0x1010), 1 << 20, None) == rfx.ERR_INVALID_ARG
    assert lib.rfx_prox_sparse_ws(fake, 10, 4, 8, 1, rfx.U32, 0, None, None, None, None, ctypes.c_void_p(0x1004), fake, 1 << 20, None) == rfx.ERR_INVALID_ARG
    assert lib.rfx_prox_outlier_ws(fake, 10, 4, 8, None, fake, None, fake, 16, None) == rfx.ERR_CAPACITY
    assert lib.rfx_lowrank_workspace_bytes(1000, 16, ctypes.byref(nb)) == 0 and nb.value > 2 * 1000 * 16 * 4
    assert lib.rfx_lowrank_workspace_bytes(10, 16, ctypes.byref(nb)) == rfx.ERR_INVALID_ARG
    assert lib.rfx_prox_lowrank_plan(None, 4, 5, fake, fake, fake, None, None, None, fake, 1 << 20, None) == rfx.ERR_NULL
    assert lib.rfx_pv_plan_reserve(None, 4) == rfx.ERR_NULL and lib.rfx_pv_plan_info(None, None, None, None) == rfx.ERR_NULL
    assert lib.rfx_mds3d_workspace_bytes(1000, 16, 12, rfx.MDS_SQUARED, ctypes.byref(nb)) == 0 and nb.value > 3 * 1000 * 12 * 4
    sq = nb.value
    assert lib.rfx_mds3d_workspace_bytes(1000, 16, 12, rfx.MDS_LINEAR, ctypes.byref(nb)) == 0 and nb.value < sq
    assert lib.rfx_mds3d_workspace_bytes(1000, 16, 2, rfx.MDS_SQUARED, ctypes.byref(nb)) == rfx.ERR_INVALID_ARG
    assert lib.rfx_mds3d_ws(fake, fake, 1000, 16, rfx.MDS_SQUARED, 12, 10, fake, fake, fake, None, fake, 64, None) == rfx.ERR_CAPACITY
    assert lib.rfx_mds3d_ws(fake, fake, 1000, 16, rfx.MDS_SQUARED, 12, 0, fake, fake, fake, None, fake, 1 << 30, None) == rfx.ERR_INVALID_ARG
    assert lib.rfx_mds3d(fake, fake, 1000, 16, rfx.MDS_SQUARED, 12, 10, -1.0, fake, fake, fake, None, None) == rfx.ERR_INVALID_ARG
    out = ctypes.c_double(0)
    assert lib.rfx_probe_valu(0, ctypes.byref(out), None) == rfx.ERR_INVALID_ARG
    assert lib.rfx_probe_copy(5, ctypes.byref(out), None) == rfx.ERR_INVALID_ARG


def test_growth_draw_follows_the_published_generator():
    """The library's counter-based draw (host side of the function the kernels call) against splitmix64's
    published first outputs and a restatement of the composition; the oracle is not involved."""
    mask, K = (1 << 64) - 1, 0x9E3779B97F4A7C15

    def mix(z):
        z = (z + K) & mask
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & mask
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & mask
        return z ^ (z >> 31)

    assert mix(0) == 0xE220A8397B1DCDAF and mix(K) == 0x6E789E6AA1B965F4
    for seed, tree, a, b in ((0, 0, 0, 0), (12345, 7, 0, 99), (2 ** 63 + 5, 999, 1 + 4021, 9), (1, 2, 3, 4)):
        want = mix(mix(mix(seed ^ (((tree + 1) * K) & mask)) ^ a) ^ b)
        assert rfx.growth_draw(seed, tree, a, b) == want
