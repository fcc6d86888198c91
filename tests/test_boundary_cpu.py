"""CPU-only checks of the C boundary: the library loads, exports every declared symbol, and the
host-side argument validation returns error codes before anything is launched."""
import ctypes
import os
import re

import pytest

from paper_2603_18636_amd import svoo

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "svoo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(svoo_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(svoo.LIB_PATH):
        from paper_2603_18636_amd import build
        build.build(verbose=False)
    return svoo._lib()


def test_exports_match_header(lib):
    names = declared_symbols()
    assert set(names) == set(svoo.EXPORTS)
    for name in names:
        assert getattr(lib, name) is not None


def test_status_strings_and_version(lib):
    assert svoo.status_string(0) == "ok"
    assert "workspace" in svoo.status_string(3)
    assert svoo.status_string(99) == "unknown status"
    assert svoo.version() >= 100


def test_workspace_bytes_and_shape_validation(lib):
    good = svoo.Shape(12, 75600, 128, svoo.SVOO_BF16, 256, 256)
    need = svoo.workspace_bytes(good)
    assert need > 0 and need % 256 == 0
    assert need < 2 ** 31  # well under a GB-scale budget for the headline workload
    # asymmetric cluster counts: the workspace also covers svoo_kmeans with k = the larger count
    assert svoo.workspace_bytes(svoo.Shape(2, 5000, 128, svoo.SVOO_BF16, 8, 1024)) > 0
    for bad in (svoo.Shape(0, 100, 128, 0, 4, 4), svoo.Shape(1, 0, 128, 0, 4, 4), svoo.Shape(1, 100, 96, 0, 4, 4),
                svoo.Shape(1, 100, 128, 7, 4, 4), svoo.Shape(1, 100, 128, 0, 0, 4), svoo.Shape(1, 100, 128, 0, 4, 2000),
                svoo.Shape(1, 100, 128, 0, 200, 4)):
        assert svoo.workspace_bytes(bad) == 0


def test_entry_points_reject_bad_arguments_on_host(lib):
    """Null pointers, bad sizes and misalignment come back as status codes; nothing is launched, so
    this runs without a GPU."""
    s = svoo.Shape(1, 1024, 64, svoo.SVOO_F32, 16, 16)
    sp = ctypes.byref(s)
    null = None
    fake = ctypes.c_void_p(0x1000)       # aligned, never dereferenced on these paths
    odd = ctypes.c_void_p(0x1008)        # 8-byte aligned only
    ws_bytes = svoo.workspace_bytes(s)
    INVALID, UNSUPPORTED, TOO_SMALL = 1, 2, 3
    assert lib.svoo_cocluster(sp, null, fake, fake, fake, null, null, 2, fake, fake, fake, fake, fake, fake, null,
                              fake, ws_bytes, null) == INVALID
    assert lib.svoo_cocluster(sp, fake, fake, null, fake, null, null, 2, fake, fake, fake, fake, fake, fake, null,
                              fake, ws_bytes, null) == INVALID       # neither init indices nor centroids for q
    assert lib.svoo_cocluster(sp, fake, fake, fake, fake, null, null, 0, fake, fake, fake, fake, fake, fake, null,
                              fake, ws_bytes, null) == INVALID       # iters < 1
    assert lib.svoo_cocluster(sp, fake, fake, fake, fake, null, null, 2, fake, fake, fake, fake, fake, fake, null,
                              fake, 16, null) == TOO_SMALL
    assert lib.svoo_cocluster(sp, odd, fake, fake, fake, null, null, 2, fake, fake, fake, fake, fake, fake, null,
                              fake, ws_bytes, null) == INVALID       # misaligned q
    assert lib.svoo_cocluster_sorted(sp, fake, fake, fake, fake, null, null, 2, fake, fake, fake, fake, fake, fake, null,
                                     fake, fake, fake, null, fake, ws_bytes, null) == INVALID   # a layout output missing
    assert lib.svoo_cocluster_sorted(sp, fake, fake, fake, fake, null, null, 2, fake, fake, fake, fake, fake, fake, null,
                                     fake, fake, fake, fake, fake, 16, null) == TOO_SMALL
    bad_d = svoo.Shape(1, 1024, 80, svoo.SVOO_F32, 16, 16)
    assert lib.svoo_attn(ctypes.byref(bad_d), fake, fake, fake, 0.125, fake, null, fake, 4096, null) == UNSUPPORTED
    assert lib.svoo_attn(sp, fake, fake, null, 0.125, fake, null, fake, 4096, null) == INVALID
    assert lib.svoo_attn(sp, fake, fake, fake, 0.125, fake, null, fake, 8, null) == TOO_SMALL
    assert lib.svoo_attn(sp, fake, fake, fake, float("nan"), fake, null, fake, 4096, null) == INVALID
    assert lib.svoo_block_mask(sp, fake, fake, fake, fake, fake, 1.5, 0.1, 0.125, fake, fake, null, null, 0,
                               null) == INVALID                      # tau outside (0, 1]
    assert lib.svoo_block_mask(sp, fake, fake, fake, fake, null, 0.9, 0.1, 0.125, fake, fake, null, null, 0,
                               null) == INVALID
    assert lib.svoo_block_mask(sp, fake, fake, fake, fake, fake, 0.9, 0.1, 0.125, fake, fake, null, null, 0,
                               null) == INVALID                      # the block estimate needs the workspace
    assert lib.svoo_block_mask(sp, fake, fake, fake, fake, fake, 0.9, 0.1, 0.125, fake, fake, null, fake, 64,
                               null) == TOO_SMALL
    assert lib.svoo_block_sparse_attn(sp, fake, fake, fake, fake, fake, fake, null, 0.125, fake, null, fake, 4096,
                                      null) == INVALID
    assert lib.svoo_block_sparse_attn(sp, fake, fake, fake, fake, fake, fake, fake, 0.125, fake, null, fake, 8,
                                      null) == TOO_SMALL
    assert lib.svoo_block_sparse_attn_tokens(sp, fake, null, fake, fake, fake, fake, fake, fake, 0.125, fake, null, fake,
                                             4096, null) == INVALID            # no permutation
    assert lib.svoo_block_sparse_attn_tokens(sp, fake, fake, fake, fake, fake, fake, fake, fake, 0.125, fake, null, fake,
                                             8, null) == TOO_SMALL
    static = lib.svoo_block_sparse_attn_static
    assert static(sp, fake, fake, fake, fake, fake, fake, null, 0.125, fake, null, null) == INVALID
    assert static(sp, fake, odd, fake, fake, fake, fake, fake, 0.125, fake, null, null) == INVALID
    big = svoo.Shape(300, 2048, 64, svoo.SVOO_BF16, 1024, 16)           # 300 * 1025 schedule entries > 262,144
    assert static(ctypes.byref(big), fake, fake, fake, fake, fake, fake, fake, 0.125, fake, null, null) == 5
    assert "allocation-free" in svoo.status_string(5)
    assert lib.svoo_row_recall(sp, fake, fake, null, fake, null) == INVALID
    assert svoo._lib().svoo_permute_workspace_bytes(sp, 0) == 0
    assert svoo._lib().svoo_permute_workspace_bytes(sp, 1024) == 2 * 1024 * 4          # 2 chunks of 512 tokens x 1024 bins
    arr = (ctypes.c_void_p * 1)(0x1000)
    arr2 = (ctypes.c_void_p * 1)(0x2000)
    assert lib.svoo_permute(sp, fake, 0, 1, arr, arr2, fake, fake, fake, ws_bytes, null) == INVALID      # 0 clusters
    assert lib.svoo_permute(sp, fake, 16, 5, arr, arr2, fake, fake, fake, ws_bytes, null) == INVALID     # > 4 tensors
    assert lib.svoo_permute(sp, fake, 16, 1, arr, arr, fake, fake, fake, ws_bytes, null) == INVALID      # dst aliases src
    assert lib.svoo_permute(sp, fake, 16, 1, arr, arr2, fake, fake, fake, 4, null) == TOO_SMALL
    assert lib.svoo_gather(sp, fake, 0, arr, arr2, null) == INVALID                                      # no tensors
    assert lib.svoo_gather(sp, null, 1, arr, arr2, null) == INVALID
    assert lib.svoo_unpermute(sp, fake, fake, fake, null) == INVALID                                     # in place
    assert lib.svoo_unpermute(sp, fake, null, ctypes.c_void_p(0x2000), null) == INVALID
    assert lib.svoo_assign(sp, fake, fake, 0, fake, 4, fake, fake, ws_bytes, null) == INVALID
    assert lib.svoo_assign(sp, fake, fake, 4, fake, 4, fake, fake, 8, null) == TOO_SMALL
    dens = lib.svoo_attention_density
    assert dens(sp, fake, fake, null, 100, 0.95, 0.125, fake, fake, null, null) == INVALID    # no row list, n_rows != n
    assert dens(sp, fake, fake, fake, 2000, 0.95, 0.125, fake, fake, null, null) == INVALID   # more rows than tokens
    assert dens(sp, fake, fake, fake, 10, 0.0, 0.125, fake, fake, null, null) == INVALID      # tau outside (0, 1]
    assert dens(sp, fake, fake, fake, 10, 1.5, 0.125, fake, fake, null, null) == INVALID
    assert dens(sp, fake, null, fake, 10, 0.95, 0.125, fake, fake, null, null) == INVALID
    assert dens(sp, fake, fake, fake, 10, 0.95, -1.0, fake, fake, null, null) == INVALID
    assert lib.svoo_kmeans(sp, fake, 16, null, null, 2, fake, fake, fake, null, fake, ws_bytes, null) == INVALID  # no start
    assert lib.svoo_kmeans(sp, fake, 0, fake, null, 2, fake, fake, fake, null, fake, ws_bytes, null) == INVALID
    assert lib.svoo_kmeans(sp, fake, 2000, fake, null, 2, fake, fake, fake, null, fake, ws_bytes, null) == INVALID
    assert lib.svoo_kmeans(sp, fake, 16, fake, null, 0, fake, fake, fake, null, fake, ws_bytes, null) == INVALID
    assert lib.svoo_kmeans(sp, fake, 16, fake, null, 2, fake, fake, fake, null, fake, 64, null) == TOO_SMALL
    assert lib.svoo_microbench_mfma_bf16(0, 10, 1, fake, null, null) == INVALID
    assert lib.svoo_microbench_mfma_bf16(8, 0, 1, fake, null, null) == INVALID
    assert lib.svoo_microbench_mfma_bf16(8, 10, 1, null, null, null) == INVALID
    assert lib.svoo_microbench_copy(fake, ctypes.c_void_p(0x2000), 24, null) == INVALID       # not a multiple of 16
    assert lib.svoo_microbench_copy(odd, ctypes.c_void_p(0x2000), 32, null) == INVALID
    assert lib.svoo_microbench_copy(fake, null, 32, null) == INVALID
    assert lib.svoo_microbench_attn_tile(5, 10, fake, fake, null) == INVALID                 # subset not instantiated
    assert lib.svoo_microbench_attn_tile(1, 0, fake, fake, null) == INVALID


def test_binding_refuses_missing_library(monkeypatch, tmp_path):
    monkeypatch.setattr(svoo, "_LIB", None)
    monkeypatch.setattr(svoo, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        svoo.version()
