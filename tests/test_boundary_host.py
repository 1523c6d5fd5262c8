"""Host-side checks of the C boundary that need no GPU: the library loads, exports every symbol
the header declares, and its pure host logic (bounds, workspace sizes, argument checks) behaves."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2503_01281_amd as dci
    if not os.path.exists(dci.library_path()):
        from paper_2503_01281_amd import build
        build.build()
    return dci.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "dci.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = sorted(set(re.findall(r"\b(dci_[a-z_0-9]+)\s*\(", header)))
    assert {"dci_presample_count", "dci_fill_caches", "dci_sample_khop", "dci_gather_features",
            "dci_sage_forward", "dci_create", "dci_destroy", "dci_sync", "dci_last_error"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in include/dci.h but not exported by libdci.so"


def test_blocks_bounds():
    import paper_2503_01281_amd as dci
    assert dci.blocks_bounds(232965, 1024, [5, 10, 15]) == ([1024, 6144, 67584, 233989], [5120, 61440, 1013760])
    assert dci.blocks_bounds(16384, 256, [5, 10]) == ([256, 1536, 16640], [1280, 15360])
    assert dci.blocks_bounds(10, 0, [3]) == ([0, 0], [0])
    for bad in ([], [0], [65], [5] * 9):
        with pytest.raises(dci.DciError):
            dci.blocks_bounds(1000, 10, bad)
    with pytest.raises(dci.DciError) as e:           # a bound at or above 2^31
        dci.blocks_bounds(2**31 - 1, 2**26, [64, 64])
    assert e.value.code == -4


def test_workspace_queries_grow_with_the_problem(lib):
    f3 = (C.c_int32 * 3)(5, 10, 15)
    small = lib.dci_sample_workspace_bytes(232965, 256, f3, 3)
    big = lib.dci_sample_workspace_bytes(232965, 1024, f3, 3)
    assert 0 < small < big
    assert lib.dci_sample_workspace_bytes(232965, 1024, (C.c_int32 * 1)(0), 1) == 0      # invalid fan-out
    assert 0 < lib.dci_fill_workspace_bytes(1000) < lib.dci_fill_workspace_bytes(10**6)
    assert lib.dci_fill_workspace_bytes(0) == 0
    rows = (C.c_int64 * 8)(1024, 6144, 67584, 0, 0, 0, 0, 0)
    dims = (C.c_int32 * 4)(602, 256, 256, 41)
    need = lib.dci_sage_workspace_bytes(rows, 3, dims)
    assert need >= 67584 * 602 * 4 + 2 * 67584 * 256 * 4


def test_static_scratch_size_query(lib):
    """The no-allocation sampler's size query (host arithmetic only): a Medium-sized batch fits the
    static array, a Large-sized one does not, invalid fan-outs give 0."""
    lib.dci_sample_khop_scratch_bytes.restype = C.c_size_t
    f3 = (C.c_int32 * 3)(5, 10, 15)
    limit = 32 << 20
    assert 0 < lib.dci_sample_khop_scratch_bytes(232965, 1024, f3, 3) <= limit
    assert lib.dci_sample_khop_scratch_bytes(2449029, 4096, f3, 3) > limit
    assert lib.dci_sample_khop_scratch_bytes(232965, 1024, (C.c_int32 * 1)(65), 1) == 0
    assert lib.dci_sample_khop_static(None, None, None, None, 0, 0, None, 0, 0, None, None) == -1


def test_null_context_and_missing_gpu_are_errors_not_crashes(lib):
    assert lib.dci_sync(None) == -1
    assert lib.dci_set_workspace(None, None, 0) == -1
    assert lib.dci_last_error(None) == b"null context"
    assert lib.dci_sample_khop(None, None, None, None, 0, 0, None, 0, 0, None, None) == -1
    assert lib.dci_gather_features(None, None, None, None, 0, None, None, None) == -1
    assert lib.dci_fill_caches(None, None, None, None, None, 0, 0, 0, 0, None, None, None, None, None) == -1
    assert lib.dci_create(None, 0, None, None, 0) == -1
    import torch
    if not torch.cuda.is_available():
        h = C.c_void_p()
        assert lib.dci_create(C.byref(h), 0, None, None, 0) == -3      # no device: a HIP error, reported
        assert not h.value


def test_the_binding_has_no_fallback():
    """The Python layer only marshals arguments: it must not import the oracle or implement the path."""
    for fn in ("binding.py", "__init__.py"):
        src = open(os.path.join(ROOT, "paper_2503_01281_amd", fn)).read()
        assert "oracle" not in src and "numpy" not in src
