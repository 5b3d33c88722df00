"""The C-ABI library loads without a GPU and exports every function lpq.h declares;
argument checks that precede any device work return the documented codes."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    from paper_2110_08919_amd import build, lpq
    if not os.path.exists(lpq.LIB_PATH):
        build.build()
    return lpq.lib()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "lpq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lpq_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(L):
    names = _declared_functions()
    assert len(names) >= 20
    for n in names:
        assert hasattr(L, n), n


def test_binding_covers_every_declared_symbol(L):
    from paper_2110_08919_amd import lpq
    for n in _declared_functions():
        assert getattr(L, n).argtypes is not None, f"{n} has no signature in the binding"


def test_argument_checks_without_device(L):
    from paper_2110_08919_amd import lpq
    h = C.c_void_p()
    assert L.lpq_quantizer_create(None, 8, 8) == lpq.EINVAL
    assert L.lpq_quantizer_create(C.byref(h), 0, 8) == lpq.EINVAL
    assert L.lpq_quantizer_create(C.byref(h), 8, 0) == lpq.EINVAL
    assert L.lpq_quantizer_create(C.byref(h), 8, 9) == lpq.EINVAL
    assert b"bits" in L.lpq_last_error()
    assert L.lpq_quantizer_create(C.byref(h), 1 << 20, 8) == lpq.ERANGE
    assert h.value is None                                    # never written on failure
    assert L.lpq_index_size(None) == -1
    assert L.lpq_index_create(None, None, 10) == lpq.EINVAL
    assert L.lpq_search_workspace_bytes(None, 10, 10, 0) == 0
    assert L.lpq_search(None, None, 1, 1, 1, 0, None, None, None, 0, None) == lpq.EINVAL
    assert L.lpq_search_f32(None, 10, 4, None, 1, 4, 4, 11, 0, None, None, None, 0, None) == lpq.ERANGE
    assert L.lpq_search_f32(None, 10, 4, None, 1, 4, 4, 5, 7, None, None, None, 0, None) == lpq.EINVAL
    assert L.lpq_search_f32(None, 10, 4, None, 0, 4, 4, 5, 0, None, None, None, 0, None) == lpq.OK  # nq = 0
    assert L.lpq_search_f32_workspace_bytes(0, 1, 4, 1) == 0
    assert L.lpq_set_tuning(99, 0) == lpq.EINVAL
    assert L.lpq_set_tuning(lpq.TUNE_SPLITS, 0) == lpq.OK
    assert L.lpq_profile_read(None, None) == lpq.EINVAL
    assert L.lpq_index_create_packed(None, None, 10) == lpq.EINVAL
    assert L.lpq_gather_dist_i8(None, None, 1, 4, None, 3, 0, None, None) == lpq.EINVAL
    assert L.lpq_search_overflow_stats(None, 1, 1, 0, None, None, None) == lpq.EINVAL
    assert L.lpq_search_overflow_left(None, 1, 1, 0, None, None) == lpq.EINVAL
    one = C.c_int(1)
    p1 = C.addressof(one)                                     # any non-null address: checks come before any use
    assert L.lpq_rerank_f32(p1, 10, 4, p1, 1, 4, 4, p1, 5000, 5, 0, p1, p1, None) == lpq.ERANGE   # kc > 4096
    assert L.lpq_rerank_f32(p1, 10, 4, p1, 1, 4, 4, p1, 8, 0, 0, p1, p1, None) == lpq.EINVAL      # k < 1
    assert L.lpq_rerank_f32(None, 10, 4, p1, 1, 4, 4, p1, 8, 5, 0, p1, p1, None) == lpq.EINVAL    # null corpus
    # workspace of the fp32 search: host arithmetic only, grows with the batch
    small, large = L.lpq_search_f32_workspace_bytes(1_000_000, 10, 128, 10), L.lpq_search_f32_workspace_bytes(1_000_000, 1000, 128, 10)
    assert 0 < small <= large
    # fp32 search: d beyond what a workgroup's LDS holds is refused, and the workspace query says so too
    assert L.lpq_search_f32(p1, 100, 20000, p1, 1, 20000, 20000, 5, 0, p1, p1, p1, 1 << 20, None) == lpq.ERANGE
    assert b"at most" in L.lpq_last_error()
    assert L.lpq_search_f32_workspace_bytes(100, 1, 20000, 5) == 0
    assert L.lpq_search_f32_workspace_bytes(100, 1, 15328, 5) > 0
    assert L.lpq_search_f32_workspace_bytes(2000, 1, 12260, 1024) == 0
    # the plan of a search, on the host: the benchmark shape takes the collecting scan with 128 queries per wave
    info = lpq.search_plan_info(128, 8, False, 1_000_000, 10_000, 10)
    assert info[0] == 3 and info[3] == 128 and info[5] > 0 and info[16] > 0
    assert lpq.search_plan_info(128, 8, False, 1_000_000, 16, 10)[1] == 1          # few queries: row-split workgroups
    out64 = (C.c_int64 * 35)()
    assert L.lpq_search_plan_info(128, 8, 0, 1000, 10, 10, out64, 10) == lpq.EINVAL
    # probes: argument checks precede any device work
    out = C.c_double(-1.0)
    assert L.lpq_probe_mfma_i8(None, 0, 100, None, None) == lpq.EINVAL
    assert L.lpq_probe_mfma_i8(None, 0, 0, C.byref(out), None) == lpq.EINVAL
    assert L.lpq_probe_mfma_i8(p1, 8, 100, C.byref(out), None) == lpq.EINVAL       # fewer than 16 operand bytes
    assert L.lpq_probe_stream(None, 1 << 20, 0, 1, C.byref(out), None) == lpq.EINVAL
    assert L.lpq_probe_stream(p1, 1 << 20, 2, 1, C.byref(out), None) == lpq.EINVAL  # unknown mode
    assert L.lpq_probe_stream(p1, 100, 0, 1, C.byref(out), None) == lpq.EINVAL      # less than one 4 KB chunk
    assert out.value == -1.0
    # the timing ablations are not compiled into the shipped library
    assert L.lpq_set_tuning(lpq.TUNE_DRY_RUN, 1) == lpq.EINVAL
    assert L.lpq_set_tuning(lpq.TUNE_DRY_RUN, 0) == lpq.OK
    L.lpq_quantizer_destroy(None)
    L.lpq_index_destroy(None)


def test_product_path_does_not_import_the_oracle():
    """The package (binding, generators, build) never touches oracle/."""
    pkg = os.path.join(ROOT, "paper_2110_08919_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", src, flags=re.M), f
                assert "lpq_oracle" not in src and "lpqo_" not in src, f
