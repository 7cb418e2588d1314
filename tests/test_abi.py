"""The C-ABI library loads, exports every symbol its header declares, and rejects
bad arguments on the host before anything is launched.  CPU only: no compute call
is made (every call below fails its argument check first)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_1901_01544_amd import iwp
    if not os.path.exists(iwp.LIB_PATH):
        from paper_1901_01544_amd.build import build
        build()
    return iwp.load()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "iwp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"^\s*(?:const\s+)?[A-Za-z_][A-Za-z0-9_]*\s*\*?\s*([a-z][A-Za-z0-9_]*)\s*\(", text, flags=re.M)
    return sorted(set(names))


def test_header_declares_the_five_named_calls():
    names = declared_functions()
    for must in ("compress_layer", "select_threshold", "compact_pairs", "gather_sum_at_indices",
                 "apply_sparse_update", "compress_segmented", "iwp_step_segmented", "iwp_plan_create",
                 "iwp_workspace_bytes"):
        assert must in names, (must, names)


def test_every_declared_symbol_is_exported(lib):
    for name in declared_functions():
        assert hasattr(lib, name), "libiwp.so does not export %s" % name


def test_bad_arguments_are_rejected_on_the_host(lib):
    from paper_1901_01544_amd import iwp
    fake = 0x10000                                    # never dereferenced: the checks come first
    ws_bytes = lib.iwp_workspace_bytes(1000, 1)
    assert ws_bytes > 0 and lib.iwp_workspace_bytes(10 ** 9, 10 ** 6) > lib.iwp_workspace_bytes(1000, 10)
    cl = lib.compress_layer
    assert cl(fake, fake, fake, 10, 11, 1e-8, fake, fake, fake, ws_bytes, None) == iwp.IWP_EINVAL      # k > n
    assert cl(fake, fake, fake, 10, 1, -1.0, fake, fake, fake, ws_bytes, None) == iwp.IWP_EINVAL       # eps < 0
    assert cl(fake, fake, fake, 10, 1, float("nan"), fake, fake, fake, ws_bytes, None) == iwp.IWP_EINVAL
    assert cl(fake, fake, None, 10, 1, 1e-8, fake, fake, fake, ws_bytes, None) == iwp.IWP_EINVAL       # r NULL
    assert cl(fake, None, fake, 10, 1, 1e-8, fake, fake, fake, ws_bytes, None) == iwp.IWP_EINVAL       # g NULL
    assert cl(fake, fake, fake, 10, 1, 1e-8, None, fake, fake, ws_bytes, None) == iwp.IWP_EINVAL       # idx NULL
    assert cl(fake + 2, fake, fake, 10, 1, 1e-8, fake, fake, fake, ws_bytes, None) == iwp.IWP_EALIGN
    assert cl(fake, fake, fake, 1000, 1, 1e-8, fake, fake, fake, ws_bytes - 1, None) == iwp.IWP_EWORKSPACE
    assert cl(fake, fake, fake, 1000, 1, 1e-8, fake, fake, None, 0, None) == iwp.IWP_EWORKSPACE
    assert cl(fake, fake, fake, 0, 0, 1e-8, None, None, None, 0, None) == iwp.IWP_OK                   # empty layer: no-op
    assert lib.select_threshold(fake, fake, 10, 0, 1e-8, fake, fake, ws_bytes, None) == iwp.IWP_EINVAL  # k = 0
    assert lib.compact_pairs(fake, fake, 10, 1e-8, None, 1, fake, fake, fake, ws_bytes, None) == iwp.IWP_EINVAL
    tab = (C.c_void_p * 1)(fake)
    assert lib.gather_sum_at_indices(tab, 0, fake, 5, fake, None) == iwp.IWP_EINVAL                    # W = 0
    assert lib.gather_sum_at_indices(tab, 33, fake, 5, fake, None) == iwp.IWP_EINVAL                   # W too large
    assert lib.gather_sum_at_indices(tab, 1, fake, 0, fake, None) == iwp.IWP_OK                        # k = 0: no-op
    assert lib.apply_sparse_update(None, fake, fake, 5, 1.0, tab, 1, None) == iwp.IWP_EINVAL
    assert lib.apply_sparse_update(fake, fake, fake, 0, 1.0, tab, 1, None) == iwp.IWP_OK
    h = C.c_void_p()
    rows = (iwp.Layer * 2)()
    rows[0].offset, rows[0].n, rows[0].k, rows[0].out_offset = 0, 10, 11, 0
    assert lib.iwp_plan_create(rows, 1, C.byref(h)) == iwp.IWP_EINVAL and not h.value                  # k > n
    rows[0].k = 1
    rows[1].offset, rows[1].n, rows[1].k, rows[1].out_offset = 5, 10, 1, 1
    assert lib.iwp_plan_create(rows, 2, C.byref(h)) == iwp.IWP_EINVAL                                   # overlap
    rows[1].offset, rows[1].out_offset = 10, 7
    assert lib.iwp_plan_create(rows, 2, C.byref(h)) == iwp.IWP_EINVAL                                   # not packed
    rows[0].offset, rows[0].n = 0xFFFF0000 - 5, 10
    assert lib.iwp_plan_create(rows, 1, C.byref(h)) == iwp.IWP_ERANGE
    assert lib.iwp_plan_create(None, 1, C.byref(h)) == iwp.IWP_EINVAL
    # plan-taking entry points without a plan: nothing to launch on
    assert lib.iwp_plan_set_momentum(None, 0.9) == iwp.IWP_EINVAL
    assert lib.iwp_plan_mask_bytes(None) == 0 and lib.iwp_plan_threshold_workspace_bytes(None, 2, 1, 16) == 0
    assert lib.iwp_plan_workspace_bytes(None) == 0 and lib.iwp_plan_total_pairs(None) == 0
    tabs = (C.c_void_p * 2)(fake, fake)
    assert lib.iwp_step_threshold_segmented(None, fake, tabs, tabs, 2, fake, 1, fake, 1e-8, 1.0, fake, fake, fake,
                                            fake, 16, fake, 1 << 20, None) == iwp.IWP_EINVAL
    assert lib.iwp_step_threshold_random_segmented(None, fake, tabs, tabs, 2, fake, 1, fake, 1, 2, 1e-8, 1.0, fake,
                                                   fake, fake, fake, 16, fake, 1 << 20, None) == iwp.IWP_EINVAL
    assert lib.iwp_step_layerwise_segmented(None, fake, tabs, tabs, 2, fake, 1, 0.1, 0.1, 1.0, 1e-8, 1.0, fake, fake,
                                            fake, fake, fake, fake, 16, fake, 1 << 20, None) == iwp.IWP_EINVAL
    assert lib.iwp_step_segmented(None, fake, tabs, tabs, 2, fake, None, 1e-8, 1.0, fake, fake, fake, fake, fake,
                                  1 << 20, None) == iwp.IWP_EINVAL
    assert lib.compress_segmented(None, fake, tabs, tabs, 2, fake, None, 1e-8, fake, fake, fake, fake, 1 << 20,
                                  None) == iwp.IWP_EINVAL
    for code in (0, -1, -2, -3, -4, -5, -99):
        assert lib.iwp_strerror(code)


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    from paper_1901_01544_amd import iwp
    monkeypatch.setattr(iwp, "_lib", None)
    monkeypatch.setattr(iwp, "LIB_PATH", str(tmp_path / "libiwp.so"))
    with pytest.raises(FileNotFoundError):
        iwp.workspace_bytes(10, 1)
