"""The C-ABI library loads and exports every symbol the header declares (no GPU needed)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "tsdg_ann.h")
PROBE_HEADER = os.path.join(ROOT, "include", "tsdg_probe.h")


def declared_functions(header=HEADER):
    text = open(header).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ann_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    import paper_2204_00824_amd as P
    return P.load_library()


def test_header_declares_the_boundary():
    names = declared_functions()
    for must in ("ann_build_graph", "ann_search", "ann_search_ex", "ann_build_graph_ex", "ann_graph_export",
                 "ann_graph_import", "ann_graph_free", "ann_last_error", "ann_knn", "ann_bruteforce"):
        assert must in names


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert len(names) >= 20 and "ann_search_multi_static" in names and "ann_knn_ex" in names
    for name in names:
        assert hasattr(lib, name), f"{name} declared in tsdg_ann.h but not exported"


def test_probes_are_declared_apart_from_the_boundary(lib):
    """The two measurement probes live in the library but are no part of the method's header."""
    probes = declared_functions(PROBE_HEADER)
    assert probes == ["ann_probe_gather", "ann_probe_mfma"]
    assert not [n for n in declared_functions() if "probe" in n]
    for name in probes:
        assert hasattr(lib, name)


def test_the_library_reads_no_environment_variables():
    pkg = os.path.join(ROOT, "paper_2204_00824_amd", "csrc")
    for f in os.listdir(pkg):
        assert "getenv" not in open(os.path.join(pkg, f)).read(), f


def test_defaults_and_host_side_validation(lib):
    import paper_2204_00824_amd.api as api
    bp = api._BuildParams()
    lib.ann_build_params_default(C.byref(bp))
    assert (bp.dtype, bp.lambda0, bp.rev_cap, bp.metric) == (0, 9, 0, 0) and abs(bp.alpha - 1.2) < 1e-6
    assert (bp.knn_filter, bp.knn_row_block, bp.progress_user) == (0, 0, None) and not bp.progress and not bp.stats
    assert lib.ann_search_multi_workspace_bytes(16, 128) == 16 * 128 * 33 * 8
    assert lib.ann_search_multi_workspace_bytes(0, 5) == 0
    sp = api._SearchParams()
    lib.ann_search_params_default(C.byref(sp))
    assert (sp.mode, sp.lambda_visit, sp.n_seeds, sp.seed, sp.max_hops, sp.metric) == (0, 0, 32, 0, 0, 0)
    # argument errors are caught before any device work
    assert lib.ann_graph_info(None, None, None, None) == 1
    assert b"null graph" in lib.ann_last_error()
    assert lib.ann_search(None, None, None, 1, 1, 1, None, None) == 1
    out = C.c_void_p()
    assert lib.ann_build_graph(None, 100, 16, 8, C.byref(out)) == 1
    assert lib.ann_graph_import(None, None, 100, 8, 16, None, C.byref(out)) == 1
    lib.ann_graph_free(None)


def test_no_oracle_in_the_product_path():
    """The package never imports, links or runs anything under oracle/."""
    pkg = os.path.join(ROOT, "paper_2204_00824_amd")
    for root, _, files in os.walk(pkg):
        if "_build" in root:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(root, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "liboracle" not in text, f
