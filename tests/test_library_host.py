"""Host-side checks that need no GPU: the C-ABI library loads, exports every symbol that
include/dgn.h declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def d():
    import paper_1707_08265_amd as d
    return d


def declared_functions():
    text = open(os.path.join(ROOT, "include", "dgn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dgn_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(d):
    names = declared_functions()
    assert len(names) >= 12
    lib = ctypes.CDLL(d.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in dgn.h but not exported"
    assert sorted(d.EXPORTS) == names, "binding and header disagree on the entry points"
    for n in names:
        assert hasattr(d, n), f"binding lacks {n}"


def test_version_and_strerror(d):
    assert d.dgn_version() == 100
    seen = set()
    for code in range(0, -10, -1):
        s = d.dgn_strerror(code)
        assert s and s != "unknown error" and s not in seen
        seen.add(s)
    assert d.dgn_strerror(-10) == "unknown error" and d.dgn_strerror(-1234) == "unknown error"


def test_workspace_queries_validate_sizes(d):
    mk = lambda **kw: d.make_coo_desc(kw.get("P", 10), kw.get("T", 20), None, None, None, None,
                                      kw.get("G", 1), kw.get("oo"), kw.get("to"), kw.get("ein", 5), kw.get("eout", 5))
    assert d.dgn_graph_build_workspace(None)[0] == d.DGN_ERR_NULL_PTR
    assert d.dgn_graph_build_workspace(mk(P=-1))[0] == d.DGN_ERR_INVALID_ARG
    assert d.dgn_graph_build_workspace(mk(ein=-3))[0] == d.DGN_ERR_INVALID_ARG
    assert d.dgn_graph_build_workspace(mk(G=0))[0] == d.DGN_ERR_INVALID_ARG
    assert d.dgn_graph_build_workspace(mk(T=2**31 - 1))[0] == d.DGN_ERR_TOO_LARGE
    assert d.dgn_graph_build_workspace(mk(G=2))[0] == d.DGN_ERR_NULL_PTR            # offsets missing
    oo, to = np.array([0, 4, 10], np.int64), np.array([0, 9, 20], np.int64)
    rc, gb, sb = d.dgn_graph_build_workspace(mk(G=2, oo=oo, to=to))
    assert rc == 0 and gb > 0 and sb > 0
    bad = np.array([0, 11, 10], np.int64)
    assert d.dgn_graph_build_workspace(mk(G=2, oo=bad, to=to))[0] == d.DGN_ERR_INVALID_ARG
    assert d.dgn_graph_build_workspace(mk(G=2, oo=oo, to=np.array([0, 9, 21], np.int64)))[0] == d.DGN_ERR_INVALID_ARG
    # sizes grow with the graph and are 256-byte granular
    rc1, g1, s1 = d.dgn_graph_build_workspace(mk())
    rc2, g2, s2 = d.dgn_graph_build_workspace(mk(P=1000, T=2000, ein=3000, eout=1500))
    assert rc1 == rc2 == 0 and g2 > g1 and s2 > s1 and g1 % 256 == 0 and s2 % 256 == 0
    # the bench workload fits comfortably in one GPU's memory
    rc, gb, sb = d.dgn_graph_build_workspace(mk(P=50_000_000, T=100_000_000, ein=128_700_000, eout=100_000_000))
    assert rc == 0 and gb < 4 * 2**30 and sb < 4 * 2**30


def test_build_rejects_bad_arguments_before_any_device_work(d):
    desc = d.make_coo_desc(4, 8, None, None, None, None, nnz_in=0, nnz_out=0)
    rc, gb, sb = d.dgn_graph_build_workspace(desc)
    assert rc == 0
    assert d.dgn_graph_build(desc, None, gb, None, sb, stream=0)[0] == d.DGN_ERR_NULL_PTR
    assert d.dgn_graph_build(desc, 256, gb - 1, 512, sb, stream=0)[0] == d.DGN_ERR_WORKSPACE_TOO_SMALL
    assert d.dgn_graph_build(desc, 256, gb, 516, sb, stream=0)[0] == d.DGN_ERR_INVALID_ARG      # misaligned
    desc2 = d.make_coo_desc(4, 8, None, None, None, None, nnz_in=3, nnz_out=0)                  # edges but no arrays
    rc, gb2, sb2 = d.dgn_graph_build_workspace(desc2)
    assert d.dgn_graph_build(desc2, 256, gb2, 512, sb2, stream=0)[0] == d.DGN_ERR_NULL_PTR
    opts = d.dgn_options(defer_percent=101)
    assert d.dgn_graph_build(desc, 256, gb, 512, sb, options=opts, stream=0)[0] == d.DGN_ERR_INVALID_ARG


def test_prune_entry_points_reject_null_graph_and_bad_set_counts(d):
    assert d.dgn_prune_workspace(None, 4)[0] == d.DGN_ERR_NULL_PTR
    assert d.dgn_prune(None, 4, 0, None, None, None, None, None, None, None, None, None, None, 0,
                       stream=0) == d.DGN_ERR_NULL_PTR
    assert d.dgn_keep_compact(None, None, None, None, None, None, None, None, None, 0, stream=0) == d.DGN_ERR_NULL_PTR
    assert d.dgn_graph_get_csr(None)[0] == d.DGN_ERR_NULL_PTR
    assert d.dgn_graph_get_sizes(None)[0] == d.DGN_ERR_NULL_PTR
    d.dgn_graph_destroy(None)          # accepted


def test_product_package_does_not_import_the_oracle():
    import subprocess
    import sys
    code = ("import sys; import paper_1707_08265_amd; "
            "assert 'oracle' not in sys.modules and 'graphgen' not in sys.modules")
    subprocess.check_call([sys.executable, "-c", code], cwd=ROOT)
    src = open(os.path.join(ROOT, "paper_1707_08265_amd", "binding.py")).read()
    assert "import oracle" not in src and "from oracle" not in src


def test_a_missing_library_is_an_import_error_not_a_fallback(monkeypatch, tmp_path):
    """Without libdgn.so the package must refuse to load: there is no CPU path behind it."""
    import paper_1707_08265_amd.binding as b
    monkeypatch.setattr(b, "LIB_PATH", str(tmp_path / "libdgn.so"))
    with pytest.raises(ImportError, match="no fallback"):
        b._load()


def test_other_entry_points_reject_bad_arguments_before_any_device_work(d):
    """Backward prune, in-place pass and read-outs: NULL handles and impossible sizes are refused on the host."""
    rc, _ = d.dgn_backward_prune_workspace(None)
    assert rc == d.DGN_ERR_NULL_PTR
    assert d.dgn_backward_prune(None, 4, None, None, None, None, None, None, None, None, None, None, 0, stream=0) == d.DGN_ERR_NULL_PTR
    rc, _ = d.dgn_inplace_workspace(None)
    assert rc == d.DGN_ERR_NULL_PTR
    rc, _ = d.dgn_inplace(None, None, 1, None, None, None, 0, stream=0)
    assert rc == d.DGN_ERR_NULL_PTR
    assert d.dgn_ignore_mask(None, None, None, None, None, None, None, stream=0) == d.DGN_ERR_NULL_PTR
    rc, _ = d.dgn_per_set_lists_workspace(-1)
    assert rc == d.DGN_ERR_INVALID_ARG
    rc, _ = d.dgn_per_set_lists_workspace(2**31)
    assert rc == d.DGN_ERR_TOO_LARGE
    rc, nbytes = d.dgn_per_set_lists_workspace(0)
    assert rc == 0 and nbytes > 0
    assert d.dgn_per_set_lists(None, None, -1, None, None, 0, None, 0, stream=0) == d.DGN_ERR_INVALID_ARG
    assert d.dgn_per_set_lists(None, None, 0, None, None, 0, None, 0, stream=0) == d.DGN_ERR_NULL_PTR
    assert d.dgn_prune_words(None, 100, 0, None, None, None, None, None, None, None, None, None, None, 0, stream=0) == d.DGN_ERR_NULL_PTR
    assert d.dgn_options(incremental=1).incremental == 1
    rc, _ = d.dgn_inplace_kept(None, None, 1, None, None, None, None, None, 0, stream=0)
    assert rc == d.DGN_ERR_NULL_PTR
    rc, nbytes = d.dgn_target_digest_workspace()
    assert rc == 0 and nbytes >= 16
    rc, _ = d.dgn_target_digest(None, 4, 0, None, None, None, 0, stream=0)
    assert rc == d.DGN_ERR_NULL_PTR
    o = d.dgn_options(recycle=1, profile=2)
    assert (o.recycle, o.profile) == (1, 2) and d.dgn_stats().recycled == 0
