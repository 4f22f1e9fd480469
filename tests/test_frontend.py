"""Front end (graph description -> generated dispatch -> library), host side: what is generated, that it builds
for gfx950 and that the built library carries the functions.  CPU only (hipcc cross-compiles)."""
import ctypes
import os
import shutil

import pytest

from paper_2604_13327_amd import binding, frontend


def test_generated_header_has_one_case_per_device_function():
    g = frontend.sumsq_example()
    src = frontend.emit_dispatch_header(g)
    assert "constexpr int kUserFnCount = 3;" in src
    for k, name in enumerate(("square_tile", "partial_sum", "final_sum")):
        assert f"__device__ __forceinline__ void fn{k}_{name}(const Args &a, int c0, int c1, int c2)" in src
        assert f"case {k}: etc_user::fn{k}_{name}(a, c0, c1, c2); break;" in src
    assert src.count("case ") == 3 and "default:" in src
    assert frontend.emit_dispatch_header(frontend.sumsq_example()) == src            # deterministic
    assert g.fingerprint() != frontend.rowsum_example().fingerprint()


def test_graph_description_is_checked():
    g = frontend.Graph("g", ["n"])
    E = g.event("E", [g.sym("n")])
    f = g.device_fn("f", "", {0: lambda s: 4})
    with pytest.raises(ValueError):
        g.device_fn("f", "", {})                                     # defined twice
    with pytest.raises(ValueError):
        g.device_fn("h", "", {8: lambda s: 4})                       # slot out of range
    with pytest.raises(ValueError):
        g.call(f, [g.sym("n")], notifies=[frontend.Edge(E, [("dim", 1, 1)])])      # src is no grid dimension
    with pytest.raises(ValueError):
        g.call(f, [g.sym("n")], notifies=[frontend.Edge(E, [("dim", 0, 1), ("dim", 0, 1)])])   # rank mismatch
    with pytest.raises(ValueError):
        g.call(3, [4])
    assert frontend.Dim(0, 2, 1).eval([5]) == 11 and (g.sym("n") * 4 + 3).eval([2]) == 11


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not available")
def test_generated_library_builds_and_exports_the_c_abi(tmp_path):
    g = frontend.rowsum_example()
    lib = frontend.build_library(g, out_dir=str(tmp_path))
    assert os.path.exists(lib) and os.path.exists(tmp_path / "rowsum_dispatch.h")
    L = ctypes.CDLL(lib)
    for name in binding.EXPORTS:
        assert hasattr(L, name), name
    n = ctypes.c_int32(-1)
    assert L.etc_graph_user_fn_count(ctypes.byref(n)) == 0 and n.value == 2
    stock = binding.lib()
    assert stock.etc_graph_user_fn_count(ctypes.byref(n)) == 0 and n.value == 0       # the stock library has none
