"""The C-ABI library loads without a GPU, exports every symbol the header
declares, and rejects bad arguments on the host before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "lantern.h")


@pytest.fixture(scope="module")
def lib():
    import paper_2410_03355_amd as lantern
    if not os.path.exists(lantern.LIB_PATH):
        lantern.build()
    return lantern.load()


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lantern_[a-z_]+)\s*\(", text)))


def test_exports_match_header(lib):
    import paper_2410_03355_amd as lantern
    declared = _declared_functions()
    assert declared, "no functions found in the header"
    for name in declared:
        assert hasattr(lib, name), f"{name} declared in lantern.h but not exported"
    assert sorted(lantern.EXPORTS) == declared


def test_status_strings_and_version(lib):
    import paper_2410_03355_amd as lantern
    assert lib.lantern_version() >= 100
    seen = set()
    for code in (0, -1, -2, -3, -4, -5, -6, -7):
        s = lantern.status_string(code)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 8
    assert lantern.status_string(-99) == "unknown status"


def test_bench_records_are_of_this_library(lib):
    """bench.py reports HBM traffic and the table build's per-kernel split from profiler runs that it
    cannot repeat itself; each record names the library version it was measured at, and is only
    reported while lantern_version() still says so.  A kernel change must come with a new version and
    new measurements, or the bench line silently loses those fields: this keeps the two in step."""
    import importlib.util
    spec = importlib.util.spec_from_file_location("bench_for_test", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    version = lib.lantern_version()
    assert bench.MEASURED_TRAFFIC and bench.MEASURED_KNN_SPLIT
    for key, (nbytes, measured_at, source) in bench.MEASURED_TRAFFIC.items():
        assert measured_at == version, f"traffic of {key} was measured at version {measured_at}, the library is {version}"
        assert nbytes > 0 and os.path.exists(os.path.join(ROOT, source.split(" ")[0]))
    for key, (us, extra_flop, measured_at, source) in bench.MEASURED_KNN_SPLIT.items():
        assert measured_at == version, f"table-build split of {key} was measured at version {measured_at}"
        assert os.path.exists(os.path.join(ROOT, source.split(" ")[0]))
        assert f"version {version}" in open(os.path.join(ROOT, source.split(" ")[0])).read()


def test_verify_argument_errors(lib):
    import paper_2410_03355_amd as L
    p = ctypes.c_void_p(4096)  # never dereferenced: validation fails first
    nul = ctypes.c_void_p(0)

    def call(tl=p, dl=p, dt=L.F32, N=4, V=16, stride=16, tok=p, knn=p, k=4, delta=0.1, un=p,
             oa=p, orr=p):
        return lib.lantern_verify(tl, dl, dt, N, V, stride, tok, knn, k, delta, un, oa, orr, nul)

    assert call(dt=7) == L.binding.E_DTYPE
    for kw in (dict(N=-1), dict(V=0), dict(k=0), dict(k=17), dict(stride=15), dict(V=L.MAX_VOCAB + 1,
                                                                                  stride=L.MAX_VOCAB + 1)):
        assert call(**kw) == L.binding.E_SHAPE
    assert call(delta=-0.5) == L.binding.E_DELTA
    assert call(delta=float("nan")) == L.binding.E_DELTA
    for name in ("tl", "dl", "tok", "knn", "un", "oa", "orr"):
        assert call(**{name: nul}) == L.binding.E_NULL
    assert call(N=0, tl=nul, dl=nul) == L.binding.OK  # nothing to do


def test_build_knn_argument_errors(lib):
    import paper_2410_03355_amd as L
    p = ctypes.c_void_p(4096)
    nul = ctypes.c_void_p(0)
    assert lib.lantern_build_knn_workspace_bytes(L.F32, 0, 8, 1) == 0
    assert lib.lantern_build_knn_workspace_bytes(L.F32, 16, 8, 17) == 0
    assert lib.lantern_build_knn_workspace_bytes(5, 16, 8, 4) == 0
    need = lib.lantern_build_knn_workspace_bytes(L.F32, 1024, 8, 16)
    assert need > 1024 * 4
    assert lib.lantern_build_knn(p, 9, 16, 8, 4, p, p, 1 << 30, nul) == L.binding.E_DTYPE
    assert lib.lantern_build_knn(p, L.F32, 16, 8, 17, p, p, 1 << 30, nul) == L.binding.E_SHAPE
    assert lib.lantern_build_knn(p, L.F32, 16, 0, 4, p, p, 1 << 30, nul) == L.binding.E_SHAPE
    assert lib.lantern_build_knn(nul, L.F32, 16, 8, 4, p, p, 1 << 30, nul) == L.binding.E_NULL
    assert lib.lantern_build_knn(p, L.F32, 16, 8, 4, nul, p, 1 << 30, nul) == L.binding.E_NULL
    assert lib.lantern_build_knn(p, L.F32, 16, 8, 4, p, nul, 1 << 30, nul) == L.binding.E_WORKSPACE
    assert lib.lantern_build_knn(p, L.F32, 16, 8, 4, p, p, 16, nul) == L.binding.E_WORKSPACE
    assert lib.lantern_build_knn(p, L.F32, 16, 8, 4, p, ctypes.c_void_p(4096 + 8), 1 << 30, nul) == \
        L.binding.E_WORKSPACE
    assert lib.lantern_build_knn_metric(p, L.F32, 16, 8, 4, 5, p, p, 1 << 30, nul) == L.binding.E_SHAPE


def test_binding_refuses_host_tensors():
    import torch
    import paper_2410_03355_amd as L
    t = torch.zeros(2, 8)
    with pytest.raises(ValueError):
        L.verify(t, t, torch.zeros(2, dtype=torch.int32), torch.zeros(8, 1, dtype=torch.int32), 0.1,
                 torch.zeros(2, 2))
    with pytest.raises(ValueError):
        L.build_knn(torch.zeros(8, 2), 2)


def test_tree_and_split_argument_errors(lib):
    """Host-side validation of the tree, shared-row, split and random-table entry points."""
    import paper_2410_03355_amd as L
    B_ = L.binding
    p = ctypes.c_void_p(4096)  # never dereferenced: validation fails first
    nul = ctypes.c_void_p(0)

    def rows(ri=p, R=3, N=4, V=16, k=4, div=0, delta=0.1, oa=p, orr=p):
        return lib.lantern_verify_rows(p, p, L.F32, R, V, 16, ri, N, p, p, k, div, delta, p, oa, orr, nul)

    assert rows(ri=nul) == B_.E_NULL
    assert rows(R=0) == B_.E_SHAPE
    assert rows(div=2) == B_.E_SHAPE
    assert rows(delta=-1.0) == B_.E_DELTA
    assert rows(orr=nul) == B_.E_NULL
    assert rows(N=0, ri=nul) == B_.OK

    def decide(ri=p, R=4, N=4, oa=p):
        return lib.lantern_decide_rows(p, p, L.F32, R, 16, 16, ri, N, p, p, 4, 0, 0.1, p, oa, nul, nul)

    assert decide(ri=nul, R=3) == B_.E_SHAPE          # no index array: one row per verification
    assert decide(oa=nul) == B_.E_NULL
    assert decide(N=0, R=0, ri=nul) == B_.OK

    def selected(sel=p, n_sel=2, N=4, out=p):
        return lib.lantern_resample_selected(p, p, L.F32, N, 16, 16, nul, N, p, p, 4, 0, 0.1, p, sel, n_sel, out, nul)

    assert selected(sel=nul) == B_.E_NULL
    assert selected(out=nul) == B_.E_NULL
    assert selected(n_sel=-1) == B_.E_SHAPE
    assert selected(n_sel=2, N=0) == B_.E_SHAPE
    assert selected(n_sel=0) == B_.OK

    def trees(B=2, M=3, par=p, ri=p, on=p):
        return lib.lantern_verify_trees(p, p, L.F32, 8, 16, 16, ri, par, B, M, p, p, 4, 0, 0.1, p, p, p, p, on, nul)

    assert trees(M=0) == B_.E_SHAPE
    assert trees(B=-1) == B_.E_SHAPE
    assert trees(B=1 << 20, M=1 << 12) == B_.E_SHAPE   # B*M beyond int
    assert trees(par=nul) == B_.E_NULL
    assert trees(ri=nul) == B_.E_SHAPE               # no index array: one row per candidate (R = 8, B*M = 6)
    assert trees(on=nul) == B_.E_NULL
    assert trees(B=0) == B_.OK

    assert lib.lantern_accept_trees(p, p, p, 2, 0, p, p, p, nul) == B_.E_SHAPE
    assert lib.lantern_accept_trees(p, nul, nul, 2, 3, p, p, p, nul) == B_.E_NULL
    assert lib.lantern_accept_trees(nul, nul, nul, 0, 3, nul, nul, nul, nul) == B_.OK
    assert lib.lantern_accept_chains(p, p, 2, 0, p, p, nul) == B_.E_SHAPE

    assert lib.lantern_build_random(0, 1, 1, p, nul) == B_.E_SHAPE
    assert lib.lantern_build_random(8, 9, 1, p, nul) == B_.E_SHAPE
    assert lib.lantern_build_random(8192, L.binding.RANDOM_MAX_K + 1, 1, p, nul) == B_.E_SHAPE
    assert lib.lantern_build_random(L.MAX_VOCAB + 1, 2, 1, p, nul) == B_.E_SHAPE
    assert lib.lantern_build_random(8, 4, 1, nul, nul) == B_.E_NULL


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    """No fallback implementation: without the built library every call raises."""
    import paper_2410_03355_amd.binding as B
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "liblantern.so"))
    with pytest.raises(FileNotFoundError):
        B.load()
    with pytest.raises(FileNotFoundError):
        B.knn_workspace_bytes(0, 16, 8, 4)


def test_static_build_and_prepare_argument_errors(lib):
    """The entry point that allocates nothing refuses sizes beyond its scratch on the host."""
    import paper_2410_03355_amd as L
    p = ctypes.c_void_p(4096)
    nul = ctypes.c_void_p(0)
    call = lib.lantern_build_knn_static
    assert call(p, 9, 16, 8, 4, 0, p, nul, nul) == L.binding.E_DTYPE
    assert call(p, L.F32, 16, 8, 17, 0, p, nul, nul) == L.binding.E_SHAPE
    assert call(p, L.F32, 16, 8, 4, 5, p, nul, nul) == L.binding.E_SHAPE
    assert call(nul, L.F32, 16, 8, 4, 0, p, nul, nul) == L.binding.E_NULL
    assert call(p, L.F32, 16, 8, 4, 0, nul, nul, nul) == L.binding.E_NULL
    assert call(p, L.F32, L.binding.STATIC_MAX_V + 1, 8, 4, 0, p, nul, nul) == L.binding.E_WORKSPACE
    assert lib.lantern_prepare(7, 16, 4) == L.binding.E_DTYPE
    assert lib.lantern_prepare(L.F32, 0, 1) == L.binding.E_SHAPE
    assert lib.lantern_prepare(L.F32, 16, 17) == L.binding.E_SHAPE
    assert lib.lantern_prepare(L.BF16, L.MAX_VOCAB + 1, 4) == L.binding.E_SHAPE


def test_sequential_tree_argument_errors(lib):
    """Host-side validation of lantern_verify_trees_sequential and of its workspace size."""
    import paper_2410_03355_amd as L
    B_ = L.binding
    p = ctypes.c_void_p(4096)  # never dereferenced: validation fails first
    nul = ctypes.c_void_p(0)
    size = lib.lantern_verify_trees_sequential_workspace_bytes
    assert size(3, 5, 16) == 3 * 2 * 16 * 8 + 256
    assert size(3, 100, 16) == 3 * 2 * 16 * 8 + 1280
    assert size(0, 5, 16) == 0 and size(-1, 5, 16) == 0 and size(3, 0, 16) == 0 and size(3, 5, 0) == 0
    assert size(3, 5, L.MAX_VOCAB + 1) == 0 and size(1 << 20, 1 << 20, 16) == 0

    def call(tl=p, dl=p, dt=L.F32, R=5, V=16, stride=16, ri=p, par=p, B=2, M=3, tok=p, knn=p, k=4, div=0, delta=0.1,
             un=p, ol=p, op=p, on=p, ws=p, ws_bytes=1 << 20):
        return lib.lantern_verify_trees_sequential(tl, dl, dt, R, V, stride, ri, par, B, M, tok, knn, k, div, delta,
                                                   un, ol, op, on, ws, ws_bytes, nul)

    assert call(dt=9) == B_.E_DTYPE
    for kw in (dict(B=-1), dict(M=0), dict(B=1 << 20, M=1 << 20), dict(R=-1), dict(R=0), dict(V=0), dict(k=0),
               dict(k=17), dict(stride=15), dict(div=2), dict(ri=nul, R=5), dict(V=L.MAX_VOCAB + 1,
                                                                                stride=L.MAX_VOCAB + 1)):
        assert call(**kw) == B_.E_SHAPE, kw
    assert call(delta=-0.1) == B_.E_DELTA and call(delta=float("nan")) == B_.E_DELTA
    for name in ("tl", "dl", "par", "tok", "knn", "un", "ol", "op", "on"):
        assert call(**{name: nul}) == B_.E_NULL, name
    assert call(ws=nul) == B_.E_WORKSPACE
    assert call(ws=ctypes.c_void_p(4096 + 64)) == B_.E_WORKSPACE
    assert call(ws_bytes=2 * 2 * 16 * 8 + 255) == B_.E_WORKSPACE
    assert call(B=0, tl=nul, dl=nul, ws=nul, ws_bytes=0) == B_.OK   # nothing to do
