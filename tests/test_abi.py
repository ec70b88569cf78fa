"""The C-ABI library loads without a GPU and exports every symbol the header declares;
argument validation that precedes any device work is exercised here."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    src = open(os.path.join(ROOT, "include", "lsgd.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(lsgd_[a-z_]+)\s*\(", src)))


def test_header_declares_the_five_entry_points():
    names = declared_functions()
    for n in ["lsgd_create_population", "lsgd_grad_loss", "lsgd_select_leaders", "lsgd_pull_update", "lsgd_step"]:
        assert n in names


def test_library_exports_every_declared_symbol():
    import paper_1905_10395_amd as L
    lib = L.lib()
    for n in declared_functions():
        assert hasattr(lib, n), n


def test_validation_happens_before_device_work():
    import paper_1905_10395_amd as L
    from paper_1905_10395_amd import binding as b
    lib = L.lib()
    with pytest.raises(L.LsgdError, match="ld="):
        L.workspace_bytes(4, 100, 50, 1)
    with pytest.raises(L.LsgdError, match="not divisible"):
        L.workspace_bytes(5, 10, 10, 2)
    with pytest.raises(L.LsgdError, match="group_offsets"):
        L.workspace_bytes(5, 10, 10, 2, group_offsets=[0, 2, 4])
    with pytest.raises(L.LsgdError, match="empty"):
        L.workspace_bytes(5, 10, 10, 2, group_offsets=[0, 0, 5])
    with pytest.raises(L.LsgdError, match="momentum"):
        L.workspace_bytes(4, 10, 10, 2, momentum=float("nan"))
    with pytest.raises(L.LsgdError, match="flag"):
        L.workspace_bytes(4, 10, 10, 2, flags=1 << 20)
    assert L.workspace_bytes(5, 10, 10, 2, group_offsets=[0, 2, 5]) > 0
    # create: NULL buffers are rejected with a status, not a crash
    cfg, keep = b._config(4, 10, 12, 2, None, 0.9, 0, 0.0)
    h = C.c_void_p()
    st = lib.lsgd_create_population(C.byref(cfg), None, None, None, None, None, None, 0, None, C.byref(h))
    assert st == 1 and b"required" in lib.lsgd_last_error()
    st = lib.lsgd_pull_update(None, 0.1, 0.1, 0.1)
    assert st == 1
    # batch shape checks through the workspace query
    class Fake:
        def __init__(self, kind, d):
            self._d = d
            self.c = b._Batch(kind, C.cast(C.pointer(d), C.c_void_p))
    mc = Fake(b.BATCH_MC, b._MC(3, 4, 2, 1, 1, 1, 5, None, 0, 0.5))
    with pytest.raises(L.LsgdError, match=r"\(m\+n\)\*r"):
        L.workspace_bytes(4, 10, 12, 2, batch=mc)
    assert L.workspace_bytes(4, 14, 16, 2, batch=mc) > 0


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU; the benchmark says so instead of starting ranks."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
