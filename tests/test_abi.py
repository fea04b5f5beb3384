"""The C-ABI library loads, exports every function declared in include/vlq.h and
rejects bad arguments before touching the GPU (no compute calls here)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def vlq():
    import paper_1901_00275_amd as vlq
    from paper_1901_00275_amd import build as vlq_build

    if not os.path.exists(vlq.LIB_PATH):
        vlq_build.build()
    return vlq


def _declared():
    src = open(os.path.join(ROOT, "include", "vlq.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(vlq_[a-z_]+)\s*\(", src)))


def test_every_declared_symbol_is_exported(vlq):
    names = _declared()
    assert {"vlq_build_index", "vlq_encode", "vlq_search"} <= set(names) and len(names) >= 15
    L = vlq.lib()
    for name in names:
        assert hasattr(L, name), name
    assert vlq.vlq_version() == 1


def test_binding_has_the_same_names(vlq):
    for name in _declared():
        assert hasattr(vlq, name), name


def test_binding_has_the_same_constants(vlq):
    """Options, stages and error codes of the header agree with the binding's constants."""
    src = open(os.path.join(ROOT, "include", "vlq.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    opts, stages = 0, []
    for body in re.findall(r"enum\s*\{(.*?)\}", src, flags=re.S):
        value = -1
        for item in body.split(","):
            item = item.strip()
            if not item:
                continue
            m = re.match(r"(VLQ_[A-Z0-9_]+)\s*(?:=\s*(-?\d+))?$", item)
            assert m, item
            value = int(m.group(2)) if m.group(2) is not None else value + 1
            name = m.group(1)
            if name.endswith("_COUNT"):
                continue
            if name.startswith("VLQ_STAGE_"):
                assert value == len(stages)
                stages.append(name[len("VLQ_STAGE_"):].lower())
            else:
                assert getattr(vlq, name) == value, name
                opts += 1
    assert opts >= 8 and tuple(stages) == tuple(vlq.STAGES)
    for name, value in re.findall(r"#define\s+(VLQ_(?:OK|E[A-Z]+))\s+\(?(-?\d+)\)?", src):
        assert getattr(vlq, name) == int(value), name


@pytest.mark.parametrize("d,nlist,n,m,lo,hi", [
    (0, 16, 4, 1, 0, 0), (128, 16, 4, 7, 0, 0), (128, 4, 4, 8, 0, 0), (128, 16, 0, 8, 0, 0),
    (128, 16, 4, 8, 0.1, 0.5), (128, 16, 4, 8, -0.3, 0.5), (2048, 16, 4, 8, 0, 0), (128, 16, 4, 128, 0, 0),
])
def test_bad_params_are_rejected_without_a_gpu(vlq, d, nlist, n, m, lo, hi):
    L = vlq.lib()
    prm = vlq.vlq_params_t(d, nlist, n, m, lo, hi)
    out = C.c_void_p()
    fake = C.c_void_p(256)
    rc = L.vlq_build_index(C.byref(prm), fake, fake, None, 0, None, None, C.byref(out))
    assert rc == vlq.VLQ_EINVAL and not out.value
    assert vlq.vlq_last_error() != ""


def test_null_arguments(vlq):
    L = vlq.lib()
    prm = vlq.vlq_params_t(128, 16, 4, 8, 0, 0)
    out = C.c_void_p()
    assert L.vlq_build_index(None, None, None, None, 0, None, None, C.byref(out)) == vlq.VLQ_EINVAL
    assert L.vlq_build_index(C.byref(prm), None, None, None, 0, None, None, C.byref(out)) == vlq.VLQ_EINVAL
    assert L.vlq_build_index(C.byref(prm), C.c_void_p(256), C.c_void_p(256), None, 5, None, None, C.byref(out)) == vlq.VLQ_EINVAL
    assert L.vlq_search(None, None, 1, 1, 1, 1, None, None, None) == vlq.VLQ_EINVAL
    assert L.vlq_encode(None, None, 1, None, None, None, None, None) == vlq.VLQ_EINVAL
    assert L.vlq_index_finalize(None, None) == vlq.VLQ_EINVAL
    assert L.vlq_index_ntotal(None) == -1
    L.vlq_index_free(None)  # allowed


def test_missing_library_fails_loudly(vlq, monkeypatch):
    monkeypatch.setattr(vlq, "_lib", None)
    monkeypatch.setattr(vlq, "LIB_PATH", "/nonexistent/libvlq.so")
    with pytest.raises(FileNotFoundError):
        vlq.lib()


def test_bench_refuses_more_than_one_gpu():
    """The build runs on one GPU only: bench.py --gpus N (N > 1) exits with a message saying so,
    before anything touches the GPU."""
    import subprocess
    import sys

    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=120)
    assert res.returncode != 0
    assert "ONE GPU" in res.stderr and res.stdout.strip() == ""
