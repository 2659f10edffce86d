"""CPU-only checks of the C-ABI library: it loads without a GPU, exports every symbol the header declares,
and its host-only entry points reject bad arguments.  No kernel is launched here."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _header_functions():
    text = open(os.path.join(ROOT, "include", "cnnc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cnnc_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    import paper_1508_01292_amd as P
    if not os.path.exists(P.library_path()):
        pytest.fail("libcnnc.so is not built; run __graft_entry__.build()")
    L = P.lib()
    declared = _header_functions()
    assert len(declared) >= 20
    for name in declared:
        assert hasattr(L, name), "libcnnc.so does not export " + name
    # the binding's own list names the same functions
    assert sorted(P.EXPORTS) == declared
    assert L.cnnc_version().decode().startswith("cnnc")


def test_host_only_argument_checks_need_no_gpu():
    import paper_1508_01292_amd as P
    L = P.lib()
    # null handles are rejected before anything touches a device
    assert L.cnnc_destroy(C.c_void_p(0)) == -1
    assert L.cnnc_set_params(C.c_void_p(0), C.c_void_p(0)) == -1
    assert L.cnnc_stage1_scoremap(C.c_void_p(0), C.c_void_p(0)) == -1
    assert L.cnnc_eval_stage(C.c_void_p(0), C.c_int(2), C.c_void_p(0)) == -1
    assert L.cnnc_measure_peaks(C.c_void_p(0), C.c_void_p(0), C.c_void_p(0)) == -1
    out = C.c_void_p(123)
    assert L.cnnc_create(C.byref(out), C.c_void_p(0), C.c_int(640), C.c_int(480), C.c_int(100)) == -1
    assert out.value is None            # the handle is cleared on failure
    assert L.cnnc_last_error(C.c_void_p(0)) == b"null context"


def test_missing_library_is_an_error_not_a_fallback(monkeypatch):
    import paper_1508_01292_amd.binding as B
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "_LIB_PATH", os.path.join(ROOT, "does_not_exist", "libcnnc.so"))
    with pytest.raises(ImportError):
        B.lib()


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_1508_01292_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower() or f == "__init__.py" and False, f + " mentions the oracle"


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr


def test_struct_sizes_and_step_names_match_the_library():
    """The ctypes mirrors of the C structs and the list of timed steps must be what the library was compiled with
    (cnnc_get_timings writes CNNC_T_COUNT entries into arrays sized by the binding)."""
    import ctypes as C
    from paper_1508_01292_amd import binding as B
    sizes = B.cnnc_abi_sizes()
    assert sizes == (C.sizeof(B._Layer), C.sizeof(B._StageDesc), C.sizeof(B._Params), C.sizeof(B.Detection),
                     C.sizeof(B.Region), len(B.STEP_NAMES), C.sizeof(B.RegionDetection))


def test_records_view_the_memory_the_library_fills():
    """The binding hands back what a call wrote as one block; records are made from it only when asked for."""
    import numpy as np
    from paper_1508_01292_amd.binding import Detection, RegionDetection, Records
    r = Records(Detection, 64)
    assert C.sizeof(Detection) == 32 and r._raw.size == 64 * 32
    words = np.frombuffer(r._raw, np.int32)
    words[:24] = np.arange(24)                        # what a C call would leave: three records
    assert r._filled(3, 64) is r and len(r) == 3 and r._raw.size == 96          # the unused tail is given back
    assert [d.x for d in r] == [0, 8, 16] and r[2].index == 22 and r[-1].y == 17
    assert [d.as_dict()["neighbors"] for d in r[1:]] == [13, 21]
    assert r.array.dtype.names[:3] == ("x", "y", "size") and list(r.array["level"]) == [4, 12, 20]
    with pytest.raises(IndexError):
        r[3]
    empty = Records(RegionDetection, 0)._filled(0, 0)
    assert len(empty) == 0 and not empty and list(empty) == []
    assert len(Records(Detection, 4)._filled(9, 4)) == 4                         # never more than the capacity
    assert empty == [] and r == [d.as_dict() for d in r] and r == list(r) and r != [] and r != list(r)[:2]
    twin = Records(Detection, 3)
    twin._raw[:] = r._raw
    assert twin._filled(3, 3) == r
