"""The C-ABI library loads on a machine without a GPU and exports every entry
point that include/dpaps.h declares (no compute call is made here)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "dpaps.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"^\s*(?:const\s+char\s*\*|int)\s*\*?\s*((?:ps|mf|kge)_\w+)\s*\(", text, flags=re.M)
    assert len(names) >= 14
    return names


def test_library_exports_every_declared_symbol():
    path = os.path.join(ROOT, "paper_2002_00655_amd", "libdpaps.so")
    if not os.path.exists(path):
        from paper_2002_00655_amd import build
        build.build(verbose=False)
    lib = ctypes.CDLL(path)
    for name in _declared():
        assert hasattr(lib, name), name


def test_binding_names_match_header():
    import importlib.util
    spec = importlib.util.find_spec("paper_2002_00655_amd.ps")
    src = open(spec.origin).read()
    for name in _declared():
        assert f"_lib.{name}" in src or f'"{name}"' in src, name


def test_host_side_argument_checks_need_no_gpu():
    """Null handles and null outputs are rejected before anything touches a device."""
    path = os.path.join(ROOT, "paper_2002_00655_amd", "libdpaps.so")
    lib = ctypes.CDLL(path)
    assert lib.ps_create(ctypes.c_int64(10), ctypes.c_int32(4), ctypes.c_int32(2), None) == -1
    h = ctypes.c_void_p()
    assert lib.ps_create(ctypes.c_int64(0), ctypes.c_int32(4), ctypes.c_int32(2), ctypes.byref(h)) == -1
    assert lib.ps_create(ctypes.c_int64(10), ctypes.c_int32(2000), ctypes.c_int32(2), ctypes.byref(h)) == -1
    assert lib.ps_destroy(None) == -1
    assert lib.ps_pull(None, 0, None, ctypes.c_int64(0), None, None) == -1
    assert lib.ps_status(None, None) == -1
