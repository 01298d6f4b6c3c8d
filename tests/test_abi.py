"""CPU-side checks of the C-ABI library: it loads, exports what the header declares, and rejects
bad arguments before touching a GPU.  No compute call is made here."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "adacons.h")


@pytest.fixture(scope="module")
def lib():
    import paper_2411_03742_amd as pkg
    return pkg


def _declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(adacons_[a-z_]+)\s*\(", text)))


def test_header_declares_the_named_entry_points():
    syms = _declared_symbols()
    for name in ("adacons_init_state", "adacons_aggregate", "adacons_coeffs"):
        assert name in syms


def test_library_exports_every_declared_symbol(lib):
    cdll = ctypes.CDLL(lib.library_path())
    declared = _declared_symbols()
    assert len(declared) >= 15
    for name in declared:
        assert hasattr(cdll, name), f"{name} declared in adacons.h but not exported"
    assert sorted(lib.EXPORTS) == declared


def test_status_strings(lib):
    cdll = ctypes.CDLL(lib.library_path())
    cdll.adacons_status_string.restype = ctypes.c_char_p
    seen = {cdll.adacons_status_string(i) for i in range(6)}
    assert len(seen) == 6 and b"ok" in seen


def test_argument_validation_needs_no_gpu(lib):
    cdll = ctypes.CDLL(lib.library_path())
    cdll.adacons_init_state.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int, ctypes.c_int64,
                                        ctypes.c_double, ctypes.c_uint, ctypes.c_void_p]
    cdll.adacons_last_error.restype = ctypes.c_char_p
    st = ctypes.c_void_p()
    EINVAL, EUNSUPPORTED = 1, 2
    assert cdll.adacons_init_state(None, 4, 10, 0.9, 3, None) == EINVAL
    assert cdll.adacons_init_state(ctypes.byref(st), 0, 10, 0.9, 3, None) == EINVAL
    assert cdll.adacons_init_state(ctypes.byref(st), 129, 10, 0.9, 3, None) == EUNSUPPORTED
    assert b"ADACONS_N_MAX" in cdll.adacons_last_error()
    assert cdll.adacons_init_state(ctypes.byref(st), 4, 0, 0.9, 3, None) == EINVAL
    assert cdll.adacons_init_state(ctypes.byref(st), 4, 10, 1.0, 3, None) == EINVAL
    assert cdll.adacons_init_state(ctypes.byref(st), 4, 10, float("nan"), 3, None) == EINVAL
    assert cdll.adacons_init_state(ctypes.byref(st), 4, 10, 0.9, 16, None) == EINVAL
    assert st.value is None
    # NULL state handles are rejected by every call that takes one
    cdll.adacons_aggregate.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int,
                                       ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    assert cdll.adacons_aggregate(None, 4, 10, 0, None, None, None) == EINVAL
    assert cdll.adacons_destroy_state(None) == 0
    # the layer-wise and worker-share entry points check their arguments before touching the device too
    i64p = ctypes.POINTER(ctypes.c_int64)
    cdll.adacons_init_layers.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int, ctypes.c_int, i64p,
                                         ctypes.c_int, ctypes.c_double, ctypes.c_uint, ctypes.c_void_p]
    ls = ctypes.c_void_p()
    good = (ctypes.c_int64 * 3)(0, 40, 100)
    for args in [(None, 4, 2, good, 0, 0.9, 3, None),
                 (ctypes.byref(ls), 4, 2, None, 0, 0.9, 3, None),
                 (ctypes.byref(ls), 0, 2, good, 0, 0.9, 3, None),
                 (ctypes.byref(ls), 4, 0, good, 0, 0.9, 3, None),
                 (ctypes.byref(ls), 4, 2, good, 0, 1.5, 3, None),
                 (ctypes.byref(ls), 4, 2, good, 0, 0.9, 32, None),
                 (ctypes.byref(ls), 4, 2, (ctypes.c_int64 * 3)(1, 40, 100), 0, 0.9, 3, None),
                 (ctypes.byref(ls), 4, 2, (ctypes.c_int64 * 3)(0, 40, 40), 0, 0.9, 3, None)]:
        assert cdll.adacons_init_layers(*args) == EINVAL, args
    assert cdll.adacons_init_layers(ctypes.byref(ls), 129, 2, good, 0, 0.9, 3, None) == EUNSUPPORTED
    assert cdll.adacons_init_layers(ctypes.byref(ls), 4, 2, good, 7, 0.9, 3, None) == EUNSUPPORTED
    assert ls.value is None
    assert cdll.adacons_destroy_layers(None) == 0
    cdll.adacons_aggregate_layers.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int,
                                              ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    assert cdll.adacons_aggregate_layers(None, 4, 100, 0, None, None, None) == EINVAL
    cdll.adacons_worker_stats.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int,
                                          ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    assert cdll.adacons_worker_stats(None, None, 10, 0, None, None, None) == EINVAL


def test_product_path_never_touches_the_oracle():
    """The GPU package and the benchmark's GPU leg must not route through the CPU oracle."""
    pkg = os.path.join(ROOT, "paper_2411_03742_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f"{f} mentions the oracle"
    otext = open(os.path.join(ROOT, "oracle", "adacons_oracle.py")).read()
    assert "paper_2411_03742_amd" not in otext and "libadacons" not in otext


def test_no_cuda_shims_or_dual_paths():
    pkg = os.path.join(ROOT, "paper_2411_03742_amd", "csrc")
    for f in os.listdir(pkg):
        text = open(os.path.join(pkg, f)).read()
        for banned in ("__HIP_PLATFORM_AMD__", "__CUDACC__", "cuda_runtime", "hipify"):
            assert banned not in text


def test_noalloc_entry_point_rejects_sizes_beyond_its_maximum_before_touching_a_gpu(lib):
    cdll = ctypes.CDLL(lib.library_path())
    vp = ctypes.c_void_p
    cdll.adacons_aggregate_noalloc.argtypes = [vp, ctypes.c_int, ctypes.c_int64, ctypes.c_int, ctypes.c_double,
                                               ctypes.c_uint, vp, vp, vp, vp, vp]
    cdll.adacons_last_error.restype = ctypes.c_char_p
    EINVAL, EUNSUPPORTED, EALIGN = 1, 2, 3
    assert cdll.adacons_aggregate_noalloc(None, 129, 10, 0, 0.9, 3, 8, None, None, 16, None) == EUNSUPPORTED
    assert b"maximum of 128 workers" in cdll.adacons_last_error()
    assert cdll.adacons_aggregate_noalloc(None, 0, 10, 0, 0.9, 3, 8, None, None, 16, None) == EINVAL
    assert cdll.adacons_aggregate_noalloc(None, 4, 10, 0, 1.5, 3, 8, None, None, 16, None) == EINVAL
    assert cdll.adacons_aggregate_noalloc(None, 4, 10, 0, 0.9, 3, None, None, None, 16, None) == EINVAL
    assert cdll.adacons_aggregate_noalloc(None, 4, 10, 0, 0.9, 3, 12, None, None, 16, None) == EALIGN


def test_binding_constants_equal_the_header(lib):
    """Every enumerator and flag the header defines with a value (status codes, dtypes, flags, numeric
    flags, tuning keys, limits) has the same value under the same name in the Python binding."""
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    found = {}
    for name, value in re.findall(r"\b(ADACONS_[A-Z0-9_]+)\s*=\s*(0x[0-9a-fA-F]+|\d+)u?\b", text):
        found[name] = int(value, 0)
    for name, value in re.findall(r"#define\s+(ADACONS_[A-Z0-9_]+)\s+(0x[0-9a-fA-F]+|\d+)u?\b", text):
        found[name] = int(value, 0)
    assert len(found) >= 20, found
    missing = [n for n in found if not n.endswith("_") and not hasattr(lib, n)]
    assert not missing, missing
    for name, value in found.items():
        if hasattr(lib, name):
            assert getattr(lib, name) == value, (name, getattr(lib, name), value)
