"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, and rejects bad arguments before touching HIP."""
import ctypes as C
import os
import re

import pytest

import paper_2510_10129_amd as cc
from paper_2510_10129_amd import _lib

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _header_symbols():
    txt = open(os.path.join(ROOT, "include", "cacheclip.h")).read()
    txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
    return sorted(set(re.findall(r"\b(cc_[a-z_]+)\s*\(", txt)))


def test_library_exports_every_declared_symbol():
    lib = cc.load_library()
    names = _header_symbols()
    assert "cc_select" in names and "cc_recompute_layer" in names and len(names) >= 14
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(_lib.EXPORTS)


def test_create_rejects_bad_arguments_without_a_gpu():
    lib = cc.load_library()
    h = C.c_void_p()
    assert lib.cc_create(None, None, None) == _lib.CC_ERR_NULL
    good = dict(d=256, H_q=4, H_kv=2, d_h=64, f=1024, rope_base=1e4, rms_eps=1e-5,
                N_cap=128, M_cap=64, T_cap=128)
    for k, v in (("d", 100), ("d_h", 96), ("H_kv", 3), ("f", 1000), ("T_cap", 1 << 20),
                 ("M_cap", 0), ("rope_base", 1.0), ("H_q", 128)):
        bad = dict(good)
        bad[k] = v
        if k == "H_q":
            bad["H_kv"] = 2          # ratio 64 > 32
        desc = cc.ModelDesc(**bad)
        assert lib.cc_create(C.byref(h), C.byref(desc), None) == _lib.CC_ERR_SHAPE, k
        assert h.value is None
        assert len(lib.cc_last_error(None)) > 0


def test_null_context_is_an_error():
    lib = cc.load_library()
    assert lib.cc_select(None, None, 1, 1, 1, 0, 8, 0, 0, 0, 0, None, None, None) == _lib.CC_ERR_NULL
    assert lib.cc_recompute_layer(None, None, 0, None, None, None, 0, None, None, 0) == _lib.CC_ERR_NULL
    assert lib.cc_destroy(None) == _lib.CC_OK


def test_product_package_does_not_touch_the_oracle():
    pkg = os.path.join(ROOT, "paper_2510_10129_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                txt = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in txt, os.path.join(dirpath, f)
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith(".py"):
            txt = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2510_10129_amd" not in txt and "cacheclip" not in txt.lower().replace(
                "cacheclip hot path", ""), f


def test_context_free_calls_reject_bad_arguments_without_a_gpu():
    lib = cc.load_library()
    # cc_select_noalloc checks its arguments before it touches the device
    assert lib.cc_select_noalloc(None, None, 1, 1, 1, 0, 8, 0, 0, 0, 0, None, None) == _lib.CC_ERR_NULL
    buf = (C.c_float * 8)()
    out = (C.c_int32 * 8)()
    p, o = C.cast(buf, C.c_void_p), C.cast(out, C.c_void_p)
    for args, code in (((p, 0, 4, 4, 0, 8, 0, 0, 0, 0, o, o), _lib.CC_ERR_SHAPE),              # Q_a < 1
                       ((p, 1, 4, 2, 0, 8, 0, 0, 0, 0, o, o), _lib.CC_ERR_SHAPE),              # ld < T
                       ((p, 1, 131073, 131073, 0, 8, 0, 0, 0, 0, o, o), _lib.CC_ERR_WORKSPACE),  # beyond the scratch
                       ((p, 1, 4, 4, 10001, 8, 0, 0, 0, 0, o, o), _lib.CC_ERR_SHAPE),
                       ((p, 1, 4, 4, 100, 0, 0, 0, 0, 0, o, o), _lib.CC_ERR_SHAPE),
                       ((p, 1, 4, 4, 100, 8, 9, 0, 0, 0, o, o), _lib.CC_ERR_SHAPE),
                       ((p, 1, 4, 4, 100, 8, 0, 0, -1, 0, o, o), _lib.CC_ERR_SHAPE)):
        assert lib.cc_select_noalloc(None, *args) == code, args
        assert len(lib.cc_last_error(None)) > 0
    assert lib.cc_debug_set_launch(None, None) == _lib.CC_ERR_NULL


def test_launch_override_struct_matches_the_header():
    txt = open(os.path.join(ROOT, "include", "cacheclip.h")).read()
    body = txt[txt.index("typedef struct cc_launch_override {"):txt.index("} cc_launch_override;")]
    fields = re.findall(r"int32_t\s+(\w+);", body)
    assert fields == [n for n, _ in _lib.LaunchOverride._fields_]
    assert C.sizeof(_lib.LaunchOverride) == 4 * len(fields)
