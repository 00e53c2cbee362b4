"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header
declares, and rejects bad configurations before touching any device."""

import ctypes
import os
import re

import pytest

from paper_2501_19309_amd import binding as jb


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(jb.LIB_PATH):
        from paper_2501_19309_amd.build import build_library
        build_library()
    return jb.load_library()


def test_header_symbols_are_exported(lib, repo_root):
    hdr = open(os.path.join(repo_root, "include", "jd_verify.h")).read()
    declared = set(re.findall(r"\b(jd_verify_[a-z0-9_]+)\s*\(", hdr))
    assert {"jd_verify_create", "jd_verify_run", "jd_verify_destroy"} <= declared
    assert declared == set(jb.EXPORTED_SYMBOLS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_header_constants_match_binding(repo_root):
    hdr = open(os.path.join(repo_root, "include", "jd_verify.h")).read()
    consts = {m[0]: m[1] for m in re.findall(r"#define\s+(JD_[A-Z0-9_]+)\s+(-?\d+)u?\b", hdr)}
    for name, val in consts.items():
        assert getattr(jb, name) == int(val), name
    assert len(consts) >= 20


def test_struct_layout_matches_header():
    assert ctypes.sizeof(jb.jd_verify_config) == 16 * 4
    assert ctypes.sizeof(jb.jd_verify_outputs) == 11 * 8


def test_strerror(lib):
    for code in (0, -1, -2, -3, -4, -5):
        assert jb.strerror(code)
    assert jb.strerror(-99) == "unknown error code"


def test_validate_config_error_paths(lib):
    ok = dict(d=4096, V=128256, max_B=1, max_M=25)
    assert jb.jd_verify_validate_config(jb.make_config(**ok)) == jb.JD_OK
    assert jb.jd_verify_validate_config(jb.make_config(**ok, w_dtype=jb.JD_F32)) == jb.JD_OK
    assert lib.jd_verify_validate_config(None) == jb.JD_ERR_INVALID_ARG
    bad_shape = [dict(ok, max_M=64), dict(ok, max_M=0), dict(ok, max_B=0), dict(ok, d=0), dict(ok, V=-1),
                 dict(ok, d=4100)]
    for kw in bad_shape:
        assert jb.jd_verify_validate_config(jb.make_config(**kw)) == jb.JD_ERR_SHAPE, kw
    bad_arg = [dict(delta=0.4), dict(delta=1.1), dict(delta=float("nan")), dict(temperature=0.0),
               dict(temperature=-1.0), dict(w_dtype=7), dict(w_layout=2), dict(draft_kind=3), dict(mode=-1),
               dict(device=-1), dict(judge_bias=float("inf")), dict(rule=2), dict(resample=-1)]
    for kw in bad_arg:
        assert jb.jd_verify_validate_config(jb.make_config(**ok, **kw)) == jb.JD_ERR_INVALID_ARG, kw
    assert jb.jd_verify_validate_config(jb.make_config(**ok, w_dtype=jb.JD_BF16, emb_dtype=jb.JD_F32)) \
        == jb.JD_ERR_UNSUPPORTED_DTYPE
    for k in (0, -3, 128257):
        assert jb.jd_verify_validate_config(jb.make_config(**ok, rule=jb.JD_RULE_TOPK, top_k=k)) == jb.JD_ERR_SHAPE
    assert jb.jd_verify_validate_config(jb.make_config(**ok, rule=jb.JD_RULE_TOPK, top_k=128256)) == jb.JD_OK
    assert jb.jd_verify_validate_config(jb.make_config(**ok, top_k=0)) == jb.JD_OK  # ignored under Eq. 4
    fp8 = dict(ok, w_dtype=jb.JD_FP8_E4M3)
    assert jb.jd_verify_validate_config(jb.make_config(**fp8)) == jb.JD_OK
    assert jb.jd_verify_validate_config(jb.make_config(**fp8, emb_dtype=jb.JD_F32)) == jb.JD_ERR_UNSUPPORTED_DTYPE
    assert jb.jd_verify_validate_config(jb.make_config(**dict(fp8, d=4104))) == jb.JD_ERR_SHAPE
    # fp32 has no 8-element alignment requirement
    assert jb.jd_verify_validate_config(jb.make_config(100, 1000, 1, 5, w_dtype=jb.JD_F32)) == jb.JD_OK


def test_create_rejects_before_touching_the_device(lib):
    h = ctypes.c_void_p(123)
    cfg = jb.make_config(4096, 128256, 1, 64)
    assert lib.jd_verify_create(ctypes.byref(cfg), 1, 1, ctypes.byref(h)) == jb.JD_ERR_SHAPE
    assert h.value is None
    cfg = jb.make_config(4096, 128256, 1, 5)
    assert lib.jd_verify_create(ctypes.byref(cfg), None, 1, ctypes.byref(h)) == jb.JD_ERR_INVALID_ARG
    assert lib.jd_verify_create(ctypes.byref(cfg), 1, 1, None) == jb.JD_ERR_INVALID_ARG
    # a weight scale is only meaningful for quantised weights
    assert lib.jd_verify_create_scaled(ctypes.byref(cfg), 1, 1, 1, ctypes.byref(h)) == jb.JD_ERR_INVALID_ARG
    assert lib.jd_verify_destroy(None) == jb.JD_OK
    assert lib.jd_verify_run(None, 1, 1, None, None, None, None, 1, None, None, None) == jb.JD_ERR_INVALID_ARG
    assert lib.jd_verify_profile_begin(None, 4) == jb.JD_ERR_INVALID_ARG


def test_no_oracle_import_in_product_path(repo_root):
    pkg = os.path.join(repo_root, "paper_2501_19309_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.replace("no oracle", ""), os.path.join(dirpath, f)
