"""Boundary checks that need no GPU: the built library loads, exports every function that
include/ds.h declares, and rejects bad configurations before touching a device."""
import ctypes as C
import os
import re

import pytest

import paper_1905_05957_amd as P
from paper_1905_05957_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "ds.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(ds_[a-z_]+)\s*\(", text)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    lib = P.load_library()
    names = _declared_functions()
    assert set(names) == set(B.EXPORTS), (names, B.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings_and_version():
    lib = P.load_library()
    assert lib.ds_status_string(0) == b"ok"
    seen = {lib.ds_status_string(c) for c in range(0, 7)}
    assert len(seen) == 7
    assert re.fullmatch(rb"\d+\.\d+", lib.ds_version())


def _create(**kw):
    cfg = B.ds_config_t()
    cfg.comp, cfg.n, cfg.d = kw.get("comp", B.COMP_SIGN), kw.get("n", 4), kw.get("d", 1024)
    cfg.grad_dtype = kw.get("grad_dtype", 0)
    cfg.scale_mode, cfg.chunk = kw.get("scale_mode", 0), kw.get("chunk", 0)
    cfg.k, cfg.bucket, cfg.levels = kw.get("k", 0), kw.get("bucket", 512), kw.get("levels", 15)
    keep = None
    if "seg" in kw:
        keep = (C.c_int64 * len(kw["seg"]))(*kw["seg"])
        cfg.seg_offsets = C.cast(keep, C.POINTER(C.c_int64))
        cfg.n_seg = len(kw["seg"]) - 1
    h = C.c_void_p()
    rc = P.load_library().ds_create(C.byref(cfg), C.byref(h))
    assert rc != 0 and not h.value
    return rc


def test_create_rejects_bad_arguments_before_any_device_work():
    lib = P.load_library()
    h = C.c_void_p()
    assert lib.ds_create(None, C.byref(h)) == 1                      # DS_ERR_NULL
    assert _create(n=0) == 2 and _create(d=0) == 2                   # DS_ERR_SHAPE
    assert _create(d=1 << 31) == 2
    assert _create(comp=9) == 3                                      # DS_ERR_CONFIG
    assert _create(grad_dtype=5) == 3
    assert _create(scale_mode=7) == 3
    assert _create(scale_mode=B.SCALE_CHUNK, chunk=0) == 3
    assert _create(scale_mode=B.SCALE_SEGMENTS) == 1                 # offsets missing
    assert _create(scale_mode=B.SCALE_SEGMENTS, seg=[0, 10, 10, 1024]) == 3
    assert _create(scale_mode=B.SCALE_SEGMENTS, seg=[0, 10, 1000]) == 3
    assert _create(comp=B.COMP_TOPK, k=0) == 2 and _create(comp=B.COMP_TOPK, k=2000) == 2
    assert _create(comp=B.COMP_QSGD, bucket=100) == 3
    assert _create(comp=B.COMP_QSGD, levels=16) == 3
    assert _create(comp=B.COMP_CLIP, levels=0) == 3 and _create(comp=B.COMP_CLIP, levels=32) == 3
    assert _create(comp=B.COMP_RSPARSE, k=0) == 3 and _create(comp=B.COMP_RSPARSE, k=(1 << 24) + 1) == 3


def test_destroy_accepts_null():
    assert P.load_library().ds_destroy(None) == 0


def test_bench_refuses_more_than_one_gpu():
    import subprocess, sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr


def test_header_is_plain_c99_and_cxx():
    """include/ds.h is the boundary: it must compile on its own as C99 and as C++ (no torch or
    HIP types in the signatures)."""
    import shutil
    import subprocess
    header = os.path.join(ROOT, "include", "ds.h")
    if shutil.which("gcc") is None:
        pytest.skip("no host compiler")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c", header], check=True)
    subprocess.run(["g++", "-std=c++17", "-Wall", "-Werror", "-fsyntax-only", "-x", "c++", header], check=True)
    text = open(header).read()
    assert "torch" not in text and "hipStream_t hip" not in text and "#include <hip" not in text
