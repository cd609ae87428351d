"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only, no GPU): a
private copy of oracle/ is built with -fsanitize=address,undefined and the pin files run against
it in a subprocess.  Any out-of-bounds access, use after free, signed overflow, misaligned access
or invalid shift in the oracle's C ends that run with an error."""
import os
import shutil
import subprocess
import sys
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PIN_FILES = ["tests/test_oracle_pins.py", "tests/test_oracle_c1_toy.py", "tests/test_oracle_more_compressors.py"]


def _runtime(name):
    if shutil.which("gcc") is None:
        pytest.skip("no host compiler")
    path = subprocess.run(["gcc", f"-print-file-name={name}"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(path) or not os.path.exists(path):
        pytest.skip(f"{name} is not installed")
    return path


def test_pins_pass_on_a_sanitized_build_of_the_oracle():
    asan = _runtime("libasan.so")
    tmp = tempfile.mkdtemp(prefix="oracle_sanitized_")
    try:
        for sub in ("oracle", "tests"):
            shutil.copytree(os.path.join(ROOT, sub), os.path.join(tmp, sub),
                            ignore=shutil.ignore_patterns("__pycache__", "*.so", "*.tmp*", "c_abi_check"))
        shutil.copy(os.path.join(ROOT, "ds_workloads.py"), tmp)
        init = os.path.join(tmp, "oracle", "__init__.py")
        text = open(init).read()
        plain = '_CFLAGS = ["-O2",'
        assert plain in text
        with open(init, "w") as f:
            f.write(text.replace(plain, '_CFLAGS = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", '
                                        '"-fno-omit-frame-pointer", "-g", "-O1",'))
        env = dict(os.environ, OMP_NUM_THREADS="1", OPENBLAS_NUM_THREADS="1", MKL_NUM_THREADS="1",
                   ASAN_OPTIONS="detect_leaks=0:halt_on_error=1:abort_on_error=0",
                   UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
        env["LD_PRELOAD"] = ":".join(p for p in (asan, os.environ.get("LD_PRELOAD", "")) if p)   # the runtime comes first
        r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider", *PIN_FILES],
                           cwd=tmp, capture_output=True, text=True, env=env, timeout=1200)
        assert r.returncode == 0, (r.stdout[-3000:], r.stderr[-3000:])
        built = os.path.join(tmp, "oracle", "libds_oracle.so")
        syms = subprocess.run(["nm", "-D", built], capture_output=True, text=True).stdout
        assert "__asan_init" in syms and "__ubsan_handle" in syms, "the copy was not built with the sanitizers"
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
