"""Builds tests/c_abi_check (a plain C program on the C-ABI, linked with the HIP library, the
HIP runtime and the oracle) with the host compiler.  Called by __graft_entry__.build() and, if
the binary is missing, by tests/test_gpu_c_program.py."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
BINARY = os.path.join(HERE, "c_abi_check")


def build(force: bool = True) -> str:
    src = os.path.join(HERE, "c_abi_check.c")
    deps = [src, os.path.join(ROOT, "include", "ds.h"), os.path.join(ROOT, "paper_1905_05957_amd", "libds_hip.so"),
            os.path.join(ROOT, "oracle", "libds_oracle.so")]
    if not force and os.path.exists(BINARY) and all(os.path.getmtime(BINARY) >= os.path.getmtime(p) for p in deps):
        return BINARY
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    tmp = BINARY + ".tmp%d" % os.getpid()
    cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-Wextra", "-D__HIP_PLATFORM_AMD__", f"-I{rocm}/include",
           "-I" + os.path.join(ROOT, "include"), src, "-o", tmp,
           "-L" + os.path.join(ROOT, "paper_1905_05957_amd"), "-lds_hip", "-L" + os.path.join(ROOT, "oracle"), "-lds_oracle",
           f"-L{rocm}/lib", "-lamdhip64", "-lm",
           f"-Wl,-rpath,$ORIGIN/../paper_1905_05957_amd:$ORIGIN/../oracle:{rocm}/lib"]
    subprocess.run(cmd, check=True)
    os.replace(tmp, BINARY)
    return BINARY


if __name__ == "__main__":
    print(build())
