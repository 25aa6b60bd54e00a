"""Build tests/bin/c_abi_caller: tests/c_abi_caller.c (a C99 program that calls the library through
include/dit_attn.h) linked with the C oracle it checks the results against.  gcc only; needs
libdit_attn.so to be built first.  `python tests/build_c_caller.py`."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def build_c_caller():
    out_dir = os.path.join(HERE, "bin")
    os.makedirs(out_dir, exist_ok=True)
    exe = os.path.join(out_dir, "c_abi_caller")
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    lib_dir = os.path.join(ROOT, "paper_2601_20655_amd")
    cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-fopenmp", "-I", os.path.join(ROOT, "include"),
           "-I", os.path.join(rocm, "include"), os.path.join(HERE, "c_abi_caller.c"),
           os.path.join(ROOT, "oracle", "dit_oracle.c"), "-o", exe, "-L", lib_dir, "-ldit_attn",
           "-L", os.path.join(rocm, "lib"), "-lamdhip64", "-lm",
           "-Wl,-rpath,$ORIGIN/../../paper_2601_20655_amd", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    subprocess.check_call(cmd)
    return exe


if __name__ == "__main__":
    print(build_c_caller())
