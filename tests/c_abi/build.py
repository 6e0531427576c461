"""Build tests/c_abi/c_abi_check: a plain C99 program linked against the HIP
library, the HIP runtime and the C oracle.  Test infrastructure."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
EXE = os.path.join(HERE, "c_abi_check")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def build() -> str:
    from oracle import build as oracle_build
    oracle_lib = oracle_build.build()
    pkg = os.path.join(ROOT, "paper_2510_15882_amd")
    tmp = EXE + ".tmp.%d" % os.getpid()
    subprocess.check_call([
        "gcc", "-std=c99", "-O1", "-Wall", "-Wextra", "-Werror",
        "-I", os.path.join(ROOT, "include"), "-isystem", os.path.join(ROCM, "include"),
        os.path.join(HERE, "c_abi_check.c"), "-o", tmp,
        "-L", pkg, "-lflexlink", "-L", os.path.dirname(oracle_lib), "-lflex_oracle",
        "-L", os.path.join(ROCM, "lib"), "-lamdhip64",
        "-Wl,-rpath,$ORIGIN/../../paper_2510_15882_amd", "-Wl,-rpath,$ORIGIN/../../oracle",
        "-Wl,-rpath," + os.path.join(ROCM, "lib"),
    ])
    os.replace(tmp, EXE)
    return EXE


if __name__ == "__main__":
    print(build())
