"""Builds tests/c_client/zeco_c_client: the plain-C client of libzeco.so together with the C oracle
(gcc, C11, -pedantic on the library's header; links libzeco.so and the HIP runtime).  No GPU needed to build."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
EXE = os.path.join(HERE, "zeco_c_client")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def build(force=True):
    src = os.path.join(HERE, "zeco_c_client.c")
    csrc = os.path.join(ROOT, "paper_2507_01004_amd", "csrc")
    if not force and os.path.exists(EXE) and os.path.getmtime(EXE) >= os.path.getmtime(src):
        return EXE
    subprocess.check_call(
        ["gcc", "-std=c11", "-O2", "-Wall", "-Wextra", "-pedantic", "-fopenmp", "-D__HIP_PLATFORM_AMD__",
         "-I" + os.path.join(ROOT, "include"), "-isystem", os.path.join(ROCM, "include"),
         src, os.path.join(ROOT, "oracle", "gla_oracle.c"),
         "-L" + csrc, "-L" + os.path.join(ROCM, "lib"), "-lzeco", "-lamdhip64", "-lm",
         "-Wl,-rpath,$ORIGIN/../../paper_2507_01004_amd/csrc", "-Wl,-rpath," + os.path.join(ROCM, "lib"), "-o", EXE])
    return EXE


if __name__ == "__main__":
    print(build())
