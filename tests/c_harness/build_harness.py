"""Compile kvl_c_parity.c (plain C, gcc) against the built library, the HIP runtime
and the oracle's C source.  The binary lands beside this file."""
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(_HERE))
EXE = os.path.join(_HERE, "kvl_c_parity")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def build() -> str:
    pkg = os.path.join(ROOT, "paper_2602_21548_amd")
    if not os.path.exists(os.path.join(pkg, "libkvl.so")):
        raise RuntimeError("libkvl.so is not built: run python -m paper_2602_21548_amd.build first")
    cmd = ["gcc", "-std=c11", "-O1", "-Wall", "-Wextra", "-D__HIP_PLATFORM_AMD__",
           "-I", os.path.join(ROCM, "include"), "-I", os.path.join(ROOT, "include"),
           os.path.join(_HERE, "kvl_c_parity.c"), os.path.join(ROOT, "oracle", "kvl_oracle.c"),
           "-o", EXE + ".tmp", "-L", pkg, "-lkvl", "-L", os.path.join(ROCM, "lib"), "-lamdhip64",
           "-Wl,-rpath,$ORIGIN/../../paper_2602_21548_amd", "-Wl,-rpath," + os.path.join(ROCM, "lib")]
    p = subprocess.run(cmd, capture_output=True, text=True)
    if p.returncode != 0:
        raise RuntimeError("gcc failed:\n" + p.stderr)
    os.replace(EXE + ".tmp", EXE)
    return EXE


if __name__ == "__main__":
    print(build())
