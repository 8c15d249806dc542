"""Compile tests/abi_client/client.c with the C compiler (gcc, C11) against include/taco.h, the built HIP
library and the HIP runtime's C API.  Run as `python tests/abi_client/build.py` or call build()."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
SRC = os.path.join(HERE, "client.c")
EXE = os.path.join(HERE, "client")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def build() -> str:
    libdir = os.path.join(ROOT, "paper_2604_24088_amd")
    cmd = ["gcc", "-std=c11", "-Wall", "-Wextra", "-Werror", "-O1", f"-I{ROCM}/include", f"-I{ROOT}/include", SRC, "-o", EXE,
           f"-L{ROCM}/lib", "-lamdhip64", f"-L{libdir}", "-ltaco_hip",
           "-Wl,-rpath,$ORIGIN/../../paper_2604_24088_amd", f"-Wl,-rpath,{ROCM}/lib", "-lm"]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("gcc failed:\n" + res.stdout)
    return EXE


def ensure_built() -> str:
    return EXE if os.path.exists(EXE) else build()


if __name__ == "__main__":
    print(build())
