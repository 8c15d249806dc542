"""Compile the HIP library (csrc/taco_api.hip and the kernel headers it includes) for gfx950
into paper_2604_24088_amd/libtaco_hip.so.  hipcc cross-compiles without a GPU.

Run as `python -m paper_2604_24088_amd.build` or call build()."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
SRC = os.path.join(CSRC, "taco_api.hip")
LIB = os.path.join(HERE, "libtaco_hip.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 instructions are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # keep MFMA accumulators in ordinary VGPRs: the epilogue reads every result with VALU ops
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return [SRC] + sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")) + \
        [os.path.join(os.path.dirname(HERE), "include", "taco.h")]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(s) > t for s in sources())


def build(force: bool = True, extra=()) -> str:
    if not force and not is_stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + list(extra) + [SRC, "-o", LIB]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # The host pass warns that it does not know the packed-fp32 target feature: harmless.
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if out.strip():
        print(out, file=sys.stderr)
    return LIB


def ensure_built() -> str:
    """Build only when no library is there (tests, smoke and bench call this; the binding itself never builds)."""
    return LIB if os.path.exists(LIB) else build(force=True)


if __name__ == "__main__":
    print(build(force=True))
