"""Compile the HIP library for gfx950 into paper_2604_24088_amd/libtaco_hip.so.

Sources: csrc/taco_api.hip (C ABI, checks, diagnostics) and csrc/block_kernels.hip, which holds the
operator's kernels and is compiled once per block size (-DTACO_BLOCK=32 ... 512); the six objects are
built in parallel and linked.  hipcc cross-compiles without a GPU.

The library carries a digest of the sources it was built from (taco_build_id()); is_stale() compares
that digest with the sources on disk, so a library older than its sources is never used silently,
whatever the files' time stamps say.

Run as `python -m paper_2604_24088_amd.build` or call build()."""
import hashlib
import os
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtaco_hip.so")
BLOCKS = (32, 64, 128, 256, 512)
ID_MARKER = b"taco-build-id:"

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed-fp32 instructions are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # keep MFMA accumulators in ordinary VGPRs: the epilogue reads every result with VALU ops
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",
    "-Wall", "-Wno-unused-function",
]


def sources():
    """Every file the library is built from, in a fixed order."""
    own = sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".h", ".hip")))
    inc = os.path.join(os.path.dirname(HERE), "include")
    return own + [os.path.join(inc, "taco.h"), os.path.join(inc, "taco_debug.h")]


def source_digest() -> str:
    h = hashlib.sha256()
    for path in sources():
        h.update(os.path.basename(path).encode() + b"\0")
        with open(path, "rb") as f:
            h.update(f.read())
    h.update(" ".join(HIPCC_FLAGS).encode())
    return h.hexdigest()[:32]


def library_digest(path: str = LIB):
    """The digest embedded in a built library (read from the file, nothing is loaded), or None."""
    try:
        with open(path, "rb") as f:
            data = f.read()
    except OSError:
        return None
    at = data.find(ID_MARKER)
    if at < 0:
        return None
    at += len(ID_MARKER)
    return data[at:at + 32].decode("ascii", "replace")


def is_stale() -> bool:
    return library_digest() != source_digest()


def _run(cmd):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # The host pass warns that it does not know the packed-fp32 target feature: harmless.
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + out)
    return out


def build(force: bool = True, extra=(), jobs: int = 6) -> str:
    if not force and not is_stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    digest = source_digest()
    with tempfile.TemporaryDirectory(prefix="taco_build_") as tmp:
        units = [(os.path.join(CSRC, "taco_api.hip"), os.path.join(tmp, "api.o"), [f'-DTACO_BUILD_ID="{digest}"'])]
        units += [(os.path.join(CSRC, "block_kernels.hip"), os.path.join(tmp, f"block{b}.o"), [f"-DTACO_BLOCK={b}"]) for b in BLOCKS]
        cmds = [[hipcc] + HIPCC_FLAGS + list(extra) + defs + ["-c", src, "-o", obj] for src, obj, defs in units]
        with ThreadPoolExecutor(max_workers=max(1, jobs)) as pool:
            outs = list(pool.map(_run, cmds))
        outs.append(_run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + [u[1] for u in units] + ["-o", LIB + ".tmp"]))
    os.replace(LIB + ".tmp", LIB)
    text = "\n".join(o for o in outs if o.strip())
    if text:
        print(text, file=sys.stderr)
    if library_digest() != digest:
        raise RuntimeError(f"{LIB}: built, but its embedded digest does not match the sources")
    return LIB


def ensure_built() -> str:
    """The library that matches the sources on disk: built if missing or stale (tests, smoke and bench call this;
    the binding itself never builds)."""
    return build(force=False)


if __name__ == "__main__":
    print(build(force=True))
