"""Do the pins pin?  Each entry below plants ONE plausible mistake in a copy of the oracle's source (a dropped
term, a wrong constant, a wrong sign or index, a swapped branch), builds the copy and runs the pin tests against
it (TACO_REF_LIB points the oracle's loader at the copy): at least one pin must fail for every mutant.  Nothing
here touches the real oracle or the HIP path."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "taco_ref.cpp")

CORE = ["tests/test_oracle_e4m3.py", "tests/test_oracle_hadamard.py", "tests/test_oracle_blocks.py", "tests/test_oracle_roundtrip.py"]
VARIANTS = ["tests/test_oracle_ablation.py", "tests/test_oracle_e4m3.py", "tests/test_oracle_blocks.py"]

# (name, text in the source, replacement, pin files)
MUTANTS = [
    ("eps dropped", "std::sqrt(energy / B + eps)", "std::sqrt(energy / B)", CORE),
    ("sigma divides by B - 1", "std::sqrt(energy / B + eps)", "std::sqrt(energy / (B - 1) + eps)", CORE),
    ("alpha inverted", "static_cast<float>(tau / sigma)", "static_cast<float>(sigma / tau)", CORE),
    ("Hadamard sign from i | j", "parity_of(static_cast<unsigned>(i & j))", "parity_of(static_cast<unsigned>(i | j))", CORE),
    ("Q_max 240", "constexpr double kQmax = 448.0;", "constexpr double kQmax = 240.0;", CORE),
    ("ties round up", "if (diff > 0.5) return fl + 1.0;", "if (diff >= 0.5) return fl + 1.0;", CORE),
    ("saturation gives the NaN code", "if (a >= kQmax) return sign | 0x7e;", "if (a >= kQmax) return sign | 0x7f;", CORE),
    ("E4M3 bias off by one", "mag = std::ldexp(8.0 + static_cast<double>(m), e - 10);",
     "mag = std::ldexp(8.0 + static_cast<double>(m), e - 11);", CORE),
    ("E4M3 subnormal step", "mag = std::ldexp(static_cast<double>(m), -9);", "mag = std::ldexp(static_cast<double>(m), -10);", CORE),
    ("bf16 truncates", "if (rest > 0x8000u || (rest == 0x8000u && (keep & 1u))) keep += 1;", "", CORE),
    ("energy of |g|", "energy += g[j] * g[j];", "energy += std::fabs(g[j]);", CORE),
    ("matrix product reads x backwards", "acc += row[j] * x[j];", "acc += row[j] * x[B - 1 - j];", CORE),
    ("E5M2 bias off by one", "else mag = std::ldexp(4.0 + static_cast<double>(m), e - 17);",
     "else mag = std::ldexp(4.0 + static_cast<double>(m), e - 18);", VARIANTS),
    ("E5M2 subnormal step", "else if (e == 0) mag = std::ldexp(static_cast<double>(m), -16);",
     "else if (e == 0) mag = std::ldexp(static_cast<double>(m), -17);", VARIANTS),
    ("E5M2 Q_max", "constexpr double kQmaxE5M2 = 57344.0;", "constexpr double kQmaxE5M2 = 49152.0;", VARIANTS),
    ("E5M2 saturates to infinity", "if (a >= kQmaxE5M2) return sign | 0x7b;", "if (a >= kQmaxE5M2) return sign | 0x7c;", VARIANTS),
    ("E5M2 carry lost", "if (steps == 8.0) { steps = 4.0; p += 1; }", "if (steps == 8.0) { steps = 4.0; }", VARIANTS),
    ("INT8 clamps at 128", "double r = a >= 127.0 ? 127.0 : round_half_even(a);", "double r = a >= 128.0 ? 128.0 : round_half_even(a);",
     VARIANTS),
    ("INT8 sign dropped", "if (std::signbit(v)) q = -q;", "", VARIANTS),
    ("INT8 truncates", "double r = a >= 127.0 ? 127.0 : round_half_even(a);", "double r = a >= 127.0 ? 127.0 : std::floor(a);", VARIANTS),
    ("decoders swapped", "return format == FORMAT_E4M3 ? e4m3_decode(c) : format == FORMAT_E5M2 ? e5m2_decode(c) : int8_decode(c);",
     "return format == FORMAT_E4M3 ? e4m3_decode(c) : format == FORMAT_E5M2 ? int8_decode(c) : e5m2_decode(c);", VARIANTS),
    ("decode ignores the rotate bit", "    if (mode & MODE_ROTATE) {", "    if (true) {", VARIANTS),
]


def run_mutant(args):
    name, old, new, pins, tmp = args
    text = open(SRC).read()
    if old not in text:
        return name, "pattern not found in oracle/taco_ref.cpp (update this test with the oracle)"
    d = os.path.join(tmp, name.replace(" ", "_").replace("|", "or"))
    os.makedirs(d, exist_ok=True)
    src, lib = os.path.join(d, "taco_ref_mutant.cpp"), os.path.join(d, "libtaco_ref_mutant.so")
    open(src, "w").write(text.replace(old, new, 1))
    build = subprocess.run(["g++", "-std=c++17", "-O2", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", src, "-o", lib],
                           stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if build.returncode != 0:
        return name, "mutant does not compile:\n" + build.stdout[-500:]
    env = dict(os.environ, TACO_REF_LIB=lib, OMP_NUM_THREADS="2")
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + pins, cwd=ROOT, env=env,
                         stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    return name, None if res.returncode == 1 else f"SURVIVED (pytest exit {res.returncode}): no pin noticed it"


def test_every_planted_mistake_is_caught(tmp_path):
    with ThreadPoolExecutor(max_workers=6) as pool:
        results = list(pool.map(run_mutant, [m + (str(tmp_path),) for m in MUTANTS]))
    problems = [f"{name}: {why}" for name, why in results if why]
    assert not problems, "\n".join(problems)
