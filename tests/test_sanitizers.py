"""Host-side sanitizer builds (CPU only): the C checker and the library's host code (validation, closed-form sizes,
budget rule, plan layout, latency table, tuning, batching) run under AddressSanitizer and UndefinedBehaviorSanitizer.
Device code is compiled as usual and never executed here; GPU sanitizers are not used."""
import os
import subprocess
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
CSRC = os.path.join(ROOT, "paper_2604_13847_amd", "csrc")


def _run(cmd, **kw):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
    assert r.returncode == 0, f"{' '.join(cmd)}\n{out[-4000:]}"
    return out


def test_checker_under_asan_and_ubsan():
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "oracle_san")
        _run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
              "-o", exe, os.path.join(SAN, "oracle_driver.c"), "-lm"])
        out = _run([exe], env={**os.environ, "OMP_NUM_THREADS": "4"})
        assert "mode 1 checksum" in out


def test_library_host_code_under_asan_and_ubsan():
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "host_san")
        srcs = [os.path.join(CSRC, f) for f in ("sb_host.hip", "sb_sab.hip", "sb_coverage.hip", "sb_topk.hip", "sb_scores.hip")]
        _run(["hipcc", "-O1", "-g", "--offload-arch=gfx950", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
              "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined",
              "-w", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, os.path.join(SAN, "host_driver.cpp"), *srcs, "-o", exe], cwd=tmp)
        # (the HIP runtime keeps a few allocations for the life of the process: leak checking is left off)
        out = _run([exe], env={**os.environ, "ASAN_OPTIONS": "detect_leaks=0"})
        assert "host driver OK" in out
