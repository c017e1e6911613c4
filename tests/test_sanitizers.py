"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

Builds libagg.so with its HOST side instrumented (geometry, counts, index lists, every
validation path, the launch planning in the .hip files; device code is compiled as usual) and
the C oracle likewise, then runs the host-API tests and the oracle's pin tests against the two
instrumented libraries in a child interpreter that has the sanitizer runtime loaded first.
Any report (out-of-bounds access, use after free, signed overflow, misaligned access, ...)
aborts the child and fails this test."""
import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]


def _runtime():
    hits = glob.glob("/opt/rocm/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    return hits[0] if hits else None


def _preload_in_use():
    if os.environ.get("LD_PRELOAD"):
        return True
    try:
        return bool(open("/etc/ld.so.preload").read().strip())
    except OSError:
        return False


@pytest.mark.skipif(_runtime() is None, reason="clang's shared ASan runtime is not installed")
@pytest.mark.skipif(_preload_in_use(), reason="this environment preloads a library of its own; "
                    "the sanitizer runtime must be the first one loaded, so the run is skipped here")
def test_host_api_and_oracle_under_asan_ubsan(tmp_path):
    from paper_2512_02541_amd import build as b

    clang = os.path.join(os.path.dirname(os.path.realpath(b.HIPCC)), "..", "llvm", "bin", "clang")
    if not os.path.exists(clang):
        clang = "/opt/rocm/llvm/bin/clang"
    flags = [f for f in b.FLAGS if f != "-O3"] + ["-O1", "-g"]
    host_san = [x for f in SAN for x in ("-Xarch_host", f)]

    def compile_one(src):
        obj = str(tmp_path / (os.path.splitext(src)[0] + ".o"))
        subprocess.check_call([b.HIPCC, *flags, *host_san, "-I", os.path.join(ROOT, "include"),
                               "-I", b.CSRC, "-c", os.path.join(b.CSRC, src), "-o", obj],
                              stderr=subprocess.DEVNULL)
        return obj

    with ThreadPoolExecutor(max_workers=4) as pool:
        objs = list(pool.map(compile_one, b.SOURCES))
    agg_lib = str(tmp_path / "libagg_san.so")
    subprocess.check_call([b.HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *SAN,
                           "-shared-libasan", "-o", agg_lib, *objs], stderr=subprocess.DEVNULL)
    orc_lib = str(tmp_path / "libsga_oracle_san.so")
    subprocess.check_call([clang, "-O1", "-g", *SAN, "-shared-libasan", "-fopenmp", "-fPIC",
                           "-shared", "-std=c11", "-o", orc_lib,
                           os.path.join(ROOT, "oracle", "sga_oracle.c"), "-lm"])

    env = dict(os.environ)
    env.update({
        "LD_PRELOAD": _runtime(),
        "ASAN_OPTIONS": "detect_leaks=0:halt_on_error=1:abort_on_error=1",
        "UBSAN_OPTIONS": "halt_on_error=1:print_stacktrace=1",
        "AGG_LIBRARY_PATH": agg_lib,
        "SGA_ORACLE_LIBRARY_PATH": orc_lib,
        "OMP_NUM_THREADS": "4",
    })
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider",
           os.path.join(ROOT, "tests", "test_host_api.py"),
           os.path.join(ROOT, "tests", "test_oracle_pins.py"),
           "-k", "not attention_kernel_leaves_m0"]
    run = subprocess.run(cmd, cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                         text=True, timeout=900)
    tail = "\n".join(run.stdout.splitlines()[-40:])
    assert run.returncode == 0, tail
    assert "passed" in tail and "ERROR: AddressSanitizer" not in run.stdout \
        and "runtime error:" not in run.stdout, tail
