"""CPU-only hygiene checks that need a compiler, not a GPU:
  * the oracle under AddressSanitizer + UndefinedBehaviorSanitizer on a sweep of every method x compressor;
  * include/comp_ams.h handed to a C11 compiler (the ABI is C, and every other test reaches it through ctypes);
  * the library's host side (argument validation, error paths) under the same sanitizers, driven by a C program.
Each runs in a subprocess with its own freshly built binary; nothing here loads the built libraries."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all"]


def run(cmd, **kw):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert r.returncode == 0, f"{' '.join(cmd)}\n{r.stdout[-4000:]}"
    return r.stdout


def test_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_sanitize_sweep")
    run(["gcc", "-std=c11", "-O1", "-g", *SAN, "-static-libasan", "-fopenmp", "-ffp-contract=off", "-Wall", "-Wextra",
         "-o", exe, os.path.join(ROOT, "oracle", "sanitize_sweep.c"), os.path.join(ROOT, "oracle", "comp_ams_oracle.c"),
         "-lm"])
    env = dict(os.environ, OMP_NUM_THREADS="3", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0")
    out = run([exe], env=env)
    assert "sanitize sweep: 96 cases done" in out
    assert "ERROR" not in out and "runtime error" not in out


def test_header_is_plain_c11():
    run(["gcc", "-std=c11", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only",
         "-I", os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "c", "abi_validation.c")])


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="no hipcc")
def test_host_side_validation_is_clean_under_sanitizers(tmp_path):
    """The host code of the library compiled with ASan + UBSan (the device code is compiled as always)
    and linked with a C11 program that calls every entry point with invalid arguments and NULL handles."""
    from paper_2111_00705_amd import build as B
    drv = str(tmp_path / "abi_validation.o")
    obj = str(tmp_path / "comp_ams_san.o")
    exe = str(tmp_path / "abi_validation")
    run(["gcc", "-std=c11", "-Wall", "-Wextra", "-Werror", "-c", "-I", os.path.join(ROOT, "include"), "-o", drv,
         os.path.join(ROOT, "tests", "c", "abi_validation.c")])
    host_san = []
    for f in ("-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all", "-g"):
        host_san += ["-Xarch_host", f]
    flags = [f for f in B.HIPCC_FLAGS if f not in ("-O3", "-shared", "-fPIC")]
    run([HIPCC, "-O1", *flags, *host_san, "-c", "-o", obj, B.SOURCES[0]])
    run([HIPCC, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-Wno-option-ignored", "-o", exe,
         obj, drv])
    out = run([exe], env=dict(os.environ, ASAN_OPTIONS="detect_leaks=1"))
    assert "abi validation: 0 failures" in out
    assert "ERROR" not in out and "runtime error" not in out
