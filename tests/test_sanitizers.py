"""CPU-only sanitizer builds: the oracle, and the host side of the C ABI (argument validation, workspace layout arithmetic,
knobs), each compiled with AddressSanitizer + UndefinedBehaviorSanitizer and run by a small driver program (tests/sanitize/)."""
import os
import subprocess

import pytest

from paper_2602_08404_amd import build as tb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "sanitize")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_asan")
    subprocess.run(["gcc", "-std=c11", *SAN, "-fopenmp", "-fno-fast-math", "-ffp-contract=off", "-Wall", "-Wextra", "-o", exe,
                    os.path.join(ROOT, "oracle", "team_moe_oracle.c"), os.path.join(HERE, "oracle_driver.c"), "-lm"], check=True)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=ENV)
    assert r.returncode == 0 and "ok" in r.stdout, (r.stdout[-2000:], r.stderr[-4000:])
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr


def test_host_side_of_the_abi_under_sanitizers(tmp_path):
    """api.hip and tuning.hip are rebuilt with sanitized host code (device code is unaffected) and linked with the library's other
    objects; the driver only makes calls that must be rejected on the host, so no GPU is needed."""
    if not os.path.isdir(tb.OBJ) or not os.path.exists(tb.LIB):
        tb.build()
    host_san = [a for f in SAN[:2] for a in ("-Xarch_host", f)] + ["-g", "-O1"]
    objs = []
    for src in ("api.hip", "tuning.hip"):
        o = str(tmp_path / src.replace(".hip", "_asan.o"))
        subprocess.run([tb.HIPCC, *[f for f in tb.FLAGS if f != "-O3"], *host_san, "-c", os.path.join(tb.CSRC, src), "-o", o], check=True,
                       stderr=subprocess.DEVNULL)
        objs.append(o)
    others = [os.path.join(tb.OBJ, f) for f in sorted(os.listdir(tb.OBJ)) if f.endswith(".o") and f not in ("api.o", "tuning.o")]
    drv = str(tmp_path / "abi_driver.o")
    subprocess.run([tb.HIPCC, "-x", "c++", "-std=c++17", *SAN, "-c", os.path.join(HERE, "abi_driver.cpp"), "-o", drv], check=True)
    exe = str(tmp_path / "abi_asan")
    subprocess.run([tb.HIPCC, "--offload-arch=gfx950", "-fsanitize=address,undefined", "-o", exe, drv, *objs, *others], check=True,
                   stderr=subprocess.DEVNULL)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=dict(ENV, ASAN_OPTIONS="detect_leaks=0"))
    assert r.returncode == 0 and "ok" in r.stdout, (r.stdout[-2000:], r.stderr[-4000:])
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
