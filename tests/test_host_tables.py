"""CPU-side safety net, no GPU needed: the library's host logic (descriptor validation, tile and
panel enumeration, the XCD deal) and the C oracle, each built with g++ / gcc under the address
and undefined-behaviour sanitizers and run once; and the oracle's whole pin suite once more
against a build with the undefined-behaviour sanitizer compiled in."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
NATIVE = os.path.join(ROOT, "tests", "native")
SAN = ["-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=all"]


def _run(cmd, **kw):
    res = subprocess.run(cmd, capture_output=True, text=True, timeout=600, **kw)
    assert res.returncode == 0, f"{' '.join(cmd)}\n{res.stdout[-3000:]}\n{res.stderr[-3000:]}"
    return res.stdout


def test_every_tile_exactly_once_in_every_table(tmp_path):
    exe = str(tmp_path / "host_tables_check")
    _run(["g++", "-std=c++17"] + SAN + ["-I" + os.path.join(ROOT, "include"),
         "-I" + os.path.join(ROOT, "paper_2603_11873_amd", "csrc"), "-o", exe, os.path.join(NATIVE, "host_tables_check.cpp")])
    out = _run([exe])
    assert "host tables ok" in out


def test_oracle_entry_points_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitizer_driver")
    _run(["gcc", "-std=c11", "-fopenmp"] + SAN + ["-o", exe, os.path.join(NATIVE, "oracle_sanitizer_driver.c"),
         os.path.join(ROOT, "oracle", "adafuse_oracle.c"), "-lm"])
    out = _run([exe], env=dict(os.environ, ASAN_OPTIONS="detect_leaks=1"))
    assert "oracle under sanitizers ok" in out


def test_oracle_pins_hold_with_the_ubsan_build():
    """Every oracle pin once more, in a fresh interpreter that loads the instrumented library (any
    finding aborts that process)."""
    env = dict(os.environ, ADAFUSE_ORACLE_UBSAN="1")
    out = _run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                os.path.join(ROOT, "tests", "test_oracle_bf16.py"), os.path.join(ROOT, "tests", "test_oracle_router.py"),
                os.path.join(ROOT, "tests", "test_oracle_switch.py")], env=env, cwd=ROOT)
    assert " passed" in out and "failed" not in out
