"""Sanitizer passes over the CPU-side code (no GPU): the oracle's pin suite
against an AddressSanitizer + UndefinedBehaviorSanitizer build of es_oracle.c,
and the host-side launch planning of the HIP library (reachable without a GPU
through es_spmm_launch_info and the argument checks) under UBSan."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run_pytest(files, env_extra):
    env = dict(os.environ)
    env.update(env_extra)
    # -s: a sanitizer report goes to the process's own stderr and the process
    # exits at once; with pytest's fd capture in between it would be lost
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-s", "-p", "no:cacheprovider", "-m", "not gpu"] + files
    return subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)


def test_oracle_pins_under_asan_and_ubsan(tmp_path):
    src = os.path.join(ROOT, "oracle", "es_oracle.c")
    lib = str(tmp_path / "libes_oracle_san.so")
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-fno-omit-frame-pointer",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-Wall", "-Wextra",
                    "-o", lib, src, "-lm"], check=True)
    asan_rt = subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, capture_output=True,
                             text=True).stdout.strip()
    assert os.path.isabs(asan_rt) and os.path.exists(asan_rt), "gcc has no shared ASan runtime"
    # the interpreter is not instrumented, so the runtime is preloaded (in front
    # of whatever is preloaded already); leak checking would report CPython itself
    preload = ":".join(p for p in (asan_rt, os.environ.get("LD_PRELOAD", "")) if p)
    res = _run_pytest(["tests/test_oracle_pins.py", "tests/test_oracle_properties.py"],
                      {"ES_ORACLE_LIBRARY": lib, "LD_PRELOAD": preload,
                       "ASAN_OPTIONS": "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0",
                       "UBSAN_OPTIONS": "print_stacktrace=1:halt_on_error=1"})
    out = res.stdout + res.stderr
    assert res.returncode == 0, out[-4000:]
    assert "runtime error" not in out and "AddressSanitizer" not in out, out[-4000:]
    assert " passed" in res.stdout


def test_sanitized_oracle_catches_a_planted_overrun(tmp_path):
    """The pass above means something only if the instrumented build does trap:
    a copy of the oracle with one planted off-by-one write must be reported."""
    src = open(os.path.join(ROOT, "oracle", "es_oracle.c")).read()
    needle = "for (int64_t i = 0; i < stride; ++i) {"
    assert src.count(needle) == 1
    bad = tmp_path / "es_oracle_planted.c"
    bad.write_text(src.replace(needle, "for (int64_t i = 0; i <= stride; ++i) {"))
    lib = str(tmp_path / "libes_oracle_planted.so")
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fPIC", "-shared", "-fopenmp",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-o", lib, str(bad), "-lm"],
                   check=True)
    asan_rt = subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, capture_output=True,
                             text=True).stdout.strip()
    preload = ":".join(p for p in (asan_rt, os.environ.get("LD_PRELOAD", "")) if p)
    res = _run_pytest(["tests/test_oracle_pins.py::test_bucket_is_first_k_positions"],
                      {"ES_ORACLE_LIBRARY": lib, "LD_PRELOAD": preload,
                       "ASAN_OPTIONS": "detect_leaks=0:verify_asan_link_order=0"})
    assert res.returncode != 0
    assert "heap-buffer-overflow" in (res.stdout + res.stderr)


def test_host_launch_planning_under_ubsan(tmp_path):
    """libes_spmm.so rebuilt with UBSan on the host pass only (trap mode: any
    undefined behaviour in the planning arithmetic kills the process), then the
    host-logic tests -- the launch-shape grid and the argument checks -- rerun
    against it."""
    from paper_2104_10716_amd import build
    lib = str(tmp_path / "libes_spmm_ubsan.so")
    build.build(out=lib, extra_flags=["-g", "-Xarch_host", "-fsanitize=undefined,integer-divide-by-zero",
                                      "-Xarch_host", "-fsanitize-trap=all"])
    res = _run_pytest(["tests/test_launch_shape.py", "tests/test_abi.py"], {"ES_SPMM_LIBRARY": lib})
    out = res.stdout + res.stderr
    assert res.returncode == 0, out[-4000:]
    assert " passed" in res.stdout
