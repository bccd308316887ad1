"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only, no GPU): cc_oracle.c is built
with -fsanitize=address,undefined into a temporary folder and the oracle's pins run against that build in a child
process that has the sanitizer runtime preloaded.  An out-of-bounds index, a signed overflow or a bad shift anywhere
on the paths the pins take ends the child with an error."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "cc_oracle.c")
PIN_FILES = ["test_oracle_costs.py", "test_oracle_2opt.py", "test_oracle_rdswap.py", "test_oracle_sa.py",
             "test_oracle_bcube.py", "test_oracle_dbt.py", "test_oracle_probes.py", "test_oracle_local.py"]


def _runtime(name: str) -> str:
    path = subprocess.check_output(["gcc", f"-print-file-name={name}"], text=True).strip()
    return path if os.path.isabs(path) and os.path.exists(path) else ""


def test_oracle_pins_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    asan = _runtime("libasan.so")
    if not asan:
        pytest.skip("gcc has no libasan.so here")
    lib = tmp_path / "libcc_oracle_san.so"
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c99", "-fPIC", "-shared", "-fno-omit-frame-pointer",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", SRC, "-o", str(lib)])
    env = dict(os.environ)
    env["CC_ORACLE_LIB"] = str(lib)
    env["LD_PRELOAD"] = ":".join(x for x in (asan, env.get("LD_PRELOAD", "")) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:halt_on_error=1"      # the interpreter's own leaks aside
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu"]
    cmd += [os.path.join(ROOT, "tests", f) for f in PIN_FILES]
    p = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=1500)
    tail = (p.stdout[-3000:] + "\n" + p.stderr[-3000:])
    assert p.returncode == 0, tail
    assert "passed" in p.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error" not in tail, tail


def test_the_sanitized_build_does_notice_an_overrun(tmp_path):
    """The harness above would be worthless if an instrumented build kept quiet: plant a heap overrun in a copy of
    the source (the scratch order of the definition-tier move value one rank short) and expect the child to die."""
    asan = _runtime("libasan.so")
    if not asan:
        pytest.skip("gcc has no libasan.so here")
    text = open(SRC).read()
    old = "int32_t *u = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);\n    memcpy(u, t, sizeof(int32_t) * (size_t)N);"
    assert text.count(old) >= 1
    new = old.replace("(size_t)N);\n", "(size_t)(N - 1));\n", 1)
    c_file, lib = tmp_path / "overrun.c", tmp_path / "overrun.so"
    c_file.write_text(text.replace(old, new, 1))
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c99", "-fPIC", "-shared", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", str(c_file), "-o", str(lib)])
    env = dict(os.environ)
    env["CC_ORACLE_LIB"] = str(lib)
    env["LD_PRELOAD"] = ":".join(x for x in (asan, env.get("LD_PRELOAD", "")) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:halt_on_error=1"
    code = ("import numpy as np, oracle\n"
            "n = 8\n"
            "c = np.ones((n, n), dtype=np.int32)\n"
            "print(oracle.move_value_by_definition(c, oracle.SUM, np.arange(n, dtype=np.int32), 2, 5))\n")
    p = subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=env, capture_output=True, text=True, timeout=300)
    assert p.returncode != 0 and "AddressSanitizer" in p.stderr, p.stdout + p.stderr[-2000:]
