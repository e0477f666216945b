"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only; CPU).

A C driver (tests/oracle_sanitize_driver.c) calls both oracle routines on small ragged cases with buffers
exactly as large as the documented extents.  It is built twice from the same sources, once plainly and once
with -fsanitize=address,undefined (runtime linked statically, so nothing has to be preloaded); the sanitized
run must finish without a report and print exactly what the plain build prints."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = [os.path.join(ROOT, "oracle", "dlm_oracle.c"), os.path.join(ROOT, "tests", "oracle_sanitize_driver.c")]


def build_and_run(tmp_path, name, flags):
    exe = tmp_path / name
    subprocess.check_call(["gcc", "-std=c11", "-g", "-O1", *flags, *SRC, "-o", str(exe), "-lm"])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:halt_on_error=1:verify_asan_link_order=0",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1", OMP_NUM_THREADS="4")
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, f"{name}: rc {r.returncode}\n{r.stdout}\n{r.stderr}"
    assert "ERROR" not in r.stderr and "runtime error" not in r.stderr, r.stderr
    return r.stdout


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    plain = build_and_run(tmp_path, "plain", ["-fopenmp"])
    assert plain.strip().endswith("ok")
    assert "attn empty out0 0.000 lse0 -inf" in plain and "lm V=1 conf 1.000 tok 0 z2nd -inf" in plain
    san = build_and_run(tmp_path, "sanitized", ["-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                                                "-static-libasan", "-fno-omit-frame-pointer"])
    assert san == plain          # serial, sanitized build computes the same values as the OpenMP build
