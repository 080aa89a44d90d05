"""Sanitizer leg for the host code of the oracle (no GPU): oracle/*.c built with AddressSanitizer and
UndefinedBehaviorSanitizer and driven through all of its routines by tests/oracle_sanitize_main.c.  Any report ends the
program with a non-zero status; the outputs must also be the same as those of an unsanitized build."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SOURCES = [os.path.join(ROOT, "oracle", "oracle.c"), os.path.join(ROOT, "oracle", "epilogue.c"),
           os.path.join(ROOT, "tests", "oracle_sanitize_main.c")]


def build_and_run(tmp_path, name, flags):
    exe = str(tmp_path / name)
    subprocess.check_call(["gcc", "-std=c11", "-g", "-Wall", "-Wextra"] + flags + ["-o", exe] + SOURCES + ["-lm"])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stderr[-3000:]
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-3000:]
    return r.stdout.strip()


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    plain = build_and_run(tmp_path, "plain", ["-O2"])
    sanitized = build_and_run(tmp_path, "sanitized", ["-O1", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                                                       "-fno-sanitize-recover=all"])
    assert len(plain) == 16 and plain == sanitized
