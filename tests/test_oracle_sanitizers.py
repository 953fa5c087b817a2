"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): a C driver calls
every oracle function on valid, empty and malformed inputs held in exactly sized heap buffers."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ORACLE = os.path.join(os.path.dirname(HERE), "oracle")


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    subprocess.check_call(["gcc", "-std=c11", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan", "-Wall", "-Wextra", "-I", ORACLE,
                           os.path.join(HERE, "oracle_sanitize_driver.c"), os.path.join(ORACLE, "emb_oracle.c"),
                           "-o", exe, "-lm"])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "sanitizer run clean" in r.stdout and "runtime error" not in r.stderr
