"""The CPU oracle under AddressSanitizer + UndefinedBehaviorSanitizer (host code only): a small C driver that includes
the oracle's source pushes valid, ragged, unquantizable and corrupted inputs through every entry point."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_is_clean_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "nzo_san")
    src = os.path.join(ROOT, "oracle", "sanitize_main.c")
    subprocess.run(["gcc", "-std=gnu99", "-O1", "-g", "-fno-fast-math", "-ffp-contract=off",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
                    "-o", exe, src, "-lm"], check=True, cwd=os.path.join(ROOT, "oracle"))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    p = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert p.returncode == 0 and "sanitize ok" in p.stdout, p.stdout[-4000:]
