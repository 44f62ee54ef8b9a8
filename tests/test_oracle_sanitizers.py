"""The CPU checker under AddressSanitizer and UndefinedBehaviorSanitizer (host code only)."""
import os
import subprocess
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_checker_runs_clean_under_asan_and_ubsan():
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "oracle_sanitize")
        subprocess.run(["g++", "-O1", "-g", "-std=c++17", "-ffp-contract=off",
                        "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                        os.path.join(ROOT, "oracle", "tabx_ref.cpp"),
                        os.path.join(ROOT, "tests", "oracle_sanitize_main.cpp"), "-o", exe],
                       check=True)
        env = dict(os.environ)
        env.pop("LD_PRELOAD", None)          # the sanitizer runtime must come first
        out = subprocess.run([exe], capture_output=True, text=True, timeout=120, env=env)
        assert out.returncode == 0, out.stderr[-2000:]
        assert out.stdout.strip() == "ok"
