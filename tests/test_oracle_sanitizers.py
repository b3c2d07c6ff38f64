"""The CPU oracle under AddressSanitizer + UndefinedBehaviorSanitizer (host code only): every function once on a small
problem with exactly sized heap buffers."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def test_oracle_runs_clean_under_asan_ubsan(tmp_path):
    exe = tmp_path / "oracle_san"
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-o", str(exe),
           os.path.join(ROOT, "oracle", "oracle.c"), os.path.join(HERE, "sanitize_oracle_main.c"), "-lm"]
    subprocess.run(cmd, check=True)
    env = dict(os.environ)
    env.pop("LD_PRELOAD", None)                       # the sanitizer runtime must come first in the link order
    env["ASAN_OPTIONS"] = "detect_leaks=0"
    env["OMP_NUM_THREADS"] = "2"
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "sanitizer run ok" in r.stdout
