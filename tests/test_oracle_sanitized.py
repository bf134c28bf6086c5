"""The oracle's C code under AddressSanitizer and UndefinedBehaviorSanitizer (host only, no GPU):
every function runs once on small, exactly sized heap buffers; any access past a buffer, signed
overflow or invalid shift in its index arithmetic aborts the run."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = tmp_path / "oracle_san"
    subprocess.check_call(
        ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fno-fast-math", "-ffp-contract=off",
         "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
         "-o", str(exe), os.path.join(HERE, "oracle_sanitize_main.c"), os.path.join(ROOT, "oracle", "dgq_oracle.c"), "-lm"])
    # the environment is passed on unchanged except for the sanitizer's own options (libraries
    # preloaded by the environment may come before the sanitizer runtime: do not insist on the order)
    env = dict(os.environ, OMP_NUM_THREADS="2", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0")
    r = subprocess.run([str(exe)], env=env, capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and r.stdout.strip() == "ok", r.stdout + r.stderr
