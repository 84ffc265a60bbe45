"""The CPU oracle under AddressSanitizer + UndefinedBehaviorSanitizer (host code only): a small C
driver calls every oracle entry point on bf16, fp8, grouped, local-expert and quantise-on-the-path
problems; any out-of-bounds access, overflow or misaligned load aborts the run."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    cmd = ["gcc", "-std=c11", "-O1", "-g", "-fno-omit-frame-pointer", "-fopenmp",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-Wall", "-Wextra",
           "-o", exe, os.path.join(ROOT, "tests", "oracle_sanitize_main.c"), "-lm"]
    built = subprocess.run(cmd, capture_output=True, text=True)
    assert built.returncode == 0, built.stderr
    env = dict(os.environ)
    # another library may already be preloaded into every process here; the sanitizer runtime then
    # must not insist on being first.  Leak checking needs ptrace, which containers often forbid.
    env["ASAN_OPTIONS"] = "verify_asan_link_order=0:detect_leaks=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["OMP_NUM_THREADS"] = "2"
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert run.stdout.strip().endswith("ok") and "runtime error" not in run.stderr
