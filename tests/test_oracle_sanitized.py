"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): a small driver walks every
entry point on ragged sizes; an out-of-bounds access or undefined arithmetic in the checker itself aborts the run."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_c_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_sanitized")
    build = subprocess.run(
        ["gcc", "-std=c11", "-O1", "-g", "-fopenmp", "-fno-fast-math", "-fsanitize=address,undefined",
         "-fno-sanitize-recover=all", "-static-libasan",
         os.path.join(ROOT, "tests", "c_client", "oracle_sanitized.c"), os.path.join(ROOT, "oracle", "power_smc_oracle.c"),
         "-o", exe, "-lm"], capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    run = subprocess.run([exe], capture_output=True, text=True, timeout=120,
                         env=dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0"))
    assert run.returncode == 0 and "oracle_sanitized ok" in run.stdout, run.stdout + run.stderr
