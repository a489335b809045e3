"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: a C driver calls every oracle function on
exactly sized buffers (tiny shapes, edge cases); any out-of-bounds access, signed overflow or bad shift aborts it.
Host code only -- nothing here touches the GPU."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = tmp_path / "oracle_sanitize"
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=all", "-o", str(exe), os.path.join(ROOT, "oracle", "lotts_oracle.c"),
                    os.path.join(ROOT, "tests", "oracle_sanitize_main.c"), "-lm"], check=True)
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0")
    res = subprocess.run([str(exe)], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert res.returncode == 0, res.stdout[-4000:]
    assert "oracle sanitize driver: ok" in res.stdout
