"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only, no GPU).

tests/oracle_sanitize_main.c calls every oracle entry point on small seeded inputs with exactly-sized
heap buffers; built together with oracle/mage_oracle.c under -fsanitize=address,undefined, an
out-of-bounds access or undefined arithmetic anywhere in the oracle aborts the run."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def test_oracle_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    subprocess.run(["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    "-o", exe, os.path.join(HERE, "oracle_sanitize_main.c"), os.path.join(ROOT, "oracle", "mage_oracle.c"),
                    "-lm"], check=True)
    env = dict(os.environ)
    env.pop("LD_PRELOAD", None)                      # the sanitizer runtime must be the first library loaded
    env["ASAN_OPTIONS"] = "detect_leaks=1:verify_asan_link_order=0"
    env["OMP_NUM_THREADS"] = "4"
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0 and r.stdout.strip().endswith("OK"), (r.stdout[-2000:], r.stderr[-4000:])
