"""The CPU checker under AddressSanitizer and UndefinedBehaviorSanitizer (host code only).

tests/oracle_sanitize_main.c includes oracle/attn_oracle.c and calls every exported function on
small shapes with their edge cases.  Built twice, with and without the sanitisers: the sanitised
run must end clean, and both must print the same checksum."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "oracle_sanitize_main.c")
BASE = ["gcc", "-std=c11", "-O1", "-g", "-fopenmp", "-ffp-contract=off", "-Wall", "-Wextra"]


def _build_and_run(tmp_path, name, extra, env_extra):
    exe = os.path.join(str(tmp_path), name)
    subprocess.run(BASE + extra + ["-o", exe, SRC, "-lm"], check=True, capture_output=True, text=True)
    env = dict(os.environ, OMP_NUM_THREADS="4", **env_extra)
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    return r


def test_checker_is_clean_under_asan_and_ubsan(tmp_path):
    san = _build_and_run(tmp_path, "orc_san",
                         ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
                          "-static-libasan"],
                         {"ASAN_OPTIONS": "detect_leaks=1:abort_on_error=0", "UBSAN_OPTIONS": "print_stacktrace=1"})
    assert san.returncode == 0, san.stderr[-4000:]
    assert "runtime error" not in san.stderr and "AddressSanitizer" not in san.stderr, san.stderr[-4000:]
    plain = _build_and_run(tmp_path, "orc_plain", [], {})
    assert plain.returncode == 0, plain.stderr[-2000:]
    pick = lambda out: [l for l in out.splitlines() if l.startswith("checksum")]
    assert pick(san.stdout) and pick(san.stdout) == pick(plain.stdout)
