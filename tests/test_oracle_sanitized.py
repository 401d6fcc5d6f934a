"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): a small C
driver calls every entry point on ragged, causal, grouped-head, rectangular and mirrored problems;
any report, or a non-zero return code, fails."""
import os
import subprocess
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
ORACLE = os.path.join(os.path.dirname(HERE), "oracle")


def test_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers():
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "oracle_san")
        subprocess.run(["gcc", "-std=c11", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                        "-fno-omit-frame-pointer", "-static-libasan", "-fopenmp", "-ffp-contract=off", "-mfma",
                        "-I", ORACLE, "-o", exe, os.path.join(HERE, "oracle_sanitizer_driver.c"),
                        os.path.join(ORACLE, "distr_attn_oracle.c"), os.path.join(ORACLE, "distr_attn_oracle_bwd.c"), "-lm"],
                       check=True)
        env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0")
        res = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert "ERROR: AddressSanitizer" not in res.stderr and "runtime error" not in res.stderr, res.stderr[-3000:]
    assert "LeakSanitizer" not in res.stderr or "detected memory leaks" not in res.stderr, res.stderr[-3000:]
    assert res.returncode == 0, res.stdout + res.stderr[-2000:]
    assert res.stdout.count("rc 0") == 6, res.stdout
