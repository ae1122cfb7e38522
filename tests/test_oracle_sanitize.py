"""The C oracle under the host AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): a small
C driver calls every oracle function on ragged shapes with exactly sized buffers; any access
outside a buffer or undefined integer operation ends it with a report."""
import os
import pathlib
import subprocess

ORACLE = pathlib.Path(__file__).resolve().parent.parent / "oracle"


def test_oracle_clean_under_host_sanitizers(tmp_path):
    exe = tmp_path / "oracle_sanitize"
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
                    "-o", str(exe), str(ORACLE / "sanitize_driver.c"), str(ORACLE / "w4a16_oracle.c")], check=True)
    env = dict(os.environ)
    # libraries preloaded by the environment would otherwise trip the link-order check; leak
    # detection needs ptrace, which containers often deny
    env["ASAN_OPTIONS"] = "verify_asan_link_order=0:detect_leaks=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["OMP_NUM_THREADS"] = "2"
    run = subprocess.run([str(exe)], env=env, capture_output=True, text=True, timeout=600)
    assert run.returncode == 0, run.stdout[-2000:] + run.stderr[-4000:]
    assert "oracle sanitizer run finished" in run.stdout
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr[-4000:]
