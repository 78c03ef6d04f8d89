"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: a standalone driver
(tests/sanitize/oracle_driver.cpp) includes the oracle's translation unit, calls every exported
function on small seeded inputs with exactly sized buffers (one token, budget = S, no
representatives, nothing important, units, protected ends with no middle, paged and strided
gathers, a decoding step) and must exit cleanly.  CPU only; nothing of the GPU library is involved."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = tmp_path / "oracle_driver"
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=all", "-ffp-contract=off", "-fno-fast-math", "-o", str(exe),
                    os.path.join(ROOT, "tests", "sanitize", "oracle_driver.cpp")], check=True)
    # (the harness preloads a library of its own; the sanitizer runtime only has to come first in the link order)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    run = subprocess.run([str(exe)], capture_output=True, text=True, env=env)
    assert run.returncode == 0, run.stdout[-2000:] + run.stderr[-4000:]
    assert run.stdout.strip().endswith("oracle sanitizer run ok")
