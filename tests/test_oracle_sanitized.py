"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: every exported function on
small ragged shapes (row subsets, odd populations, no history, both widths, the smallest tensor,
64-bit noise counters), in a program of its own so that the sanitizer runtime is linked in from the
start. Any report is fatal. The same program built with the oracle's ordinary flags, and the
sanitized one on a single thread, must print the same checksum of all outputs."""
import os
import subprocess


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    from oracle import build
    outs = []
    for sanitized, threads in ((True, 1), (True, 4), (False, 4)):
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
                   OMP_NUM_THREADS=str(threads))
        exe = build.build_driver(str(tmp_path), sanitized)
        r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
        assert r.returncode == 0, (sanitized, r.stderr[-4000:])
        assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr and "LeakSanitizer" not in r.stderr
        assert r.stdout.startswith("checksum ")
        outs.append(r.stdout.strip())
    # one thread or four, sanitized or plain: the same results (rows are independent, no shared writes)
    assert outs[0] == outs[1] == outs[2]
