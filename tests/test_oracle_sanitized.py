"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only, CPU).

oracle/san_check.c drives every exported function of oracle/lss_oracle.c on small seeded inputs with tight
heap buffers (ragged, single-row and empty segments, causal and not, dropout) and checks relations the
mathematics fixes on the way; built with -fsanitize=address,undefined any out-of-bounds access or undefined
operation in the oracle aborts it."""
import os
import subprocess

import oracle


def test_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers():
    exe = oracle.build_sanitized()
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300,
                       env={**os.environ, "ASAN_OPTIONS": "detect_leaks=1:abort_on_error=0", "OMP_NUM_THREADS": "4"})
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "san_check: clean" in r.stdout
