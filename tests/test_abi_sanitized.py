"""The library's host-side argument validation under AddressSanitizer + UndefinedBehaviorSanitizer
(CPU only): a native driver calls every entry point with arguments that must be rejected before
anything is launched, plus the size queries and the host-side self test of the tile map."""
import os
import subprocess

from paper_2602_07899_amd import build as b


def test_validation_layer_is_clean_under_asan_ubsan():
    exe = b.build_sanitized_driver()
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300,
                       env=dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0"))
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "0 failed" in r.stdout and "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
    assert int(r.stdout.split()[0]) >= 120
