"""The library's host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): tests/sanitize_driver.cpp
walks the host-only entry points (stage schedule, stored-depth schedule, sampler weights, pooled extents), every
workspace-size function (the carving arithmetic) and the argument validation of the device entry points; the device
code is compiled as usual and never runs. A sanitizer finding aborts the driver with a report."""
import os
import subprocess

from paper_2604_04451_amd import build as b

HERE = os.path.dirname(os.path.abspath(__file__))


def test_host_code_is_clean_under_asan_and_ubsan():
    exe = b.build_sanitized_driver(os.path.join(HERE, "sanitize_driver.cpp"))
    # a preloaded library may come before the sanitizer runtime in the link order; leak checking needs ptrace
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=0:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, f"rc={r.returncode}\n{r.stdout[-2000:]}\n{r.stderr[-6000:]}"
    assert "sanitize_driver: ok" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-6000:]
