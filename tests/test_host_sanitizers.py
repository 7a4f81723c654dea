"""The argument-check paths of the C-ABI under AddressSanitizer and UndefinedBehaviorSanitizer (host code only: the
device code is the ordinary build, and nothing is launched)."""
import os
import subprocess

from paper_2409_12210_amd import build as modse_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_argument_checks_are_clean_under_address_and_ub_sanitizers(tmp_path):
    objs = [os.path.join(modse_build.CSRC, s.replace(".hip", ".o")) for s in modse_build.SOURCES]
    if not all(os.path.exists(o) for o in objs):
        modse_build.build(verbose=False)
    exe = modse_build.build_host_sanitized(str(tmp_path), os.path.join(ROOT, "tests", "host_abi_driver.c"))
    env = dict(os.environ)
    # (another preloaded library may come before the sanitizer's runtime on this machine; leaks of the HIP runtime's
    # own start-up allocations are not this library's)
    env["ASAN_OPTIONS"] = "verify_asan_link_order=0:detect_leaks=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    report = r.stdout + r.stderr
    assert "AddressSanitizer" not in report and "runtime error" not in report, report
    assert r.returncode == 0, report
    assert "all checks passed" in r.stdout
