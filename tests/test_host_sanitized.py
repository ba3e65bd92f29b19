"""The host side of the library under AddressSanitizer and UBSan, on the CPU: the attention planner (counts, the lists
of the host twin of the device builder), the workspace layouts, the split-K plane sizes and the validators, over the
five benchmark shapes and 4000 seeded random batches (csrc/host_check.cpp states the properties checked).  The host
arithmetic checked here is what turns into device addresses, so an off-by-one in it would be an out-of-bounds access
on the GPU."""
import os
import subprocess

from paper_2602_18447_amd import build as B


def test_host_planner_and_layouts_under_asan_ubsan():
    exe = B.HOST_CHECK
    srcs = [os.path.join(B.CSRC, f) for f in os.listdir(B.CSRC)]
    if not os.path.exists(exe) or os.path.getmtime(exe) < max(os.path.getmtime(f) for f in srcs):
        exe = B.build_host_check(verbose=False)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0, r.stdout[-4000:] + r.stderr[-4000:]
    assert "host_check: ok" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
