"""AddressSanitizer + UndefinedBehaviorSanitizer over the host code: the oracle's C file and the
host side of the C ABI (descriptor validation, shape / workspace / plan queries, the launch
planners), driven by tests/san/san_driver.cpp.  Device code cannot be sanitised on this hardware
pool; its buffers are guarded by canaries in the GPU tests instead.  The first run compiles the
library a second time with the sanitizers on its host half (about a minute and a half)."""
import os
import subprocess


def test_oracle_and_abi_host_paths_under_asan_and_ubsan():
    from paper_2409_11902_amd import build
    exe = build.build_sanitized()
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "san ok" in r.stdout
    assert "AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-4000:]
