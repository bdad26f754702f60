"""The host side of the library under AddressSanitizer and UndefinedBehaviorSanitizer.

Needs `python -m paper_2509_03110_amd.build --host-sanitizers` first (three minutes of compiling,
which is why the test does not build it itself); skipped when that library is absent."""
import os
import subprocess
import sys

import pytest

from paper_2509_03110_amd import build


def test_host_paths_run_clean_under_asan_and_ubsan():
    runtime = build.asan_runtime()
    if not os.path.exists(build.SAN_LIB) or runtime is None:
        pytest.skip("no sanitized library: run `python -m paper_2509_03110_amd.build --host-sanitizers`")
    newest_source = max(os.path.getmtime(os.path.join(build.CSRC, f)) for f in os.listdir(build.CSRC))
    if os.path.getmtime(build.SAN_LIB) < newest_source:
        pytest.skip("the sanitized library is older than the sources: rebuild it")
    env = dict(os.environ)
    # the ASan runtime has to come first among the preloaded libraries; whatever is there stays
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["LD_LIBRARY_PATH"] = os.path.dirname(runtime) + ":" + env.get("LD_LIBRARY_PATH", "")
    env["ASAN_OPTIONS"] = "detect_leaks=0"        # the interpreter's own allocations are not ours to judge
    env["LSAM_LIB"] = build.SAN_LIB
    driver = os.path.join(os.path.dirname(os.path.abspath(__file__)), "host_paths_driver.py")
    r = subprocess.run([sys.executable, driver], env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "host paths clean" in r.stdout
