"""The host half of the library under AddressSanitizer / UndefinedBehaviorSanitizer, on the CPU:
tests/host_checked_main.cpp (ABI error paths, a planner fuzz over group sizes 1..16, 1..8 kv-heads,
both head dims, work lists that need several launches and the forced-split fallback, small and
absent workspaces, slot pool and scheduler under random operations) linked with the host sources
and stand-ins for the kernel launchers that check every work list.  No GPU is touched."""
import subprocess

from paper_2509_25762_amd import build


def test_host_sources_are_clean_under_asan_and_ubsan():
    exe = build.build_host_checked(verbose=False)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "host checks passed" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
