"""The host side of the library (host scan of the missed clusters, prefetch and cache planners,
grouping of the consolidation moves) and the C oracle, built with the address + undefined-behaviour
sanitizers and, separately, the thread sanitizer, and run through a driver that checks the host
side against the oracle.  CPU only."""
import subprocess

from paper_2502_20969_amd.build import build_sanitized


def test_host_side_under_the_sanitizers():
    for exe in build_sanitized():
        r = subprocess.run([exe], capture_output=True, text=True, timeout=600)
        assert r.returncode == 0, f"{exe}:\n{r.stdout[-3000:]}\n{r.stderr[-3000:]}"
        assert "host sanitizer driver ok" in r.stdout
        assert "ERROR" not in r.stderr and "WARNING: ThreadSanitizer" not in r.stderr, r.stderr[-3000:]
