"""The committed rocprofv3 summaries describe the library as it is: each names the SHA-256 of the
library sources it was measured on (bench.py only takes the measured traffic from a summary whose
hash matches), and that hash is the one of the sources in the tree."""
import glob
import os
import re

import bench_profile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_profile_summaries_were_measured_on_these_sources():
    want = bench_profile.library_source_hash()
    files = sorted(glob.glob(os.path.join(ROOT, "profiles", "*.txt")))
    assert len(files) >= 5
    for path in files:
        with open(path) as f:
            m = re.search(r"sha256 = ([0-9a-f]{64})", f.read())
        assert m, f"{os.path.basename(path)} names no source hash"
        assert m.group(1) == want, f"{os.path.basename(path)} was measured on other library sources"
