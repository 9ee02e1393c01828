"""The rocprofv3 summaries under profiles/ name the kernel sources they were taken from (a digest of csrc/*.hip, *.hpp):
they must be those in the tree, so that the figures `bench.py` quotes from them (roofline.traffic) and the ones the
design notes cite belong to the kernels that are built.  Every summary also carries the full command that made it."""
import glob
import os
import re
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import profile_summary  # noqa: E402


def test_profile_summaries_belong_to_the_kernel_sources_in_the_tree():
    files = sorted(glob.glob(os.path.join(ROOT, "profiles", "*.txt")))
    assert len(files) >= 4
    want = profile_summary.kernel_sources_digest()
    for f in files:
        text = open(f).read()
        assert "rocprofv3" in text and "bench.py" in text, f      # the command line that produced it
        m = re.search(r"kernel sources \(sha256 of csrc/\*\.hip, \*\.hpp\): ([0-9a-f]{16})", text)
        assert m is not None, f
        assert m.group(1) == want, f"{os.path.basename(f)} was taken from other kernel sources: refresh profiles/"
