"""The rocprofv3 summaries under profiles/ must describe the code as it is: every kernel of this
library that a summary names still exists in the kernel sources, every summary states the command
that produced it, and the traffic summaries carry the two fields bench.py reads (CPU only)."""
import glob
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2502_20566_amd", "csrc")


def kernels_in_sources():
    src = open(os.path.join(CSRC, "sr_kernels.h")).read()
    return set(re.findall(r"__global__[^;{]*?\bvoid\s+(\w+)\s*\(", src))


def test_profiles_name_only_existing_kernels_and_state_their_command():
    have = kernels_in_sources()
    assert {"adamw_kernel", "cast_kernel", "sumsq_partial_kernel"} <= have
    files = sorted(glob.glob(os.path.join(ROOT, "profiles", "*.txt")))
    assert files
    for f in files:
        text = open(f).read()
        assert "command" in text, f"{os.path.basename(f)} does not state the command that made it"
        for name in set(re.findall(r"\bsr::(\w+)\s*[<(]", text)):
            assert name in have, f"{os.path.basename(f)} names sr::{name}, which is not a kernel of csrc/sr_kernels.h"
        assert len(text) < 20000, f"{os.path.basename(f)} is not a short summary"


def test_traffic_summaries_carry_the_fields_bench_reads():
    import sys
    sys.path.insert(0, ROOT)
    import bench
    for f in glob.glob(os.path.join(ROOT, "profiles", "hbm_traffic_*.txt")):
        tag = os.path.basename(f)[len("hbm_traffic_"):-len(".txt")]
        text = open(f).read()
        assert re.search(r"^hbm_bytes_per_step = \d+$", text, re.M) and re.search(r"^kernel_source_sha16 = [0-9a-f]{16}$", text, re.M)
        traffic, source = bench.profile_traffic(tag)
        # fresh: a number and the file; stale (kernels edited since): None and a note that says so
        assert (traffic is not None and source.endswith(os.path.basename(f))) or (traffic is None and "stale" in source)
