"""The profiler-derived figures that bench.py reports (HBM traffic per launch, MFMA utilisation)
are typed into bench.PMC; this test keeps them equal to the rocprofv3 summaries under profiles/,
which carry them on lines of the form `bench.PMC[<leg>].<field> = <value>`."""
import glob
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_constants_are_the_ones_in_the_profile_summaries():
    files = glob.glob(os.path.join(ROOT, "profiles", "*.txt"))
    if not files:
        pytest.skip("profiles/ is not part of this copy of the tree")
    import bench
    found = {}
    for path in files:
        for leg, field, value in re.findall(r"bench\.PMC\[(\w+)\]\.(\w+) = ([0-9.]+)", open(path).read()):
            found[(leg, field)] = (float(value), os.path.basename(path))
    assert found, "no bench.PMC lines in profiles/"
    for leg, entry in bench.PMC.items():
        for field, value in entry.items():
            if field == "source":
                for name in value.split(", "):
                    assert os.path.exists(os.path.join(ROOT, name)), name
                continue
            assert (leg, field) in found, "bench.PMC[%s].%s has no line in profiles/" % (leg, field)
            assert value == pytest.approx(found[(leg, field)][0]), (leg, field, value, found[(leg, field)])
    for (leg, field) in found:
        assert leg in bench.PMC and field in bench.PMC[leg], "profiles/ carries %s.%s, bench.PMC does not" % (leg, field)
