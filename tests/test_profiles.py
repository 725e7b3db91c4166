"""Measured figures kept under profiles/ must describe the kernels in the tree."""
import json
import os

from paper_2310_16795_amd import build as lib_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_committed_traffic_figures_belong_to_the_present_kernel_sources():
    """bench.py reports roofline.traffic from profiles/traffic_<workload>.json (HBM bytes per launch from
    rocprofv3 --pmc); the file names the hash of the kernel sources it was measured with, and a change
    to those sources without a new measurement fails here (bench.py itself then reports traffic = null)."""
    found = 0
    for name in sorted(os.listdir(os.path.join(ROOT, "profiles"))):
        if not (name.startswith("traffic_") and name.endswith(".json")):
            continue
        with open(os.path.join(ROOT, "profiles", name)) as f:
            tj = json.load(f)
        assert tj["kernel_sources"] == lib_build.kernel_sources_hash(), f"{name} is stale: measure again"
        assert set(tj["bytes_per_launch"]) >= {"first_product_scalar", "second_product_scalar"}
        found += 1
    assert found >= 1
