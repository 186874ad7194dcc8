"""The memory-utilisation simulation reproduces the paper's closed-form waste of homogeneous
paging (Sec. 3.2: Gemma-2 up to 25 %, Ministral up to 56.25 %) and shows the two-level
allocator wasting next to nothing on the same traces (Sec. 7.3 reports 0.04 % on its traces)."""
import json
import os

import pytest

from paper_2503_18292_amd import memsim

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_examples.json")))


@pytest.mark.parametrize("model,key", [("gemma2_like", "gemma2_percent"), ("ministral_like", "ministral_percent")])
def test_static_trace_at_maximum_context(model, key):
    summary, rows = memsim.simulate(model, "static", n_requests=2, pool_gib=40.0)
    last = [r for r in rows if r["live"]][-1]      # every request close to the model's maximum context
    homogeneous = 100.0 * last["homogeneous_wasted"] / last["homogeneous_allocated"]
    assert abs(homogeneous - GOLD["window_waste"][key]) < 0.1
    assert 0 <= last["ours_wasted"] <= 0.001 * last["ours_allocated"]
    assert summary["peak_ours_bytes"] < summary["peak_homogeneous_bytes"]


def test_dynamic_trace_drains_and_wastes_little():
    summary, rows = memsim.simulate("ministral_like", "dynamic", n_requests=8, pool_gib=40.0, seed=3)
    assert summary["ours_waste_fraction"] < 0.01 < summary["homogeneous_waste_fraction"]
    assert rows[-1]["live"] == 0 and rows[-1]["ours_allocated"] == 0
    assert all(r["ours_wasted"] >= 0 for r in rows)
