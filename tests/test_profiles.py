"""The rocprofv3 summaries under profiles/ and the way bench.py reads them.

bench.py takes `traffic` (HBM-side bytes per launch) from the summary whose
recorded workload, variant and launch geometry match the run; these checks make
sure every committed summary parses, carries what bench.py needs, and that the
figure bench.py derives is the one the file's own rows give -- so a summary that
is edited or goes stale changes the bench line or fails here."""
import json
import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402

FILES = sorted(f for f in os.listdir(os.path.join(ROOT, "profiles")) if f.endswith(".txt"))


def test_there_are_summaries_for_the_headline_and_the_other_configurations():
    profs = bench.load_profiles()
    assert len(profs) == len(FILES), "a summary did not parse or two describe the same leg"
    for key in [("cfg5a", "chain"), ("cfg5a", "chain_wave_per_rank"), ("cfg5a", "direct"), ("cfg4", "chain"), ("cfg3", "chain"),
                ("cfg2", "chain"), ("cfg2", "reduce"), ("cfg4", "reduce"), ("cfg5b", "auto")]:
        assert key in profs, "no profile for %s:%s" % key


@pytest.mark.parametrize("name", FILES)
def test_summary_is_complete_and_consistent(name):
    prof = bench.parse_profile(os.path.join(ROOT, "profiles", name))
    assert prof is not None, "no '# leg:' line"
    leg = prof["leg"]
    for field in ("workload", "variant", "kernel", "geometry", "launches_per_step", "calibration_copy_bytes"):
        assert field in leg, field
    assert leg["workload"] in bench.WORKLOADS
    P, root, M, _, _ = bench.WORKLOADS[leg["workload"]]
    assert leg["calibration_copy_bytes"] == M // 4 * 4
    text = open(os.path.join(ROOT, "profiles", name)).read()
    assert "python3 bench.py --leg %s:%s" % (leg["workload"], leg["variant"]) in text, "the command that made it"
    assert leg["kernel"].split("::")[-1] in name and leg["workload"] in name, "named for its kernel and workload"
    t = bench.profile_traffic(prof)
    # the calibration copy reads and writes the message once: the counters' scale factors
    assert 1.9 < t["fetch_factor"] < 2.1 and 0.95 < t["write_factor"] < 1.05, t
    if M < (1 << 20):
        return  # a few KiB: the nominal factors were used, nothing more to cross-check
    # recompute from the rows by hand
    rows = prof["rows"]
    kern = [k for k in rows["FETCH_SIZE"] if leg["kernel"] in k]
    copy = [k for k in rows["FETCH_SIZE"] if "copyBuffer" in k]
    assert len(kern) == 1 and len(copy) == 1
    f = rows["FETCH_SIZE"][kern[0]]["avg_kib"] * (leg["calibration_copy_bytes"] / 1024.0) / rows["FETCH_SIZE"][copy[0]]["avg_kib"]
    w = rows["WRITE_SIZE"][kern[0]]["avg_kib"] * (leg["calibration_copy_bytes"] / 1024.0) / rows["WRITE_SIZE"][copy[0]]["avg_kib"]
    assert abs(t["bytes"] - (f + w) * 1024 * leg["launches_per_step"]) <= 1024 * leg["launches_per_step"]
    assert rows["stats"][[k for k in rows["stats"] if leg["kernel"] in k][0]]["calls"] >= 5
    g = leg["geometry"]
    if leg["variant"] == "reduce":
        # every contribution read once, the result written once, plus the staging round trip per stage boundary
        assert 0.95 * (P + (g["stages"] - 1)) * M <= t["fetch_bytes"] <= 1.1 * (P + (g["stages"] - 1)) * M, t
        assert 0.99 * M * g["stages"] <= t["write_bytes"] <= 1.05 * M * g["stages"], t
    elif M >= (1 << 20):
        # a broadcast writes every receiving rank's buffer exactly once and reads at least the message
        assert 0.99 * (P - 1) * M <= t["write_bytes"] <= 1.02 * (P - 1) * M, t
        assert 0.95 * M <= t["fetch_bytes"] <= 1.05 * (P - 1) * M, t
        if leg["variant"] in ("chain", "chain_wave_per_rank"):
            # the tuned chain and the wave-per-rank chain read the message from memory once per stage and no
            # more: hand-offs inside a stage stay on the compute unit (its cache, or LDS)
            assert t["fetch_bytes"] <= 1.12 * g["stages"] * M, (t, g["stages"])


def test_traffic_is_null_when_the_geometry_differs():
    profs = bench.load_profiles()
    prof = profs[("cfg5a", "chain")]
    same = json.loads(json.dumps(prof["leg"]["geometry"]))
    t, why = bench.traffic_for(profs, "cfg5a", "chain", same)
    assert t is not None and why is None and t["bytes"] > 0
    other = dict(same, lanes=same["lanes"] * 2)
    t, why = bench.traffic_for(profs, "cfg5a", "chain", other)
    assert t is None and "geometry" in why
    t, why = bench.traffic_for(profs, "cfg5a", "binomial", same)
    assert t is None and why == "no profile"
