"""The counter figures that bench.py reports as `roofline.traffic` come from a tracked file keyed by the library version:
they must have been collected with the version that the header declares, for every workload the benchmark can time."""
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _header_version():
    text = open(os.path.join(ROOT, "include", "idlm.h")).read()
    return int(re.search(r"#define\s+IDLM_VERSION\s+(\d+)", text).group(1))


def test_traffic_file_matches_the_library_version():
    version = _header_version()
    rows = {}
    for line in open(os.path.join(ROOT, "profiles", "hbm_traffic_counters.txt")):
        if line.startswith("#") or not line.strip():
            continue
        workload, kernel, *fields = line.split()
        kv = dict(f.split("=", 1) for f in fields)
        assert int(kv["lib_version"]) == version, line
        assert int(kv["bytes"]) > 0
        assert os.path.exists(os.path.join(ROOT, kv["source"])), kv["source"]
        rows[(workload, kernel)] = int(kv["bytes"])
    for workload in ("serve256", "8b", "long32k_S1", "long32k_S8", "long32k_S16", "long32k_S32"):
        assert (workload, "attention") in rows and (workload, "row_stats") in rows, workload


def test_profile_summaries_name_their_commands():
    """Every summary under profiles/ states the command that made it, and that command runs committed files only."""
    for name in sorted(os.listdir(os.path.join(ROOT, "profiles"))):
        text = open(os.path.join(ROOT, "profiles", name)).read()
        assert "bench.py" in text, name
        assert "_work/" not in text and "gpurun" not in text.replace("gpurun_out", ""), name
