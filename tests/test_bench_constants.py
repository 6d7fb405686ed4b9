"""bench.py reports `roofline.traffic` from constants that were read off the committed counter summary; this
keeps the two from drifting apart (a counter run is not part of a bench run)."""
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_traffic_constants_are_the_committed_summary_s():
    src = open(os.path.join(ROOT, "bench.py")).read()
    name = re.search(r'TRAFFIC_SOURCE = "([^"]+)"', src).group(1)
    block = src[src.index("PROFILED_TRAFFIC = {"):]
    block = block[:block.index("}") + 1]
    consts = {k: float(v) for k, v in re.findall(r'"(\w+)": ([0-9.]+e6)', block)}
    assert consts, "no constants found in bench.py"
    text = open(os.path.join(ROOT, name)).read()
    line = [l for l in text.splitlines() if "PROFILED_TRAFFIC constants" in l]
    assert len(line) == 1
    summary = {k: float(v) for k, v in re.findall(r"(\w+) ([0-9.]+e6)", line[0])}
    for k, v in consts.items():
        assert k in summary, k
        assert abs(summary[k] - v) <= 0.002 * v, (k, v, summary[k])
