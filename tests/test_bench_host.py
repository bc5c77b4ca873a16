"""Host-side pieces of bench.py (no GPU): the algorithmic byte counts and the rule that counter
traffic recorded under profiles/ is only quoted for the kernel sources it was measured on."""
import os
import re

import bench

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_algorithmic_bytes_of_the_headline_workload():
    # OLMo-1B 1/8 shard, chunk 64, k 32, R 4, bf16 gradients and parameters: 14 and 20 bytes per
    # parameter (gradient 2 + momentum read and written 8 + payload 4; 4 payloads of 4 + 2 + 2)
    n = 147_095_552
    ab = bench.algorithmic_bytes(n, 64, 32, 4, 2, 2, True)
    assert ab["compress"] == 14 * n and ab["decompress"] == 20 * n
    # Striding / Random ship values only: 12 and 12
    ab = bench.algorithmic_bytes(n, 64, 32, 4, 2, 2, False)
    assert ab["compress"] == 12 * n and ab["decompress"] == 12 * n
    # a ragged shard still ships k entries for its last chunk
    ab = bench.algorithmic_bytes(10_820_957, 32, 4, 2, 4, 4, True)
    assert ab["compress"] == 10_820_957 * 12 + 338_155 * 4 * 8


def test_recorded_traffic_belongs_to_the_current_kernel_sources():
    path = os.path.join(ROOT, "profiles", "traffic_olmo-1b-1of8_topk.txt")
    text = open(path).read()
    sha = re.search(r"^# kernel_sources_sha16 (\w+)$", text, re.M).group(1)
    assert re.search(r"^# commit \w+$", text, re.M)
    assert sha == bench.kernel_sources_sha16(), \
        "the HIP sources changed after the counters were measured: measure again or bench.py reports traffic = null"
    rows = dict(l.split() for l in text.splitlines() if l and not l.startswith("#"))
    n = 147_095_552
    # the counters agree with the algorithmic bytes to well under a per cent
    assert abs(float(rows["compress"]) / (14 * n) - 1) < 5e-3
    assert abs(float(rows["decompress"]) / (20 * n) - 1) < 5e-3
