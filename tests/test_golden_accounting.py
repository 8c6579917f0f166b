"""The byte accounting behind the benchmark's roofline, against the figures the paper fixes
(Abstract and Section 3.2: the LM head's cost is proportional to the rows kept; 32k of 128k
rows is its "75%" reduction), stored in tests/golden/lm_head_reduction.txt."""

import os
import re

from synth import CONFIGS

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "lm_head_reduction.txt")


def _golden():
    vals = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].split()
        if len(line) == 2:
            vals[line[0]] = float(line[1])
    return vals


def test_headline_config_is_the_papers_setting():
    g, c = _golden(), CONFIGS["llama3_8b"]
    assert (c.V, c.V_sub, c.d) == (int(g["V"]), int(g["V_sub"]), int(g["d"]))


def test_algorithmic_bytes_follow_the_papers_cost_model():
    # O(n d |V|) -> O(n d |V_high|): bf16 rows of d elements, each read once
    g, c = _golden(), CONFIGS["llama3_8b"]
    sub, full = c.V_sub * c.d * 2, c.V * c.d * 2
    assert sub == int(g["bytes_per_call_sub"]) and full == int(g["bytes_per_call_full"])
    kept = sub / full
    assert abs((1.0 - kept) - g["paper_reduction"]) < 0.01        # "75%", exactly 74.45%
    assert abs(full / sub - 3.914) < 5e-4                          # the latency ratio's ceiling


def test_bench_counts_the_same_bytes():
    # bench.py's algorithmic bytes per launch are V_sub * d * 2 of the same configuration
    src = open(os.path.join(os.path.dirname(GOLDEN), "..", "..", "bench.py")).read()
    assert re.search(r"bytes_per_call\s*=\s*V_sub\s*\*\s*d\s*\*\s*2", src)
    assert 'CONFIGS["llama3_8b"]' in src
