"""The synthetic workloads and the schedule defaults follow the numbers the paper prints (tests/golden)."""
import os

import numpy as np

from oracle import loqt_oracle as O
from paper_2405_16528_amd import synth

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [line.split() for line in f if line.strip() and not line.startswith("#")]


def test_workload_shapes_follow_the_papers_table():
    table = {m: (int(h), int(f), int(r)) for (m, h, f, r) in _rows("llama_shapes.txt")}
    names = {"60m_layer": "60M", "130m_block": "130M", "1b_block": "1B", "7b_block": "7B", "13b_block": "13B"}
    for wl_name, model in names.items():
        wl = synth.WORKLOADS[wl_name]
        hidden, ffn, rank = table[model]
        shapes = {(o, i) for (_, o, i) in wl.projections}
        if wl_name == "60m_layer":
            assert shapes == {(hidden, hidden)}          # one attention projection of the smallest model
        else:
            assert shapes == {(hidden, hidden), (ffn, hidden), (hidden, ffn)}
            assert len(wl.projections) == 7               # q, k, v, o, gate, up, down
        # the 13B workload uses the rank of the paper's introduction (1024), not the table's 1536
        assert wl.r == (1024 if model == "13B" else rank)


def test_schedule_defaults_are_the_papers_constants():
    (tau, psi, cap), = [(float(a), float(b), int(c)) for (a, b, c) in _rows("update_schedule.txt")]
    steps = O.merge_schedule(tau, psi, cap, 80)
    gaps = np.diff([0] + list(steps))
    assert gaps[0] == 101                                  # 100 + 1.2^0
    assert np.all(gaps >= tau) and np.all(gaps <= cap)
    assert np.all(np.diff(gaps) >= 0)                      # the intervals never shrink
    assert gaps[-1] == cap and gaps[40] < cap              # ... and reach the cap (1.2^i passes 2400 at i = 43)
    # the library's defaults are these constants
    from paper_2405_16528_amd import binding as L
    assert L.loqt_merge_schedule(80) == list(steps)
