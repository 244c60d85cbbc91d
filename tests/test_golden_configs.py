"""The paper-sized workloads carry the cluster counts the paper prints for its own method
(hyper-parameter table of the Appendix; fixture under tests/golden/), and the TopP values of that
table are valid arguments of the adaptive-budget rule -- CPU only."""
import os

import numpy as np

from oracle import svgear_oracle as orc
from workloads import get_workload

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "hyperparameters_svg_ear.txt")


def printed_rows():
    rows = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].split()
        if line:
            rows[(line[0], line[1])] = (int(line[2]), int(line[3]), float(line[4]))
    return rows


def test_paper_sized_workloads_use_the_printed_cluster_counts():
    rows = printed_rows()
    for name, key in (("wan_c300", ("wan2.2_a14b_720p", "full")), ("wan_turbo", ("wan2.2_a14b_720p", "turbo")),
                      ("hunyuan_c400", ("hunyuan_13b_720p", "full"))):
        wl = get_workload(name)
        assert (wl.Cq, wl.Ck) == rows[key][:2], name
    # the backbones' head counts and token grids are those of the headline workloads
    assert (get_workload("wan_c300").H, get_workload("wan_c300").N) == (get_workload("wan").H, get_workload("wan").N)
    assert get_workload("hunyuan_c400").N == get_workload("hunyuan").N


def test_printed_top_p_values_are_accepted_by_the_budget_rule():
    rng = np.random.default_rng(0)
    qbar, kbar = rng.standard_normal((4, 8)), rng.standard_normal((9, 8))
    q_sizes, k_sizes = rng.integers(1, 5, 4), rng.integers(1, 7, 9)
    full = q_sizes * k_sizes.sum()
    prev = None
    for p in sorted({v[2] for v in printed_rows().values()}):
        budgets, n_keep = orc.top_p_row_budgets(qbar, kbar, q_sizes, k_sizes, p, 0.3)
        assert np.all(n_keep >= 1) and np.all(budgets <= full)
        assert prev is None or np.all(budgets >= prev)
        prev = budgets
