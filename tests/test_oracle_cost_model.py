"""Pins for the oracle's analytical cost model (Section 3.2, the two cost tables)."""
from fractions import Fraction as Fr

import pytest

from oracle import cost_model as cm
from test_oracle_plan import golden


def base(**kw):
    p = dict(E=30_000_000, D=256, dtype_bytes=4, L=1000, W=8, N=4, B=4096, a2a_global=10**9, a2a_intra=8 * 10**9,
             ar_global=3 * 10**9, ar_cross=2 * 10**9, dp_multiplier=6)
    p.update(kw)
    return p


def test_activation_sizes_the_paper_prints():
    g = golden()
    # "local activation size": batch x average length x dimension x 4 bytes = the replicated strategy's
    # dynamic memory (the sharded strategies hold it twice: values plus communication buffer)
    for model, L in (("rm1", g["rm1_avg_length"]), ("rm3", g["rm3_avg_length"])):
        p = base(L=L, B=g["rm1_local_batch"], D=g["rm1_dim"])
        dp = cm.cost_model(p, cm.DP)[cm.DYNAMIC_MEMORY]
        assert round(float(dp) / 1e9, 2) == g[f"{model}_activation_gb"]
        for strat in (cm.RW, cm.CW, cm.FLEX):
            assert cm.cost_model(p, strat)[cm.DYNAMIC_MEMORY] == 2 * dp


def test_every_strategy_reads_the_same_rows():
    p = base()
    want = Fr(4096) * 1000 * 256
    assert all(cm.cost_model(p, s)[cm.ROWS_ACCESSED] == want for s in (cm.RW, cm.CW, cm.DP, cm.FLEX))
    # column-wise needs every id on every GPU; the replicated strategy needs none moved
    assert cm.cost_model(p, cm.CW)[cm.INPUT_DIST] == 32 * cm.cost_model(p, cm.RW)[cm.INPUT_DIST]
    assert cm.cost_model(p, cm.DP)[cm.INPUT_DIST] == 0


def test_static_memory_cells():
    p = base()
    row = 256 * 4
    assert cm.cost_model(p, cm.RW)[cm.STATIC_MEMORY] == Fr(30_000_000, 32) * row
    assert cm.cost_model(p, cm.CW)[cm.STATIC_MEMORY] == Fr(30_000_000, 32) * row
    assert cm.cost_model(p, cm.DP)[cm.STATIC_MEMORY] == 6 * 30_000_000 * row
    assert cm.cost_model(p, cm.FLEX)[cm.STATIC_MEMORY] == 6 * Fr(30_000_000, 8) * row


def test_break_even_probabilities_of_one_row():
    """E = 1, L = p (Section 4.2).  Memory: replicated = row-wise at p = (6 - 1/U) / B.  Traffic, with
    the all-to-all in both passes and the all-reduce in the backward pass only, and all-reduce three
    times as fast as all-to-all (the setting of the paper's cost-ratio figure): p = 1 / (6 B)."""
    U, B = 32, 4096
    p_mem = (6 - Fr(1, U)) / B
    one = base(E=1, L=p_mem)
    mem = lambda s: sum(cm.cost_model(one, s)[i] for i in (cm.STATIC_MEMORY, cm.DYNAMIC_MEMORY))
    assert mem(cm.DP) == mem(cm.RW)
    above = base(E=1, L=2 * p_mem)
    assert sum(cm.cost_model(above, cm.DP)[i] for i in (0, 3)) < sum(cm.cost_model(above, cm.RW)[i] for i in (0, 3))
    p_c = Fr(1, 6 * B)
    row = base(E=1, L=p_c)
    assert cm.cost_model(row, cm.DP)[cm.STATIC_COMM] == 2 * cm.cost_model(row, cm.RW)[cm.DYNAMIC_COMM]
    # Flex against row-wise, memory: dearer by (6/W - 1/U) rows whatever the probability
    for L in (p_c, p_mem, 5):
        r = base(E=1, L=L)
        assert mem_of(r, cm.FLEX) - mem_of(r, cm.RW) == (Fr(6, 8) - Fr(1, 32)) * 256 * 4


def mem_of(p, s):
    c = cm.cost_model(p, s)
    return c[cm.STATIC_MEMORY] + c[cm.DYNAMIC_MEMORY]


@pytest.mark.parametrize("model,tiers,pred_keys", [
    ("rm1", "2tier", ["rm1_2tier_dp_cov_pct"]), ("rm2", "3tier", ["rm2_3tier_dp_cov_pct", "rm2_3tier_flex_cov_pct"])])
def test_measured_all_to_all_reduction_matches_predicted_coverage(model, tiers, pred_keys):
    g = golden()
    before, after = g[f"{model}_a2a_rw_bytes"], g[f"{model}_a2a_{tiers}_bytes"]
    printed = g[f"{model}_a2a_{tiers}_reduction_pct"]
    assert round(100 * (1 - after / before), 1) == printed
    predicted = sum(g[k] for k in pred_keys)
    assert abs(predicted - printed) <= 2.0
    # the report from lookups per tier states the same thing: lookups outside the sharded tier never
    # enter the global all-to-all
    n = 1_000_000
    covered = int(round(predicted / 100 * n))
    rep = cm.tier_traffic([covered, 0, n - covered], 256, 1)
    assert rep[0] == n * 256 and rep[1] == (n - covered) * 256 and rep[2] == 0
    assert abs(float(rep[3]) * 100 - printed) <= 2.0
    rep3 = cm.tier_traffic([covered // 2, covered - covered // 2, n - covered], 256, 1)
    assert rep3[3] == rep[3] and rep3[2] == (covered - covered // 2) * 256
