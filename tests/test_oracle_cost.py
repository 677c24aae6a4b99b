"""Pins for the oracle of the reuse-strategy performance model (Section III-E, Eq. 7-10, Table II):
costs worked by hand, Table II's own structure, and properties the formula fixes."""
import os
import random

import pytest

from oracle import cost_oracle as C

HERE = os.path.dirname(os.path.abspath(__file__))
SPEEDS = dict(W_comp=1e10, W_comm=1e8, W_mem=5e7, sigma=1.0, mu_comp=0.8, mu_all=0.5, eta_all=0.5)


def test_hand_worked_costs():
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "cost_model_examples.txt"))
            if l.strip() and not l.startswith("#")]
    assert [r[0] for r in rows] == list(C.ORDER)
    for name, fw, bw in rows:
        got = C.strategy_cost(name, 1000, 400, 100, SPEEDS)
        assert got[0] * 1e3 == pytest.approx(float(fw), rel=1e-12)
        assert got[1] * 1e3 == pytest.approx(float(bw), rel=1e-12)
    assert C.select(C.ORDER, 1000, 400, 100, SPEEDS)[0] == "none"
    assert C.select(("S1", "S2", "S3", "S4"), 1000, 400, 100, SPEEDS) == ("S3", pytest.approx(0.028))
    assert C.select(("S4", "S2"), 1000, 400, 100, SPEEDS)[0] == "S4"


def test_table_two_is_consistent_with_what_each_strategy_restores():
    """Counts follow from the strategy: forward always has 2 GEMMs and 2 exchanges; backward has 4 GEMMs,
    +1 when T_M is recomputed; 2 exchanges, +1 when T_DI is sent again; copies: T_DI is one unit, T_M four
    (H = 4M), each way once."""
    for name, row in C.TABLE_II.items():
        copies = (1 if row["T_DI"] == "offload" else 0) + (4 if row["T_M"] == "offload" else 0)
        assert row["Q_fw"] == (2, 2, copies), name
        assert row["Q_bw"] == (4 + (row["T_M"] == "recompute"), 2 + (row["T_DI"] == "comm."), copies), name
        assert (row["eta"] is None) == (copies == 0)
        assert row["mu"] == ("mu_all" if copies else "mu_comp")


@pytest.mark.parametrize("seed", range(5))
def test_relative_form_equals_first_line_divided_by_one_gemm_unit(seed):
    rng = random.Random(seed)
    b, H, M = rng.randrange(64, 4096), rng.randrange(256, 8192), rng.randrange(64, 2048)
    Wc, Wm, Wx = 10 ** rng.uniform(9, 13), 10 ** rng.uniform(7, 10), 10 ** rng.uniform(7, 10)
    mu, eta = rng.uniform(0.3, 1.0), rng.uniform(0.3, 1.0)
    v = C.v0(b, H, M)
    unit = v[0] / Wc
    alpha, beta = (v[1] / Wm) / unit, (v[2] / Wx) / unit
    for Q in [(2, 2, 0), (4, 3, 4), (5, 2, 1), (2, 2, 5)]:
        assert C.cost(Q, v, Wc, Wm, Wx, 1.0, mu, eta) == pytest.approx(unit * C.cost_relative(Q, alpha, beta, mu, eta), rel=1e-12)


def test_properties_of_the_formula():
    # compute-bound regime: only q1 matters, recomputation costs exactly 5/4 in backward
    fast_io = dict(SPEEDS, W_comm=1e12, W_mem=1e12)
    none, s4 = C.strategy_cost("none", 512, 4096, 1024, fast_io), C.strategy_cost("S4", 512, 4096, 1024, fast_io)
    assert s4[0] == none[0] and s4[1] == pytest.approx(1.25 * none[1])
    # I/O-bound regime: the offloading strategies are the expensive ones, as the section says
    slow_mem = dict(SPEEDS, W_mem=1e5)
    costs = {n: sum(C.strategy_cost(n, 512, 4096, 1024, slow_mem)) for n in C.ORDER}
    assert costs["S1"] > costs["S2"] > costs["S3"] > costs["S4"] >= costs["none"]
    # "none" never loses to S4 (same streams, fewer operations)
    for seed in range(20):
        rng = random.Random(seed)
        sp = dict(W_comp=10 ** rng.uniform(9, 13), W_comm=10 ** rng.uniform(6, 11), W_mem=1e9, sigma=rng.uniform(0.5, 1),
                  mu_comp=rng.uniform(0.3, 1), mu_all=rng.uniform(0.3, 1), eta_all=rng.uniform(0.3, 1))
        a, b_ = C.strategy_cost("none", 777, 2048, 512, sp), C.strategy_cost("S4", 777, 2048, 512, sp)
        assert a[0] <= b_[0] and a[1] <= b_[1]
    # cost scales linearly with the micro-batch size
    x, y = C.strategy_cost("S2", 100, 2048, 512, SPEEDS), C.strategy_cost("S2", 300, 2048, 512, SPEEDS)
    assert y[0] == pytest.approx(3 * x[0]) and y[1] == pytest.approx(3 * x[1])
