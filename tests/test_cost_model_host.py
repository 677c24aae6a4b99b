"""The reuse-strategy performance model behind the C ABI (Section III-E, Eq. 7-10, Table II)
against the oracle on random sizes and speeds.  Host arithmetic only, no GPU."""
import random

import pytest

from oracle import cost_oracle as C
from paper_2506_22175_amd import binding as B


def _speeds(rng):
    d = dict(W_comp=10 ** rng.uniform(9, 14), W_comm=10 ** rng.uniform(6, 12), W_mem=10 ** rng.uniform(6, 11),
             sigma=rng.uniform(0.5, 1.0), mu_comp=rng.uniform(0.3, 1.0), mu_all=rng.uniform(0.3, 1.0),
             eta_all=rng.uniform(0.3, 1.0))
    return d, B.MoESpeeds(d["W_comp"], d["W_comm"], d["W_mem"], d["sigma"], d["mu_comp"], d["mu_all"], d["eta_all"])


@pytest.mark.parametrize("seed", range(10))
def test_costs_and_choice_equal_the_oracle(seed):
    rng = random.Random(seed)
    for _ in range(50):
        d, s = _speeds(rng)
        b, M, H = rng.randrange(1, 70000), rng.randrange(8, 4096), rng.randrange(8, 16384)
        for i, name in enumerate(C.ORDER):
            fw, bw = B.moe_strategy_cost(i, b, M, H, s)
            ofw, obw = C.strategy_cost(name, b, H, M, d)
            assert fw == pytest.approx(ofw, rel=1e-12) and bw == pytest.approx(obw, rel=1e-12)
        mask = rng.randrange(1, 32)
        allowed = [n for i, n in enumerate(C.ORDER) if (mask >> i) & 1]
        best, cost = B.moe_select_strategy(mask, b, M, H, s)
        oname, ocost = C.select(allowed, b, H, M, d)
        assert C.ORDER[best] == oname and cost == pytest.approx(ocost, rel=1e-12)


def test_errors():
    _, s = _speeds(random.Random(0))
    for args in ((5, 10, 10, 10), (-1, 10, 10, 10), (0, 0, 10, 10), (0, 10, 0, 10), (0, 10, 10, 0)):
        with pytest.raises(B.MoEError) as e:
            B.moe_strategy_cost(*args, s)
        assert e.value.status == 2
    with pytest.raises(B.MoEError) as e:
        B.moe_select_strategy(0, 10, 10, 10, s)
    assert e.value.status == 2
    bad = B.MoESpeeds(1e9, 0.0, 1e9, 1, 1, 1, 1)
    with pytest.raises(B.MoEError):
        B.moe_strategy_cost(0, 10, 10, 10, bad)
