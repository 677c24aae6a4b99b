"""Host logic of the adaptive granularity search behind the C ABI (Algorithm 1, Section III-C)
against the oracle, query by query: same answers, same searches, same range set.  No GPU."""
import random

import pytest

from oracle.gran_oracle import GranularitySearch
from paper_2506_22175_amd import binding as B


def _drive_abi(g, f, Bq, searches):
    n = B.moe_gran_lookup(g, Bq)
    if n == -1:
        n = f(Bq)
        searches.append(Bq)
        B.moe_gran_record(g, Bq, n)
    return n


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("monotone", [True, False])
def test_same_answers_searches_and_ranges_as_the_oracle(seed, monotone):
    rng = random.Random(100 + seed)
    if monotone:
        cuts = sorted(rng.sample(range(1, 4000), 3))
        table = None

        def f(b):
            return [1, 2, 4, 8][sum(b >= c for c in cuts)]
    else:
        table = {b: rng.choice([1, 2, 4, 8]) for b in range(1, 300)}

        def f(b):
            return table[b]
    orc = GranularitySearch(f)
    g = B.GranHandle()
    searches = []
    hi = 5000 if monotone else 300
    for _ in range(500):
        q = rng.randrange(1, hi)
        assert _drive_abi(g, f, q, searches) == orc.get(q)
        assert searches == orc.searches
        assert B.moe_gran_ranges(g) == orc.ranges()
    g.close()


def test_error_codes_and_empty_handle():
    g = B.GranHandle()
    assert B.moe_gran_ranges(g) == []
    assert B.moe_gran_lookup(g, 77) == -1
    for bad in (0, -5):
        with pytest.raises(B.MoEError) as e:
            B.moe_gran_lookup(g, bad)
        assert e.value.status == 2
    with pytest.raises(B.MoEError) as e:
        B.moe_gran_record(g, 10, 0)
    assert e.value.status == 2
    B.moe_gran_record(g, 10, 4)
    assert B.moe_gran_lookup(g, 10) == 4 and B.moe_gran_ranges(g) == [(10, 10, 4)]
    g.close()
