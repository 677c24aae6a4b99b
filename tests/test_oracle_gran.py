"""Pins for the oracle of the adaptive granularity search (Algorithm 1, Section III-C).

The paper prints no worked example, so the pins are: a trace worked by hand
(tests/golden/gran_trace.txt), the theorem that follows from the section's
monotonicity hypothesis (every answer equals the true best n, and a search is
needed exactly when B lies outside the span of the earlier searched batch sizes
with the same best n), the cache, and the stated reading for overlapping ranges.
"""
import os
import random

import pytest

from oracle.gran_oracle import GranularitySearch

HERE = os.path.dirname(os.path.abspath(__file__))


def step_fn(thresholds, values):
    def f(B):
        for t, v in zip(thresholds, values):
            if B < t:
                return v
        return values[-1]
    return f


def test_hand_worked_trace():
    f = step_fn([100, 1000], [1, 2, 4])
    g = GranularitySearch(f)
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "gran_trace.txt")) if l.strip() and not l.startswith("#")]
    assert len(rows) == 16
    for B, n, searched, S in rows:
        before = len(g.searches)
        assert g.get(int(B)) == int(n), B
        assert len(g.searches) - before == int(searched), B
        assert ",".join(f"{lo}-{up}:{m}" for lo, up, m in g.ranges()) == S, B


@pytest.mark.parametrize("seed", range(8))
def test_monotone_best_n_is_always_returned_and_searches_are_minimal(seed):
    rng = random.Random(seed)
    cuts = sorted(rng.sample(range(1, 5000), 3))
    f = step_fn(cuts, [1, 2, 4, 8])
    calls = []

    def search(B):
        calls.append(B)
        return f(B)

    g = GranularitySearch(search)
    asked = set()
    for _ in range(400):
        B = rng.randrange(1, 6000)
        # from the history alone: B needs a search iff it is new and outside the span of
        # the searched batch sizes whose best n is f(B)
        same = [b for b in calls if f(b) == f(B)]
        expect_search = B not in asked and not (same and min(same) <= B <= max(same))
        before = len(calls)
        assert g.get(B) == f(B)
        assert (len(calls) - before == 1) == expect_search
        asked.add(B)
    r = g.ranges()
    assert all(r[i][1] < r[i + 1][0] for i in range(len(r) - 1)), "ranges stay disjoint"
    assert [m for _, _, m in r] == sorted(m for _, _, m in r), "n grows with the range"
    assert len({m for _, _, m in r}) == len(r), "one range per n"


def test_cache_answers_without_find_or_search():
    state = {"n": 2}
    g = GranularitySearch(lambda B: state["n"])
    assert g.get(64) == 2
    state["n"] = 8                      # a new search would now say 8
    g.span_of.clear()                   # and no span would hold it
    assert g.get(64) == 2
    assert g.searches == [64]


def test_reading_for_overlapping_ranges():
    """When the hypothesis fails, ranges may overlap: the pair with the smallest lower bound wins."""
    table = {20: 1, 40: 1, 10: 2, 50: 2}
    g = GranularitySearch(lambda B: table[B])
    for B in (20, 40, 10):
        g.get(B)
    assert g.get(30) == 1 and g.searches == [20, 40, 10]      # inside 20-40, found
    g.get(50)                                                 # widens n=2 to 10-50, over 20-40
    assert g.ranges() == [(10, 50, 2), (20, 40, 1)]
    assert g.get(25) == 2
    assert g.get(30) == 1                                     # cached before the overlap arose
