"""CPU oracle for the adaptive pipeline-granularity search (Algorithm 1, Section III-C).

TEST INFRASTRUCTURE ONLY.  Nothing on the product path may import this file.
It shares no code with the C++ implementation behind the C ABI.

What the algorithm does: it answers "into how many partitions n should a batch of
B tokens be cut" with as few timed searches as possible.  It remembers every
answer it has given, and for every n it has ever found it remembers the span of
batch sizes, from the smallest to the largest searched B, whose search gave that
n.  On the section's hypothesis that the best n never decreases as B grows, any B
inside such a span must have that same n, so only a B outside every span costs a
search.  Written here from that reading as three operations:

  lookup(B)     an answer given before for this B, else the n of a span that
                holds B, else nothing;
  search        the caller's search by timed trials, used only when lookup has
                nothing;
  record(B, n)  after a search: the span of n is created as [B, B] or stretched
                to hold B.

Readings where the paper's listing is ambiguous (also in the design notes):
  * after the search the listing looks the set up a second time; the section's
    prose makes that a lookup of the span that belongs to the n just found, and
    the stretched span has to be stored back;
  * spans can overlap only when the hypothesis fails; then, among the spans that
    hold B, the one with the smallest lower end answers (two spans cannot share
    a lower end: a span's lower end is a searched B whose answer is its n).

Spans are held in a dictionary keyed by n and scanned in full; the ordered tree
the paper suggests changes the speed, not the answers.
"""
from __future__ import annotations

from typing import Callable, Dict, List, Optional, Tuple


class GranularitySearch:
    def __init__(self, search_best_gran: Callable[[int], int]):
        self.search_best_gran = search_best_gran
        self.span_of: Dict[int, Tuple[int, int]] = {}    # n -> (smallest, largest) searched B that gave n
        self.answered: Dict[int, int] = {}               # B -> n, every answer given so far
        self.searches: List[int] = []                    # every B that needed a search, in order

    def lookup(self, B: int) -> Optional[int]:
        if B in self.answered:
            return self.answered[B]
        holding = [(lo, n) for n, (lo, hi) in self.span_of.items() if lo <= B <= hi]
        return min(holding)[1] if holding else None

    def record(self, B: int, n: int) -> None:
        lo, hi = self.span_of.get(n, (B, B))
        self.span_of[n] = (min(lo, B), max(hi, B))

    def get(self, B: int) -> int:
        n = self.lookup(B)
        if n is None:
            n = int(self.search_best_gran(B))
            self.searches.append(B)
            self.record(B, n)
        self.answered[B] = n
        return n

    def ranges(self) -> List[Tuple[int, int, int]]:
        """The spans ordered by lower end, as (lower, upper, n)."""
        return sorted((lo, hi, n) for n, (lo, hi) in self.span_of.items())
