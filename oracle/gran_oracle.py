"""CPU oracle for the adaptive pipeline-granularity search (Algorithm 1, Section III-C).

TEST INFRASTRUCTURE ONLY.  Nothing on the product path may import this file.
It shares no code with the C++ implementation behind the C ABI.

The algorithm decides the number of partitions n for a batch of B tokens with
as few timed searches as possible.  It keeps two pieces of global state:

  S            the set of pairs (R_n, n): one closed range R_n = [B_n^lower,
               B_n^upper] of batch sizes per value of n that has been found;
  cache_table  B -> n for every B that has been asked before.

Steps, in the paper's order:
  1. B in cache_table: return the cached n.
  2. find(S, B): the pair whose range contains B.  Found: that n is the answer
     (no search), by the hypothesis that the best n grows monotonically with B,
     which makes the ranges disjoint.
  3. Not found: n = searchBestGran(B), a search by timed trials.  Then the pair
     of *this n* is looked up in S; absent: insert (range(B, B), n); present:
     widen its range to [min(B, lower), max(B, upper)].
  4. cache_table[B] = n; return n.

Readings where the listing is ambiguous (also in the design notes):
  * the second find of the listing is a lookup by the n just found (the prose
    of Section III-C says "if n is not in S ... otherwise merge B into R_n"),
    and the widened range is written back into S;
  * find(S, B) over ranges that overlap (possible only when the monotonicity
    hypothesis fails): the pair with the smallest lower bound among those that
    contain B wins; ties on the lower bound cannot occur, because a pair's
    lower bound is a searched B whose n is that pair's n.

S is held here as a plain list scanned from the start; the paper's binary
search tree is a matter of speed, not of result.
"""
from __future__ import annotations

from typing import Callable, Dict, List, Tuple


class GranularitySearch:
    def __init__(self, search_best_gran: Callable[[int], int]):
        self.search_best_gran = search_best_gran
        self.S: List[Tuple[int, int, int]] = []          # (lower, upper, n)
        self.cache_table: Dict[int, int] = {}
        self.searches: List[int] = []                    # every B that needed a search, in order

    def find(self, B: int) -> int:
        """n of the pair whose range holds B, or -1."""
        best = None
        for lower, upper, n in self.S:
            if lower <= B <= upper and (best is None or lower < best[0]):
                best = (lower, n)
        return -1 if best is None else best[1]

    def ranges(self) -> List[Tuple[int, int, int]]:
        """The pairs of S ordered by lower bound, as (lower, upper, n)."""
        return sorted(self.S)

    def get(self, B: int) -> int:
        if B in self.cache_table:
            return self.cache_table[B]
        n = self.find(B)
        if n == -1:
            n = int(self.search_best_gran(B))
            self.searches.append(B)
            for i, (lower, upper, m) in enumerate(self.S):
                if m == n:
                    self.S[i] = (min(B, lower), max(B, upper), n)
                    break
            else:
                self.S.append((B, B, n))
        self.cache_table[B] = n
        return n
