"""Checker written from the paper's definitions, for tiny inputs (pure Python).

Not the algorithms' loops: the definitions they implement, with the paper's
own conventions, which differ from the oracle's on purpose (strict budgets
"latency < t", whole ordered sets instead of back-pointers).

  * Eq. 5a/5b by their definition: the minimum, over every subset S of the
    layers strictly between k and l, of the summed block latencies along
    k -> S -> l (sums saturate at "not mergeable").
  * Eq. 6 by recursion on its own sub-problem: the best (A, S) for the first l
    layers under "latency < t" ends with a last kept activation k (Eq. 7a-c):
    its value is the value of the sub-problem (k, t - T_opt[k,l]) plus I[k,l],
    its A that sub-problem's A plus k, its S that sub-problem's S plus k plus
    the best boundaries inside (k, l).  Memoised; a sub-problem that no (A, S)
    satisfies has no value.

The tests check the oracle against it through the identity
D_paper(l, t) == M_oracle[l][t-1] and the equality of the sets (ties: the
lowest last activation, and inside a block the lowest last boundary).
"""
from functools import lru_cache
from itertools import combinations

import numpy as np

INF = 0x3FFFFFFF


def block_latency_by_definition(T, k, l):
    """Eq. 5a: min over S inside {k+1..l-1} of the summed T along k -> S -> l.
    -> (latency, the set of all minimisers as sorted tuples)."""
    inner = range(k + 1, l)
    best, argbest = None, []
    for n in range(len(inner) + 1):
        for S in combinations(inner, n):
            chain = (k,) + S + (l,)
            lat = 0
            for a, b in zip(chain, chain[1:]):
                lat = min(lat + int(T[a][b]), INF)
            if best is None or lat < best:
                best, argbest = lat, [S]
            elif lat == best:
                argbest.append(S)
    return best, argbest


class SubProblems:
    """Eq. 6 for one instance, every (l, t) on demand."""

    def __init__(self, L, T, I):
        self.L, self.T, self.I = L, T, I
        self.topt = lru_cache(maxsize=None)(self._topt)
        self.solve = lru_cache(maxsize=None)(self._solve)

    def _topt(self, k, l):
        """(T_opt[k,l], S_opt[k,l]): Eq. 5 through its last merged block (m, l);
        the lowest m among equally good ones, no boundary when m == k."""
        if k == l:
            return 0, ()
        best, arg = None, None
        for m in range(k, l):
            c = min(self.topt(k, m)[0] + int(self.T[m][l]), INF)
            if best is None or c < best:
                best, arg = c, m
        if arg == k or best >= INF:
            return best, ()
        return best, self.topt(k, arg)[1] + (arg,)

    def _solve(self, l, t):
        """Best (value, A, S) of Eq. 6 for the first l layers with latency < t, or None."""
        if l == 0:
            return (np.float32(0.0), (), ()) if t > 0 else None
        best = None
        for k in range(l):
            tkl = self.topt(k, l)[0]
            if tkl >= INF or t - tkl <= 0:
                continue
            sub = self.solve(k, t - tkl)          # exists iff T_opt[0,k] < t - T_opt[k,l]
            if sub is None:
                continue
            value = np.float32(sub[0] + np.float32(self.I[k][l]))
            if best is None or value > best[0]:
                keep = (k,) if k > 0 else ()
                best = (value, sub[1] + keep, tuple(sorted(sub[2] + keep + self.topt(k, l)[1])))
        return best
