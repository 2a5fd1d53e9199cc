"""Pins of the extended-solver oracle (Appendix B of the paper: importances
with end-activation flags, Algorithms 3 and 4) against things other than
itself: exhaustive enumeration of the extended objective, the reduction to
Algorithm 2 (already pinned) when identity activations are forbidden,
enumeration of the chains of Algorithm 3, invariants, and re-scoring of the
recovered sets from the raw tables."""
import itertools

import numpy as np
import pytest

import oracle
from helpers import DPC_INF, rand_tables, bits

NINF = np.float32(-np.inf)


def rand_i4(rng, L, kind="exact", ident_frac=0.4, paper_rules=True):
    """Flag-dependent importances.  kind 'exact': multiples of 1/8 (every sum is
    exact in binary32, so the order of the adds does not matter); 'float': any.
    paper_rules: the -inf pattern of the first lines of Algorithm 3 for a random
    set of positions whose original activation is an identity."""
    I4 = np.zeros((L + 1, L + 1, 2, 2), np.float32)
    for k in range(L + 1):
        for l in range(k + 1, L + 1):
            for a in range(2):
                for b in range(2):
                    if kind == "exact":
                        I4[k, l, a, b] = rng.integers(-24, 9) / 8.0
                    else:
                        I4[k, l, a, b] = rng.normal(-0.2, 0.5)
    if paper_rules:
        ident = rng.random(L + 1) < ident_frac          # sigma_x == id
        for k in range(L + 1):
            for l in range(k + 1, L + 1):
                if not ident[k]:
                    I4[k, l, 0, :] = NINF                # a kept activation cannot be dropped
                if not ident[l]:
                    I4[k, l, :, 0] = NINF
                if ident[k] and ident[l]:
                    I4[k, l, :, 0] = NINF                # blocks with identities at both ends
    return I4


@pytest.mark.parametrize("seed", range(8))
def test_extended_dp_equals_enumeration(seed):
    """Eq. (extended objective) by brute force: every A inside B, cheapest S
    containing A, free flags at both ends -- for every prefix l, budget t and
    final flag."""
    rng = np.random.default_rng(4000 + seed)
    L = int(rng.integers(2, 8))
    P = 40
    T, _ = rand_tables(rng, L, tmax=9, inf_frac=0.2 if seed % 2 else 0.0, ikind="int")
    I4 = rand_i4(rng, L, "exact", paper_rules=seed % 3 != 0)
    Topt, split = oracle.stage1(T)
    Iopt, bsplit = oracle.ext_iopt(I4)
    D, Kx = oracle.ext_dp(Topt, Iopt, P)
    for l in range(1, L + 1):
        want = oracle.brute_ext_objective(T, I4, l, P)
        assert (bits(D[l]) == bits(want)).all(), (seed, l)


@pytest.mark.parametrize("seed", range(6))
def test_reduces_to_algorithm_2_when_identities_are_forbidden(seed):
    """With flag 0 forbidden at every interior position, B = A and every block
    is a single block: the extended DP is Algorithm 2 on I[k][l] = I4[k][l][1][1]
    (any floats: the adds are the same, in the same order)."""
    rng = np.random.default_rng(4100 + seed)
    L = int(rng.integers(1, 14))
    P = 90
    T, I = rand_tables(rng, L, tmax=12, inf_frac=0.2, ikind="mixed")
    I4 = np.full((L + 1, L + 1, 2, 2), NINF, np.float32)
    for k in range(L + 1):
        for l in range(k + 1, L + 1):
            I4[k, l, 1, 1] = I[k, l]
            if k == 0:
                I4[k, l, 0, 1] = I[k, l]                 # the flag at the input is free
            if l == L:
                I4[k, l, 1, 0] = I[k, l]                 # ... and at the output
                if k == 0:
                    I4[k, l, 0, 0] = I[k, l]
    Topt, split = oracle.stage1(T)
    Iopt, bsplit = oracle.ext_iopt(I4)
    D, Kx = oracle.ext_dp(Topt, Iopt, P)
    M, K = oracle.stage2(Topt, I, P)
    assert (bits(D[L].max(axis=1)) == bits(M[L])).all()
    for l in range(1, L):
        assert (bits(D[l][:, 1]) == bits(M[l])).all(), l
        assert np.isneginf(D[l][:, 0]).all()
    for T0 in range(0, P, 7):
        r = oracle.ext_backtrack(Topt, split, bsplit, D, Kx, T0)
        r2 = oracle.backtrack(Topt, split, I, M, K, T0)
        assert r["status"] == r2["status"]
        if r["status"] == 0:
            assert list(r["A"]) == list(r2["A"]) == list(r["B"]) and list(r["S"]) == list(r2["S"])
            assert r["lat"] == r2["lat"] and bits(r["obj"]) == bits(r2["obj"])


@pytest.mark.parametrize("seed", range(5))
def test_iopt_is_the_best_chain_of_identity_points(seed):
    """Algorithm 3 by enumeration: I_opt[k,l,a,b] = max over subsets of the
    interior of (k, l) of the chain sum with flag 0 at every interior point."""
    rng = np.random.default_rng(4200 + seed)
    L = int(rng.integers(2, 9))
    I4 = rand_i4(rng, L, "exact", paper_rules=seed % 2 == 0)
    Iopt, bsplit = oracle.ext_iopt(I4)
    for k in range(L + 1):
        for l in range(k + 1, L + 1):
            inner = list(range(k + 1, l))
            for a, b in itertools.product(range(2), range(2)):
                best = NINF
                for r in range(len(inner) + 1):
                    for sub in itertools.combinations(inner, r):
                        nodes = [k, *sub, l]
                        acc = np.float32(0.0)
                        for x, y in zip(nodes[:-1], nodes[1:]):
                            acc = np.float32(acc + I4[x, y, a if x == k else 0, b if y == l else 0])
                        best = max(best, acc)
                assert bits(Iopt[k, l, a, b]) == bits(np.float32(best)), (k, l, a, b)
                assert Iopt[k, l, a, b] >= I4[k, l, a, b]
                # the recorded chain attains it
                nodes, x, flag = [l], l, b
                while True:
                    m = int(bsplit[k, x, a, flag])
                    if m == k:
                        break
                    assert k < m < x
                    nodes.append(m)
                    x, flag = m, 0
                nodes = [k] + nodes[::-1]
                acc = np.float32(0.0)
                for x, y in zip(nodes[:-1], nodes[1:]):
                    acc = np.float32(acc + I4[x, y, a if x == k else 0, b if y == l else 0])
                assert bits(acc) == bits(Iopt[k, l, a, b])


@pytest.mark.parametrize("seed", range(6))
def test_recovered_sets_rescore(seed):
    """A inside B, A inside S, the latency of S is the reported one and within
    budget, Proposition 4.2's decomposition over A holds, and the objective is
    the chain sum over B with the flags of A (exact importances)."""
    rng = np.random.default_rng(4300 + seed)
    L = int(rng.integers(3, 18))
    P = 120
    T, _ = rand_tables(rng, L, tmax=10, inf_frac=0.25, ikind="int", span=6)
    I4 = rand_i4(rng, L, "exact")
    Topt, split = oracle.stage1(T)
    Iopt, bsplit = oracle.ext_iopt(I4)
    D, Kx = oracle.ext_dp(Topt, Iopt, P)
    # monotone in the budget, unreachable exactly below the cheapest latency
    for l in range(1, L + 1):
        for a in range(2):
            col = D[l][:, a]
            fin = np.isfinite(col)
            if fin.any():
                first = int(np.argmax(fin))
                assert fin[first:].all() and (np.diff(col[first:]) >= 0).all()
                assert first >= Topt[0, l]
    for T0 in range(0, P, 5):
        r = oracle.ext_backtrack(Topt, split, bsplit, D, Kx, T0)
        if r["status"] != 0:
            assert np.isneginf(D[L][T0]).all()
            continue
        A, S, Bs = list(r["A"]), list(r["S"]), list(r["B"])
        assert set(A) <= set(Bs) and set(A) <= set(S)
        assert A == sorted(set(A)) and S == sorted(set(S)) and Bs == sorted(set(Bs))
        nodes = [0, *S, L]
        lat = sum(int(T[x, y]) for x, y in zip(nodes[:-1], nodes[1:]))
        assert lat == r["lat"] <= T0
        an = [0, *A, L]
        # (S may hold more points than A: the identity-flag steps of the DP)
        assert sum(int(Topt[x, y]) for x, y in zip(an[:-1], an[1:])) <= lat
        best = NINF
        for d0 in range(2):
            bn = [0, *Bs, L]
            acc = np.float32(0.0)
            for x, y in zip(bn[:-1], bn[1:]):
                fx = d0 if x == 0 else int(x in A)
                fy = r["a_last"] if y == L else int(y in A)
                acc = np.float32(acc + I4[x, y, fx, fy])
            best = max(best, acc)
        assert bits(np.float32(best)) == bits(r["obj"]) == bits(D[L][T0].max())
