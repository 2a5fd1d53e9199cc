"""Pins of the sweep oracle (importance normalisation, trade-off curve, latency
of a network merged at a given set) against things other than itself: exact
rational arithmetic, hand cases with dyadic values, an enumeration of every
(A, S) pair written here, and a Python fold of the latency sum."""
import itertools
from fractions import Fraction

import numpy as np
import pytest

import oracle
from helpers import DPC_INF, chain_importance, chain_latency, rand_tables


def _all_pairs(L):
    """Every (A, S) with A inside S inside {1..L-1}."""
    for code in itertools.product((0, 1, 2), repeat=L - 1):
        S = [k + 1 for k, c in enumerate(code) if c >= 1]
        A = [k + 1 for k, c in enumerate(code) if c == 2]
        yield A, S


# ---------------- importance normalisation ----------------

def test_shift_hand_case_dyadic():
    """Mean of the size-one blocks is -0.5; alpha = 0.5 lowers every block by
    -0.25, i.e. raises it by 0.25 (the appendix subtracts alpha times the mean)."""
    L = 4
    I = np.zeros((L + 1, L + 1), np.float32)
    for i, v in enumerate([-0.5, -0.25, -0.75, -0.5]):
        I[i, i + 1] = v
    I[0, 2] = -1.0
    I[1, 4] = -np.inf
    out, mean = oracle.importance_shift(I, 0.5)
    assert mean == -0.5
    assert out[0, 2] == -0.75 and out[0, 1] == -0.25 and out[1, 2] == 0.0
    assert np.isneginf(out[1, 4])
    out0, _ = oracle.importance_shift(I, 0.0)
    assert np.array_equal(out0.view(np.uint32), I.view(np.uint32))


def test_shift_constant_table_cancels():
    L = 6
    I = np.full((L + 1, L + 1), -0.375, np.float32)
    out, mean = oracle.importance_shift(I, 1.0)
    assert mean == -0.375 and np.all(out == 0.0)
    out2, _ = oracle.importance_shift(I, 3.0)
    assert np.all(out2 == 0.75)


@pytest.mark.parametrize("flags", [False, True])
@pytest.mark.parametrize("seed", range(6))
def test_shift_matches_exact_rational_arithmetic(seed, flags):
    rng = np.random.default_rng(900 + seed)
    L = int(rng.integers(1, 20))
    shape = (L + 1, L + 1, 2, 2) if flags else (L + 1, L + 1)
    I = rng.normal(-0.3, 0.4, shape).astype(np.float32)
    # excluded blocks, some of them of size one: they must not enter the mean
    I[rng.random(shape) < 0.15] = -np.inf
    alpha = np.float32(rng.uniform(-1.0, 2.5))
    out, mean = oracle.importance_shift(I, alpha)
    D = [Fraction(float(v)) for i in range(L) for v in np.ravel(I[i, i + 1]) if np.isfinite(v)]
    exact_mean = sum(D) / len(D) if D else Fraction(0)
    assert abs(Fraction(mean) - exact_mean) <= abs(exact_mean) * Fraction(1, 2 ** 48)
    flat_in, flat_out = I.ravel(), out.ravel()
    for x in rng.choice(flat_in.size, size=min(flat_in.size, 200), replace=False):
        if not np.isfinite(flat_in[x]):
            assert np.isneginf(flat_out[x])
            continue
        exact = Fraction(float(flat_in[x])) - Fraction(float(alpha)) * exact_mean
        ulp = Fraction(float(np.spacing(np.float32(abs(float(exact))))))
        assert abs(Fraction(float(flat_out[x])) - exact) <= ulp * Fraction(501, 1000), x


def test_shift_reads_only_size_one_blocks():
    rng = np.random.default_rng(7)
    L = 9
    I = rng.normal(-0.3, 0.2, (L + 1, L + 1)).astype(np.float32)
    _, mean = oracle.importance_shift(I, 1.0)
    J = I.copy()
    for i in range(L + 1):
        for j in range(L + 1):
            if j != i + 1:
                J[i, j] = rng.normal()
    _, mean2 = oracle.importance_shift(J, 1.0)
    assert mean == mean2
    J[3, 4] += np.float32(1.0)
    _, mean3 = oracle.importance_shift(J, 1.0)
    assert abs((mean3 - mean) - 1.0 / L) < 1e-6


@pytest.mark.parametrize("seed", range(4))
def test_shift_changes_the_objective_by_blocks_times_shift(seed):
    """Every block of the chain 0 -> A -> L carries the shift once, so the
    optimum over (A, S) of the shifted table is max of obj(A) - (|A|+1) shift."""
    rng = np.random.default_rng(950 + seed)
    L = int(rng.integers(2, 7))
    T, I = rand_tables(rng, L, tmax=5, ikind="neg")
    for i in range(L):
        I[i, i + 1] = -abs(rng.normal(0.2, 0.1))
    alpha = np.float32(1.5)
    Is, mean = oracle.importance_shift(I, alpha)
    shift = float(alpha) * mean
    P = 5 * L + 2
    Topt, _ = oracle.stage1(T)
    M, _ = oracle.stage2(Topt, Is, P)
    best = np.full(P, -np.inf)
    for A, S in _all_pairs(L):
        lat = chain_latency(T, [0] + S + [L])
        if lat >= P:
            continue
        an = [0] + A + [L]
        obj = sum(float(I[a, b]) for a, b in zip(an[:-1], an[1:])) - (len(A) + 1) * shift
        best[lat:] = np.maximum(best[lat:], obj)
    fin = np.isfinite(best)
    assert np.array_equal(fin, np.isfinite(M[L]))
    assert np.allclose(M[L][fin], best[fin], rtol=0, atol=1e-5)


# ---------------- trade-off curve ----------------

def test_front_hand_case_and_cap():
    row = np.array([-np.inf, -np.inf, -1, -1, -0.5, -0.5, 0, 0], np.float32)
    t, o, n = oracle.front(row)
    assert n == 3 and list(t) == [2, 4, 6] and list(o) == [-1.0, -0.5, 0.0]
    t, o, n = oracle.front(row, cap=2)
    assert n == 3 and list(t) == [2, 4] and list(o) == [-1.0, -0.5]
    t, o, n = oracle.front(np.full(5, -np.inf, np.float32))
    assert n == 0 and len(t) == 0
    t, o, n = oracle.front(np.array([0.25], np.float32))
    assert n == 1 and list(t) == [0] and list(o) == [0.25]


@pytest.mark.parametrize("seed", range(8))
def test_front_equals_nondominated_pairs_of_the_enumeration(seed):
    """A point (t, o) is on the curve iff some (A, S) has latency exactly t and
    objective o, none with latency <= t does better, and none with latency < t
    does as well."""
    rng = np.random.default_rng(1000 + seed)
    L = int(rng.integers(2, 8))
    T, I = rand_tables(rng, L, tmax=6, inf_frac=0.2, ikind=("int", "mixed", "neg")[seed % 3])
    P = 6 * L + 3
    pts = []
    for A, S in _all_pairs(L):
        lat = chain_latency(T, [0] + S + [L])
        if lat < P:
            pts.append((lat, float(chain_importance(I, [0] + A + [L]))))
    expect = []
    for lat, obj in sorted(set(pts)):
        if any(l2 <= lat and o2 > obj for l2, o2 in pts):
            continue
        if any(l2 < lat and o2 >= obj for l2, o2 in pts):
            continue
        expect.append((lat, obj))
    Topt, _ = oracle.stage1(T)
    M, _ = oracle.stage2(Topt, I, P)
    t, o, n = oracle.front(M[L])
    assert n == len(expect)
    assert [(int(a), float(b)) for a, b in zip(t, o)] == expect


def test_front_queries_hand_case_and_concatenation():
    ft = np.array([[3, 7, 9, -1], [-1, -1, -1, -1], [0, 1, 2, 3], [5, -1, -1, -1]], np.int32)
    fl = np.array([3, 0, 6, 1], np.int32)               # instance 2 had 6 points, 4 were stored
    qi, qt, n = oracle.front_queries(ft, fl, 20)
    assert n == 8
    assert list(qi) == [0, 0, 0, 2, 2, 2, 2, 3] and list(qt) == [3, 7, 9, 0, 1, 2, 3, 5]
    qi, qt, n = oracle.front_queries(ft, fl, 5)
    assert n == 8 and list(qi) == [0, 0, 0, 2, 2] and list(qt) == [3, 7, 9, 0, 1]
    rng = np.random.default_rng(3)
    B, cap = 37, 11
    ft = rng.integers(0, 1000, (B, cap)).astype(np.int32)
    fl = rng.integers(0, 16, B).astype(np.int32)
    qi, qt, n = oracle.front_queries(ft, fl, 1000)
    keep = np.minimum(fl, cap)
    assert n == keep.sum()
    assert list(qi) == list(np.repeat(np.arange(B), keep))
    assert list(qt) == list(np.concatenate([ft[b, :keep[b]] for b in range(B)]))


# ---------------- latency of a network merged at a given set ----------------

def test_chain_latency_hand_cases():
    L = 4
    T = np.full((L + 1, L + 1), DPC_INF, np.int32)
    T[0, 4] = 50
    T[0, 2], T[2, 4] = 7, 9
    T[0, 1], T[1, 2], T[2, 3], T[3, 4] = 1, 2, 3, 4
    assert oracle.chain_latency(T, []) == 50
    assert oracle.chain_latency(T, [2]) == 16
    assert oracle.chain_latency(T, [1, 2, 3]) == 10
    assert oracle.chain_latency(T, [1]) == DPC_INF          # T[1][4] cannot be merged
    assert oracle.chain_latency(T, [1, 3]) == DPC_INF       # saturates, never wraps
    assert oracle.chain_latency(T, None) == -1


@pytest.mark.parametrize("seed", range(6))
def test_chain_latency_of_S_is_lat_and_of_A_is_no_smaller(seed):
    rng = np.random.default_rng(1100 + seed)
    L = int(rng.integers(2, 13))
    T, I = rand_tables(rng, L, tmax=6, inf_frac=0.15, ikind="mixed")
    P = 6 * L + 3
    Topt, split = oracle.stage1(T)
    M, K = oracle.stage2(Topt, I, P)
    for T0 in range(0, P, 3):
        r = oracle.backtrack(Topt, split, I, M, K, T0)
        if r["status"]:
            continue
        A, S = list(r["A"]), list(r["S"])
        assert oracle.chain_latency(T, S) == r["lat"] == chain_latency(T, [0] + S + [L])
        by_A = oracle.chain_latency(T, A)
        assert by_A == chain_latency(T, [0] + A + [L]) and by_A >= r["lat"]
