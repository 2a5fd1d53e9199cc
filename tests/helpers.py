"""Shared helpers for the tests: random tiny instances, re-scoring from the
raw tables, bit-level comparison.  No dynamic program here."""
import numpy as np

DPC_INF = 0x3FFFFFFF


def rand_tables(rng, L, tmax=9, inf_frac=0.0, ikind="mixed", span=None, tmin=1):
    """Tie-rich tiny tables.  ikind: 'int' small integer-valued importances
    (many exact ties), 'neg' non-positive floats, 'mixed' any sign floats."""
    T = np.zeros((L + 1, L + 1), np.int32)
    I = np.zeros((L + 1, L + 1), np.float32)
    for i in range(L + 1):
        for j in range(i + 1, L + 1):
            T[i, j] = rng.integers(tmin, tmax + 1)
            if span is not None and j - i > span:
                T[i, j] = DPC_INF
            elif j - i >= 2 and rng.random() < inf_frac:
                T[i, j] = DPC_INF
            if ikind == "int":
                I[i, j] = float(rng.integers(-3, 4))
            elif ikind == "neg":
                I[i, j] = 0.0 if j == i + 1 else -abs(rng.normal(0, 0.1)) * (j - i - 1)
            else:
                I[i, j] = rng.normal(0, 1.0)
    return T, I + np.float32(0.0)


def chain_latency(T, nodes):
    """Sum of T over consecutive members of `nodes` (saturating at INF)."""
    s = 0
    for a, b in zip(nodes[:-1], nodes[1:]):
        s += int(T[a, b])
        if s >= DPC_INF:
            return DPC_INF
    return s


def chain_importance(I, nodes):
    """binary32 left fold from +0 over consecutive members of `nodes`."""
    acc = np.float32(0.0)
    for a, b in zip(nodes[:-1], nodes[1:]):
        acc = np.float32(acc + I[a, b])
    return acc


def bits(x):
    return np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)


def assert_bits_equal(a, b, what=""):
    a = np.ascontiguousarray(a, dtype=np.float32)
    b = np.ascontiguousarray(b, dtype=np.float32)
    assert a.shape == b.shape, (what, a.shape, b.shape)
    bad = np.nonzero(bits(a) != bits(b))
    assert bad[0].size == 0, (what, "first mismatch at",
                             tuple(int(x[0]) for x in bad), a[bad][:4], b[bad][:4])
