"""ctypes front end of the C oracle.  numpy in, numpy out; no arithmetic of
the method lives here (only marshalling and a thread pool over instances)."""
import ctypes
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from . import build as _build

DPC_INF = 0x3FFFFFFF
DPC_NOARG = 0xFF

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        lib = ctypes.CDLL(path)
        i32, vp = ctypes.c_int32, ctypes.c_void_p
        lib.oracle_stage1.argtypes = [i32, vp, vp, vp]
        lib.oracle_stage1.restype = None
        lib.oracle_relax_row.argtypes = [i32, i32, i32, vp, vp, vp, vp]
        lib.oracle_relax_row.restype = None
        lib.oracle_stage2.argtypes = [i32, i32, vp, vp, vp, vp]
        lib.oracle_stage2.restype = None
        lib.oracle_backtrack.argtypes = [i32, i32, vp, vp, vp, vp, vp, i32,
                                         vp, vp, vp, vp, vp, vp]
        lib.oracle_backtrack.restype = i32
        lib.brute_topt.argtypes = [i32, vp, i32, i32]
        lib.brute_topt.restype = i32
        lib.brute_objective.argtypes = [i32, vp, vp, i32, i32, vp]
        lib.brute_objective.restype = None
        lib.brute_min_latency_given_A.argtypes = [i32, vp, i32, ctypes.c_uint32]
        lib.brute_min_latency_given_A.restype = i32
        _lib = lib
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None else None


def _chk(a, dtype, shape):
    assert a.dtype == dtype and a.shape == shape and a.flags.c_contiguous, (
        a.dtype, a.shape, dtype, shape)
    return a


def stage1(T):
    """T int32 [L+1][L+1] -> (Topt int32 [L+1][L+1], split uint8 [L+1][L+1])."""
    L = T.shape[0] - 1
    _chk(T, np.int32, (L + 1, L + 1))
    Topt = np.empty((L + 1, L + 1), np.int32)
    split = np.empty((L + 1, L + 1), np.uint8)
    _load().oracle_stage1(L, _p(T), _p(Topt), _p(split))
    return Topt, split


def stage2(Topt, I, P, want_K=True):
    """-> (M float32 [L+1][P], K uint8 [L+1][P] or None)."""
    L = Topt.shape[0] - 1
    _chk(Topt, np.int32, (L + 1, L + 1))
    _chk(I, np.float32, (L + 1, L + 1))
    M = np.empty((L + 1, P), np.float32)
    K = np.empty((L + 1, P), np.uint8) if want_K else None
    _load().oracle_stage2(L, P, _p(Topt), _p(I), _p(M), _p(K))
    return M, K


def relax_row(j, Topt, I, M, K=None):
    """Fill row j of M (and K) in place from rows < j."""
    L = Topt.shape[0] - 1
    P = M.shape[1]
    _chk(Topt, np.int32, (L + 1, L + 1))
    _chk(I, np.float32, (L + 1, L + 1))
    _chk(M, np.float32, (L + 1, P))
    if K is not None:
        _chk(K, np.uint8, (L + 1, P))
    _load().oracle_relax_row(L, P, j, _p(Topt), _p(I), _p(M), _p(K))


def backtrack(Topt, split, I, M, K, T0):
    """-> dict(status, A, S, obj, lat).  K may be None (arg-max recomputed)."""
    L = Topt.shape[0] - 1
    P = M.shape[1]
    assert 0 <= T0 < P
    _chk(Topt, np.int32, (L + 1, L + 1))
    _chk(split, np.uint8, (L + 1, L + 1))
    _chk(I, np.float32, (L + 1, L + 1))
    _chk(M, np.float32, (L + 1, P))
    if K is not None:
        _chk(K, np.uint8, (L + 1, P))
    A = np.full(L, -1, np.int32)
    S = np.full(L, -1, np.int32)
    na, ns, lat = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    obj = ctypes.c_float()
    st = _load().oracle_backtrack(
        L, P, _p(Topt), _p(split), _p(I), _p(M), _p(K), int(T0), _p(A),
        ctypes.byref(na), _p(S), ctypes.byref(ns), ctypes.byref(obj),
        ctypes.byref(lat))
    return dict(status=st, A=A[:max(na.value, 0)].copy(),
                S=S[:max(ns.value, 0)].copy(), A_len=na.value, S_len=ns.value,
                obj=np.float32(obj.value), lat=lat.value)


def _solve_one(args):
    T, I, P, want_K = args
    Topt, split = stage1(T)
    M, K = stage2(Topt, I, P, want_K)
    return Topt, split, M, K


def solve_batch(T, I, P, want_K=True, threads=1):
    """Stages 1 and 2 for a batch.  T int32 [B][L+1][L+1], I float32 likewise.
    One instance per task on `threads` host threads (the C calls release the
    GIL).  -> Topt [B][L+1][L+1], split, M [B][L+1][P], K."""
    B = T.shape[0]
    jobs = [(np.ascontiguousarray(T[b]), np.ascontiguousarray(I[b]), P, want_K)
            for b in range(B)]
    if threads <= 1:
        res = [_solve_one(j) for j in jobs]
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            res = list(ex.map(_solve_one, jobs))
    Topt = np.stack([r[0] for r in res])
    split = np.stack([r[1] for r in res])
    M = np.stack([r[2] for r in res])
    K = np.stack([r[3] for r in res]) if want_K else None
    return Topt, split, M, K


def brute_topt(T, k, l):
    ld = T.shape[1]
    assert T.dtype == np.int32 and T.flags.c_contiguous and l - k - 1 <= 20
    return _load().brute_topt(ld, _p(T), k, l)


def brute_objective(T, I, l, P):
    """Exhaustive M[l][0..P) for the first l layers (l - 1 <= 15)."""
    ld = T.shape[1]
    assert T.dtype == np.int32 and I.dtype == np.float32
    assert T.flags.c_contiguous and I.flags.c_contiguous and 1 <= l <= 16
    out = np.empty(P, np.float32)
    _load().brute_objective(ld, _p(T), _p(I), l, P, _p(out))
    return out


def brute_min_latency_given_A(T, l, A):
    ld = T.shape[1]
    amask = 0
    for a in A:
        assert 1 <= a <= l - 1
        amask |= 1 << (int(a) - 1)
    assert l - 1 <= 20
    return _load().brute_min_latency_given_A(ld, _p(T), l, amask)


# ---- extended solver (Appendix B of the paper: Algorithms 3 and 4) ----

def _load_ext():
    lib = _load()
    if not getattr(lib, "_ext_ready", False):
        i32, vp = ctypes.c_int32, ctypes.c_void_p
        lib.oracle_ext_iopt.argtypes = [i32, vp, vp, vp]
        lib.oracle_ext_iopt.restype = None
        lib.oracle_ext_dp.argtypes = [i32, i32, vp, vp, vp, vp]
        lib.oracle_ext_dp.restype = None
        lib.oracle_ext_backtrack.argtypes = [i32, i32, vp, vp, vp, vp, vp, i32] + [vp] * 9
        lib.oracle_ext_backtrack.restype = i32
        lib.brute_ext_objective.argtypes = [i32, vp, vp, i32, i32, vp]
        lib.brute_ext_objective.restype = None
        lib._ext_ready = True
    return lib


def ext_iopt(I4):
    """I4 float32 [L+1][L+1][2][2] -> (Iopt, bsplit uint8), same shape."""
    L = I4.shape[0] - 1
    _chk(I4, np.float32, (L + 1, L + 1, 2, 2))
    Iopt = np.empty_like(I4)
    bsplit = np.empty(I4.shape, np.uint8)
    _load_ext().oracle_ext_iopt(L, _p(I4), _p(Iopt), _p(bsplit))
    return Iopt, bsplit


def ext_dp(Topt, Iopt, P):
    """-> (D float32 [L+1][P][2], Kx uint8 [L+1][P][2])."""
    L = Topt.shape[0] - 1
    _chk(Topt, np.int32, (L + 1, L + 1))
    _chk(Iopt, np.float32, (L + 1, L + 1, 2, 2))
    D = np.empty((L + 1, P, 2), np.float32)
    Kx = np.empty((L + 1, P, 2), np.uint8)
    _load_ext().oracle_ext_dp(L, P, _p(Topt), _p(Iopt), _p(D), _p(Kx))
    return D, Kx


def ext_backtrack(Topt, split, bsplit, D, Kx, T0):
    """-> dict(status, A, S, B, obj, lat, a_last)."""
    L = Topt.shape[0] - 1
    P = D.shape[1]
    assert 0 <= T0 < P
    _chk(split, np.uint8, (L + 1, L + 1))
    _chk(bsplit, np.uint8, (L + 1, L + 1, 2, 2))
    _chk(D, np.float32, (L + 1, P, 2))
    _chk(Kx, np.uint8, (L + 1, P, 2))
    A, S, Bs = (np.full(L, -1, np.int32) for _ in range(3))
    na, ns, nb, lat, al = (ctypes.c_int32() for _ in range(5))
    obj = ctypes.c_float()
    st = _load_ext().oracle_ext_backtrack(
        L, P, _p(Topt), _p(split), _p(bsplit), _p(D), _p(Kx), int(T0), _p(A),
        ctypes.byref(na), _p(S), ctypes.byref(ns), _p(Bs), ctypes.byref(nb),
        ctypes.byref(obj), ctypes.byref(lat), ctypes.byref(al))
    return dict(status=st, A=A[:max(na.value, 0)].copy(), S=S[:max(ns.value, 0)].copy(),
                B=Bs[:max(nb.value, 0)].copy(), A_len=na.value, S_len=ns.value,
                B_len=nb.value, obj=np.float32(obj.value), lat=lat.value, a_last=al.value)


def _ext_solve_one(args):
    T, I4, P = args
    Topt, split = stage1(T)
    Iopt, bsplit = ext_iopt(I4)
    D, Kx = ext_dp(Topt, Iopt, P)
    return Topt, split, Iopt, bsplit, D, Kx


def ext_solve_batch(T, I4, P, threads=1):
    """Algorithms 1, 3 and 4 for a batch.  -> Topt, split, Iopt, bsplit, D, Kx
    (leading batch dimension)."""
    jobs = [(np.ascontiguousarray(T[b]), np.ascontiguousarray(I4[b]), P)
            for b in range(T.shape[0])]
    if threads <= 1:
        res = [_ext_solve_one(j) for j in jobs]
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            res = list(ex.map(_ext_solve_one, jobs))
    return tuple(np.stack([r[x] for r in res]) for x in range(6))


def brute_ext_objective(T, I4, l, P):
    """Exhaustive D[l][0..P)[0..1] for the first l layers (l - 1 <= 9)."""
    ld = T.shape[1]
    assert T.dtype == np.int32 and I4.dtype == np.float32
    assert T.flags.c_contiguous and I4.flags.c_contiguous and 1 <= l <= 10
    out = np.empty((P, 2), np.float32)
    _load_ext().brute_ext_objective(ld, _p(T), _p(I4), l, P, _p(out))
    return out


# ---- steps around the solver in a sweep (importance normalisation, trade-off
#      curve, latency of a network merged at a given set) ----

def _load_sweep():
    lib = _load()
    if not getattr(lib, "_sweep_ready", False):
        i32, vp = ctypes.c_int32, ctypes.c_void_p
        lib.oracle_importance_shift.argtypes = [i32, i32, vp, ctypes.c_float, vp]
        lib.oracle_importance_shift.restype = ctypes.c_double
        lib.oracle_front.argtypes = [i32, vp, i32, vp, vp]
        lib.oracle_front.restype = i32
        lib.oracle_front_queries.argtypes = [i32, i32, vp, vp, i32, vp, vp]
        lib.oracle_front_queries.restype = i32
        lib.oracle_chain_latency.argtypes = [i32, vp, i32, vp]
        lib.oracle_chain_latency.restype = i32
        lib._sweep_ready = True
    return lib


def importance_shift(I_raw, alpha):
    """I_raw float32 [L+1][L+1] or [L+1][L+1][2][2] -> (shifted table, mean of D)."""
    L = I_raw.shape[0] - 1
    F = 1 if I_raw.ndim == 2 else 4
    _chk(I_raw, np.float32, (L + 1, L + 1) if F == 1 else (L + 1, L + 1, 2, 2))
    out = np.empty_like(I_raw)
    mean = _load_sweep().oracle_importance_shift(L, F, _p(I_raw), float(np.float32(alpha)), _p(out))
    return out, mean


def front(Mrow, cap=None):
    """Mrow float32 [P] -> (budgets int32 [n], objectives float32 [n], count)."""
    P = Mrow.shape[0]
    _chk(Mrow, np.float32, (P,))
    cap = P if cap is None else cap
    ft = np.full(cap, -1, np.int32)
    fo = np.full(cap, -np.inf, np.float32)
    n = _load_sweep().oracle_front(P, _p(Mrow), cap, _p(ft), _p(fo))
    return ft[:min(n, cap)], fo[:min(n, cap)], n


def chain_latency(T, X):
    """T int32 [L+1][L+1], X ascending members of [1, L-1] (None: no set) -> int."""
    L = T.shape[0] - 1
    _chk(T, np.int32, (L + 1, L + 1))
    if X is None:
        return _load_sweep().oracle_chain_latency(L, _p(T), -1, None)
    X = np.ascontiguousarray(X, np.int32)
    return _load_sweep().oracle_chain_latency(L, _p(T), len(X), _p(X))


def front_queries(front_t, front_len, qcap):
    """front_t int32 [B][cap], front_len int32 [B] -> (q_inst, q_T0 int32 [min(n, qcap)], n)."""
    B, cap = front_t.shape
    _chk(front_t, np.int32, (B, cap))
    _chk(front_len, np.int32, (B,))
    qi = np.full(qcap, -1, np.int32)
    qt = np.full(qcap, -1, np.int32)
    n = _load_sweep().oracle_front_queries(B, cap, _p(front_t), _p(front_len), qcap, _p(qi), _p(qt))
    return qi[:min(n, qcap)], qt[:min(n, qcap)], n
