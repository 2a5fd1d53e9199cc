"""Set-carrying transcription of the paper's recurrences, for tiny inputs.

Written from Eq. 5 and Eq. 7 and the prose of Section 4.3 with the paper's own
conventions, which differ from the oracle's on purpose: strict budgets
("latency < t"), cells initialised to 0 and guarded by the explicit side
constraint T_opt[0,k'] + T_opt[k',l] < t, and whole ordered sets stored per
cell instead of back-pointers.  The tests check the oracle against it through
the identity  D_paper[l][t] == M_oracle[l][t-1]  and the equality of the sets.
Pure Python + numpy scalars; first maximum / minimum wins ties.
"""
import numpy as np

INF = 0x3FFFFFFF


def time_dp(T, L):
    """Eq. 5 by dynamic programming over the last merged block."""
    Topt = [[0] * (L + 1) for _ in range(L + 1)]
    Sopt = [[() for _ in range(L + 1)] for _ in range(L + 1)]
    for l in range(1, L + 1):
        for k in range(l):
            cands = [min(Topt[k][m] + int(T[m][l]), INF) for m in range(k, l)]
            m = k + cands.index(min(cands))
            Topt[k][l] = cands[m - k]
            if m != k and cands[m - k] < INF:
                Sopt[k][l] = Sopt[k][m] + (m,)
    return Topt, Sopt


def surrogate_dp(T0, L, T, I):
    """Eq. 7 for every t in 1..T0.  Returns D, A, S as dicts keyed by (l, t);
    a key is present only where the paper's loop assigns the cell."""
    Topt, Sopt = time_dp(T, L)
    D, A, S = {}, {}, {}
    for t in range(0, T0 + 1):
        D[(0, t)] = np.float32(0.0)
        A[(0, t)] = ()
        S[(0, t)] = ()
    for l in range(1, L + 1):
        if Topt[0][l] >= INF:
            continue
        for t in range(Topt[0][l] + 1, T0 + 1):
            best, k = None, None
            for kp in range(l):
                if Topt[0][kp] + Topt[kp][l] < t:
                    c = np.float32(D[(kp, t - Topt[kp][l])] + np.float32(I[kp][l]))
                    if best is None or c > best:
                        best, k = c, kp
            tl = Topt[k][l]
            D[(l, t)] = best
            keep = (k,) if k > 0 else ()
            A[(l, t)] = A[(k, t - tl)] + keep
            S[(l, t)] = tuple(sorted(S[(k, t - tl)] + keep + Sopt[k][l]))
    return D, A, S, Topt, Sopt
