"""Seeded synthetic workloads: latency tables T and importance tables I.

Holds none of the method's arithmetic (no dynamic program, no set recovery):
it only draws the input tables that both the HIP library and the CPU checker
consume.  The paper's measured MobileNetV2 tables (171 latency blocks, 315
importance blocks, Appendix B.2) are not available; these generators stand in
for them with the same structure: a chain of L convolution layers, block
latency T[i,j] for merging layers i+1..j (Section 4.1), "not mergeable" for
spans beyond a limit (Appendix B.2), block importance I[i,j] <= 0 with
I[i,i+1] = 0 (Eq. 3: a one-layer block removes no activation).

Recipe, per instance b of config c (numpy only, vectorised):
  rng   = Generator(PCG64(SeedSequence([seed, c, b])))
  base  = rng.integers(lo, hi + 1, size=L)              per-layer latency
  pairs = all (i, j), 0 <= i < j <= L, row-major
  u     = rng.uniform(0.5, 1.2, size=npairs)
  coin  = rng.random(npairs)                            always drawn
  E     = rng.exponential(mu, npairs)
  G     = rng.normal(0, 0.01, npairs)
  T[i,j] = max(1, floor(u * sum(base[i:j]) + 0.5))      if j - i <= span
           DPC_INF                                      otherwise, or if the
                                                        config masks and
                                                        j - i >= 2, coin < 0.2
  I[i,i+1] = +0.0;  I[i,j] = float32(min(0, -(j-i-1) * E + G)),  -0.0 -> +0.0
Entries with i >= j are 0 and are never read.
"""
from dataclasses import dataclass

import numpy as np

DPC_INF = 0x3FFFFFFF


@dataclass(frozen=True)
class Config:
    cid: int
    B: int
    L: int
    P: int
    base_lo: int
    base_hi: int
    span: int          # max j - i that can be merged; >= L means dense
    mu: float          # mean of the exponential in I
    mask_frac: float   # fraction of mergeable spans >= 2 set to INF
    name: str


CONFIGS = {
    1: Config(1, 1, 16, 256, 5, 40, 6, 0.05, 0.0, "cfg1 single L=16 P=256"),
    2: Config(2, 1, 53, 1000, 5, 40, 8, 0.05, 0.0, "cfg2 MobileNetV2-shaped L=53 P=1000 B=1"),
    3: Config(3, 1024, 53, 1000, 5, 40, 8, 0.05, 0.0, "cfg3 batch B=1024 L=53 P=1000"),
    4: Config(4, 256, 100, 4000, 2, 20, 12, 0.02, 0.2, "cfg4 B=256 L=100 P=4000 masked"),
    5: Config(5, 64, 200, 16000, 1, 10, 1 << 20, 0.05, 0.0, "cfg5 stress B=64 L=200 P=16000 dense"),
}


def make_instance(L, base_lo, base_hi, span, mu, mask_frac, seed_words):
    """-> (T int32 [L+1][L+1], I float32 [L+1][L+1], base int64 [L])."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence(list(seed_words))))
    base = rng.integers(base_lo, base_hi + 1, size=L)
    ii, jj = np.triu_indices(L + 1, k=1)          # row-major pairs i < j
    n = ii.size
    u = rng.uniform(0.5, 1.2, size=n)
    coin = rng.random(n)
    E = rng.exponential(mu, n)
    G = rng.normal(0.0, 0.01, n)
    csum = np.concatenate([[0], np.cumsum(base)])
    seg = (csum[jj] - csum[ii]).astype(np.float64)
    width = jj - ii
    tval = np.maximum(1, np.floor(u * seg + 0.5)).astype(np.int64)
    blocked = width > span
    if mask_frac > 0.0:
        blocked |= (width >= 2) & (coin < mask_frac)
    tval[blocked] = DPC_INF
    ival = np.minimum(0.0, -(width - 1) * E + G).astype(np.float32)
    ival[width == 1] = 0.0
    ival = ival + np.float32(0.0)                 # -0.0 -> +0.0
    T = np.zeros((L + 1, L + 1), np.int32)
    I = np.zeros((L + 1, L + 1), np.float32)
    T[ii, jj] = tval.astype(np.int32)
    I[ii, jj] = ival
    return T, I, base


def make_batch(cfg: Config, seed: int = 0, B: int = None):
    """-> (T int32 [B][L+1][L+1], I float32 [B][L+1][L+1], base int64 [B][L])."""
    B = cfg.B if B is None else B
    Ts = np.empty((B, cfg.L + 1, cfg.L + 1), np.int32)
    Is = np.empty((B, cfg.L + 1, cfg.L + 1), np.float32)
    bases = np.empty((B, cfg.L), np.int64)
    for b in range(B):
        Ts[b], Is[b], bases[b] = make_instance(
            cfg.L, cfg.base_lo, cfg.base_hi, cfg.span, cfg.mu, cfg.mask_frac,
            (seed, cfg.cid, b))
    return Ts, Is, bases


def budgets(cfg: Config, bases):
    """Budgets T0 to recover sets for, as (q_inst int32 [Q], q_T0 int32 [Q]).

    cfg1: 60 % of the summed per-layer latency; cfg2: every t in [0, P);
    cfg3 and cfg4: 50/60/70/80/90 % of the summed per-layer latency of each
    instance; cfg5: every multiple of 100 in [0, P).  Clipped to P - 1."""
    B = bases.shape[0]
    tot = bases.sum(axis=1)
    qi, qt = [], []
    for b in range(B):
        if cfg.cid == 1:
            ts = [int(np.floor(0.6 * tot[b]))]
        elif cfg.cid == 2:
            ts = list(range(cfg.P))
        elif cfg.cid == 5:
            ts = list(range(0, cfg.P, 100))
        else:
            ts = [int(np.floor(f * tot[b])) for f in (0.5, 0.6, 0.7, 0.8, 0.9)]
        for t in ts:
            qi.append(b)
            qt.append(min(max(t, 0), cfg.P - 1))
    return np.asarray(qi, np.int32), np.asarray(qt, np.int32)


def relax_ops_exact(B, L, P):
    """Stage-2 candidates: one per (instance, pair i<j, budget t)."""
    return B * P * (L * (L + 1) // 2)


def relax_ops_nominal(B, L, P):
    return B * L * L * P


# ---- extended solver (Appendix B of the paper): importances with end flags ----

def make_flag_importances(I, seed_words, ident_every=3, bonus=0.02):
    """Flag-dependent importances I4 [L+1][L+1][2][2] around a plain table I.

    Stand-in for the paper's 315 measured MobileNetV2 blocks (Appendix B.2): the
    original activation is an identity at every `ident_every`-th layer (the end
    of an inverted-residual block) and at the two ends of the network.  Keeping
    an activation where the original has an identity adds a small positive
    amount, drawn per (block, end), as the paper reports non-linearities at
    those positions to help.  Then the exclusions of the first lines of
    Algorithm 3:
      I4[k][l][0][b] = -inf where the original activation at k is not an identity,
      I4[k][l][a][0] = -inf where the original activation at l is not an identity,
      I4[k][l][a][0] = -inf where both are identities.
    """
    L = I.shape[0] - 1
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([*seed_words, 77])))
    ident = np.zeros(L + 1, bool)
    ident[::ident_every] = True
    ident[0] = ident[L] = True
    gain = rng.exponential(bonus, size=(L + 1, L + 1, 2)).astype(np.float32)
    I4 = np.repeat(np.repeat(I[:, :, None, None], 2, axis=2), 2, axis=3).astype(np.float32)
    I4[:, :, 1, :] += (gain[:, :, 0] * ident[:, None])[:, :, None]
    I4[:, :, :, 1] += (gain[:, :, 1] * ident[None, :])[:, :, None]
    ninf = np.float32(-np.inf)
    I4[~ident, :, 0, :] = ninf
    I4[:, ~ident, :, 0] = ninf
    both = ident[:, None] & ident[None, :]
    I4[both, :, 0] = ninf
    I4 = I4 + np.float32(0.0)
    return np.ascontiguousarray(I4)


def make_ext_batch(cfg, seed=0, B=None):
    """-> (T, I4 float32 [B][L+1][L+1][2][2], base) for the extended solver."""
    T, I, base = make_batch(cfg, seed=seed, B=B)
    I4 = np.stack([make_flag_importances(I[b], (seed, cfg.cid, b)) for b in range(T.shape[0])])
    return T, I4, base


# ---- sweep over the normalisation constant alpha (appendix "Evaluating and
#      Normalizing the Importance") ----

def make_sweep_batch(cfg, seed=0, n_raw=None, n_alpha=16, alpha_max=2.0):
    """Raw tables for a sweep: -> (T int32 [n_raw][L+1][L+1], I_raw float32 (same shape),
    base, alphas float32 [n_alpha]).

    The tables are those of make_batch, except that the blocks of size one
    carry a measured accuracy change instead of 0: I[i][i+1] = -Exp(mean mu/5),
    drawn in ascending i from a stream of their own.  alphas are n_alpha evenly
    spaced values in [0, alpha_max].  Solving table b at alpha a as instance
    b * n_alpha + a gives n_raw * n_alpha instances (by default cfg.B)."""
    n_raw = max(1, cfg.B // n_alpha) if n_raw is None else n_raw
    T, I, base = make_batch(cfg, seed=seed, B=n_raw)
    for b in range(n_raw):
        rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, cfg.cid, b, 0x51])))
        idx = np.arange(cfg.L)
        I[b, idx, idx + 1] = (-rng.exponential(cfg.mu / 5.0, cfg.L)).astype(np.float32)
    alphas = np.linspace(0.0, alpha_max, n_alpha).astype(np.float32)
    return T, I, base, alphas
