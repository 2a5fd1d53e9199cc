"""GPU parity of the extended solver (Appendix B of the paper: Algorithms 3
and 4) against its CPU oracle, element by element, tolerance 0."""
import numpy as np
import pytest
import torch

import oracle
from paper_2301_12187_amd import api, inputs
from helpers import bits, rand_tables
from gpu_common import first_diff
from test_ext_oracle_pins import rand_i4

pytestmark = pytest.mark.gpu


def run_ext_gpu(T, I4, P, qi, qt):
    B, ld, _ = T.shape
    L = ld - 1
    dev = torch.device("cuda:0")
    buf = api.ExtBuffers(B, L, P, len(qi))
    buf.D.fill_(float("nan"))
    buf.Kx.fill_(0xEE)
    buf.Iopt.fill_(float("nan"))
    buf.bsplit.fill_(0xEE)
    for x in (buf.A, buf.S, buf.Bs):
        x.fill_(-9)
    api.ext_solve(torch.from_numpy(T).to(dev), torch.from_numpy(I4).to(dev),
                  torch.from_numpy(np.ascontiguousarray(qi, np.int32)).to(dev),
                  torch.from_numpy(np.ascontiguousarray(qt, np.int32)).to(dev), buf)
    api.dpc_ext_check(B, L, P, buf.workspace)
    torch.cuda.synchronize()
    return {k: getattr(buf, k).cpu().numpy() for k in
            ("Topt", "split", "Iopt", "bsplit", "D", "Kx", "A", "S", "Bs", "A_len", "S_len",
             "B_len", "obj", "lat", "a_last", "status")}


def compare_ext(g, T, I4, P, qi, qt, what, threads=8):
    B, ld, _ = T.shape
    L = ld - 1
    Topt, split, Iopt, bsplit, D, Kx = oracle.ext_solve_batch(T, I4, P, threads=threads)
    assert first_diff(g["Topt"], Topt) is None and first_diff(g["split"], split) is None
    ii, jj = np.triu_indices(L + 1, k=1)
    d = first_diff(bits(g["Iopt"]), bits(Iopt))
    assert d is None, (what, "Iopt", d, g["Iopt"][d], Iopt[d])
    d = first_diff(g["bsplit"], bsplit)
    assert d is None, (what, "bsplit", d)
    # rows 2l+a of the library's table are D[l][.][a]; rows 0, 1 the base; the last the better flag
    Dv = np.transpose(D, (0, 1, 3, 2)).reshape(B, 2 * (L + 1), P)
    Kv = np.transpose(Kx, (0, 1, 3, 2)).reshape(B, 2 * (L + 1), P)
    d = first_diff(bits(g["D"][:, 2:2 * L + 2]), bits(Dv[:, 2:]))
    assert d is None, (what, "D", d)
    d = first_diff(g["Kx"][:, 2:2 * L + 2], Kv[:, 2:])
    assert d is None, (what, "Kx", d)
    assert (bits(g["D"][:, :2]) == 0).all()
    assert (bits(g["D"][:, 2 * L + 2]) == bits(D[:, L].max(axis=2))).all()
    for q, (b, t) in enumerate(zip(qi, qt)):
        r = oracle.ext_backtrack(Topt[b], split[b], bsplit[b], D[b], Kx[b], int(t))
        assert g["status"][q] == r["status"], (what, q)
        assert (g["A_len"][q], g["S_len"][q], g["B_len"][q]) == (r["A_len"], r["S_len"], r["B_len"])
        assert g["lat"][q] == r["lat"] and g["a_last"][q] == r["a_last"]
        assert bits(g["obj"][q:q + 1])[0] == bits(np.array([r["obj"]]))[0]
        if r["status"] == 0:
            assert list(g["A"][q][:r["A_len"]]) == list(r["A"])
            assert list(g["S"][q][:r["S_len"]]) == list(r["S"])
            assert list(g["Bs"][q][:r["B_len"]]) == list(r["B"])


@pytest.mark.parametrize("seed", range(4))
def test_tiny_tie_rich_extended_instances(seed):
    rng = np.random.default_rng(7000 + seed)
    B, L, P = 5, int(rng.integers(1, 15)), int(rng.integers(20, 200))
    Ts, Is = [], []
    for b in range(B):
        T, _ = rand_tables(rng, L, tmax=6, inf_frac=0.2, ikind="int")
        Ts.append(T)
        Is.append(rand_i4(rng, L, "exact" if b % 2 else "float", paper_rules=b != 3))
    T, I4 = np.stack(Ts), np.stack(Is)
    qi = np.repeat(np.arange(B, dtype=np.int32), P)
    qt = np.tile(np.arange(P, dtype=np.int32), B)
    g = run_ext_gpu(T, I4, P, qi, qt)
    compare_ext(g, T, I4, P, qi, qt, f"tiny ext seed {seed} L={L} P={P}")


def test_extended_tables_narrower_than_the_window_kernels_take():
    """Fewer than 16 budgets: stage 2 runs row by row on the expanded virtual tables."""
    rng = np.random.default_rng(7300)
    B, L, P = 4, 9, 13
    Ts, Is = [], []
    for b in range(B):
        T, _ = rand_tables(rng, L, tmax=3, inf_frac=0.2, ikind="int")
        Ts.append(T)
        Is.append(rand_i4(rng, L, "exact" if b % 2 else "float"))
    T, I4 = np.stack(Ts), np.stack(Is)
    qi = np.repeat(np.arange(B, dtype=np.int32), P)
    qt = np.tile(np.arange(P, dtype=np.int32), B)
    g = run_ext_gpu(T, I4, P, qi, qt)
    compare_ext(g, T, I4, P, qi, qt, "narrow ext table")


def test_mobilenet_shaped_extended_batch():
    """L = 53 (the paper's MobileNetV2 chain), P = 1000, a batch of instances
    with the identity pattern and exclusions of Appendix B.2."""
    cfg = inputs.CONFIGS[3]
    T, I4, base = inputs.make_ext_batch(cfg, seed=0, B=48)
    qi, qt = inputs.budgets(cfg, base)
    sel = qi < 48
    qi, qt = qi[sel], qt[sel]
    g = run_ext_gpu(T, I4, cfg.P, qi, qt)
    compare_ext(g, T, I4, cfg.P, qi, qt, "cfg3-shaped extended", threads=16)
    assert (g["status"] == 0).any()


@pytest.mark.parametrize("L", [53, 63, 9])
def test_extended_batch_of_short_chains(L):
    """Batches of 128 instances and more with chains of at most 63 layers take the
    kernels that stage an instance's tables in LDS (Algorithms 1 and 3)."""
    rng = np.random.default_rng(7200 + L)
    B, P = 160, 260
    Ts, Is = [], []
    for b in range(B):
        T, _ = rand_tables(rng, L, tmax=7, inf_frac=0.25, ikind="int", span=8)
        Ts.append(T)
        Is.append(rand_i4(rng, L, "exact" if b % 3 == 0 else "float", paper_rules=b % 5 != 4))
    T, I4 = np.stack(Ts), np.stack(Is)
    qi = np.repeat(np.arange(B, dtype=np.int32), 3)
    qt = np.tile(np.array([P // 3, P // 2, P - 1], np.int32), B)
    g = run_ext_gpu(T, I4, P, qi, qt)
    compare_ext(g, T, I4, P, qi, qt, f"ext batch of short chains L={L}", threads=16)


def test_largest_supported_chain():
    rng = np.random.default_rng(7100)
    B, L, P = 2, api.DPC_EXT_MAX_L, 700
    Ts, Is = [], []
    for b in range(B):
        T, _ = rand_tables(rng, L, tmax=9, inf_frac=0.3, ikind="int", span=10)
        Ts.append(T)
        Is.append(rand_i4(rng, L, "float"))
    T, I4 = np.stack(Ts), np.stack(Is)
    qi = np.repeat(np.arange(B, dtype=np.int32), 20)
    qt = np.tile(np.arange(0, P, 35, dtype=np.int32), B)
    g = run_ext_gpu(T, I4, P, qi, qt)
    compare_ext(g, T, I4, P, qi, qt, "L = 126")
