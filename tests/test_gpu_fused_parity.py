"""GPU parity of the single-launch path for small instances (stage 1 and stage 2
in one kernel, then set recovery) against the CPU oracle, element by element,
tolerance 0, through the C ABI."""
import numpy as np
import pytest
import torch

from paper_2301_12187_amd import api, inputs
from helpers import rand_tables
from gpu_common import compare, run_gpu, run_oracle

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cid", [1, 2])
@pytest.mark.parametrize("store_K", [True, False])
@pytest.mark.parametrize("one_launch", [True, False])
def test_small_configs_bit_exact(cid, store_K, one_launch):
    """Stage 1 + stage 2 in one launch followed by dpc_backtrack, and the whole
    path in one launch (dpc_solve_fused: every budget of the L=53 instance is
    then answered by the instance's own workgroup)."""
    cfg = inputs.CONFIGS[cid]
    assert api.dpc_stage12_fused_supported(cfg.L, cfg.P)
    T, I, base = inputs.make_batch(cfg, seed=0)
    qi, qt = inputs.budgets(cfg, base)
    g = run_gpu(T, I, cfg.P, qi, qt, store_K=store_K, fused=True, one_launch=one_launch)
    compare(g, run_oracle(T, I, cfg.P, qi, qt), cfg.L, f"cfg{cid}")


def test_batch_of_mobilenet_shaped_instances():
    """One workgroup per instance: 40 instances of the L=53, P=1000 shape, some
    rows of M in LDS and the rest read back from the output array."""
    cfg = inputs.CONFIGS[3]
    T, I, base = inputs.make_batch(cfg, seed=4, B=40)
    qi, qt = inputs.budgets(cfg, base)
    g = run_gpu(T, I, cfg.P, qi, qt, fused=True, one_launch=False)
    compare(g, run_oracle(T, I, cfg.P, qi, qt), cfg.L, "cfg3 shape, B=40")


def test_one_launch_with_queries_in_any_order_and_bad_queries():
    """dpc_solve_fused: a shuffled query list over 40 instances, several queries
    per instance, queries that name no instance or no budget, more than 64
    queries (several chunks per wave)."""
    cfg = inputs.CONFIGS[3]
    T, I, base = inputs.make_batch(cfg, seed=6, B=40)
    qi, qt = inputs.budgets(cfg, base)
    rng = np.random.default_rng(5)
    qi = np.concatenate([qi, [-1, 40, 3, 7]]).astype(np.int32)
    qt = np.concatenate([qt, [5, 5, cfg.P, -2]]).astype(np.int32)
    perm = rng.permutation(len(qi))
    qi, qt = qi[perm], qt[perm]
    g = run_gpu(T, I, cfg.P, qi, qt, fused=True, one_launch=True)
    bad = (qi < 0) | (qi >= 40) | (qt < 0) | (qt >= cfg.P)
    assert (g["status"][bad] == 2).all() and (g["A_len"][bad] == -1).all()
    ok = ~bad
    r = run_oracle(T, I, cfg.P, qi[ok], qt[ok])
    gs = {k: (v if k in ("Topt", "split", "M", "K") else v[ok]) for k, v in g.items()}
    compare(gs, r, cfg.L, "one launch, shuffled queries")


@pytest.mark.parametrize("L,P", [(1, 1), (1, 64), (2, 65), (5, 63), (17, 1023), (31, 1024),
                                 (33, 1025), (63, 2048), (63, 1), (40, 1700), (9, 2047)])
def test_ragged_shapes_and_limits(L, P):
    rng = np.random.default_rng(L * 10000 + P)
    B = 3
    T, I = zip(*[rand_tables(rng, L, tmax=40, inf_frac=0.25, ikind=("neg", "mixed", "int")[b])
                 for b in range(B)])
    T, I = np.stack(T), np.stack(I)
    if L >= 6:
        T[1, 0, 4] = 100000                  # a shift beyond every budget
        I[2, 1, 5] = -np.inf                 # an excluded block
    qi = np.repeat(np.arange(B, dtype=np.int32), 4)
    qt = np.tile(np.array([0, P // 3, P // 2, P - 1], np.int32), B)
    for one_launch in (False, True):
        g = run_gpu(T, I, P, qi, qt, fused=True, one_launch=one_launch)
        compare(g, run_oracle(T, I, P, qi, qt), L, f"L={L} P={P} one_launch={one_launch}")


def test_unsupported_shapes_are_refused():
    assert not api.dpc_stage12_fused_supported(64, 100)
    assert not api.dpc_stage12_fused_supported(10, 2049)
    assert not api.dpc_stage12_fused_supported(0, 10)
    B, L, P = 1, 64, 100
    dev = "cuda:0"
    T = torch.ones((B, L + 1, L + 1), dtype=torch.int32, device=dev)
    I = torch.zeros((B, L + 1, L + 1), dtype=torch.float32, device=dev)
    buf = api.Buffers(B, L, P, 1)
    buf.M.fill_(7.0)
    with pytest.raises(api.DpcError):
        api.dpc_stage12_fused(T, I, buf.Topt, buf.split, buf.M, buf.K)
    torch.cuda.synchronize()
    assert (buf.M == 7.0).all()              # nothing was queued
