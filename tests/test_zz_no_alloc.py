"""dpc_stage2_knapsack_static (the entry point for callers that cannot
allocate: its workspace is a fixed array inside the library) against
dpc_stage2_knapsack, through the C ABI, bit for bit: two calls in a row on the
same GPU, the second on a smaller problem, so that what the first call left in
the array is in the way of the second."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2301_12187_amd import api, inputs

pytestmark = pytest.mark.gpu


def _tables(cfg, B, seed):
    T, I, _ = inputs.make_batch(cfg, seed=seed, B=B)
    dev = torch.device("cuda:0")
    Td, Id = torch.from_numpy(T).to(dev), torch.from_numpy(I).to(dev)
    ld = cfg.L + 1
    Topt = torch.empty((B, ld, ld), dtype=torch.int32, device=dev)
    split = torch.empty((B, ld, ld), dtype=torch.uint8, device=dev)
    api.dpc_stage1_minplus(Td, Topt, split)
    return Topt, Id


def _both(lib, Topt, I, P, store_K=True):
    """-> ((M, K) of dpc_stage2_knapsack, (M, K) of dpc_stage2_knapsack_static), raw C calls."""
    B, ld, _ = Topt.shape
    L = ld - 1
    dev = Topt.device
    vp = ctypes.c_void_p
    stream = vp(torch.cuda.current_stream().cuda_stream)
    out = []
    for static in (False, True):
        M = torch.full((B, ld, P), float("nan"), dtype=torch.float32, device=dev)
        K = torch.full((B, ld, P), 0xEE, dtype=torch.uint8, device=dev) if store_K else None
        kp = vp(K.data_ptr()) if store_K else None
        if static:
            rc = lib.dpc_stage2_knapsack_static(B, L, P, vp(Topt.data_ptr()), vp(I.data_ptr()),
                                                vp(M.data_ptr()), kp, stream)
        else:
            n = lib.dpc_stage2_workspace_bytes(B, L, P)
            ws = torch.empty(n, dtype=torch.uint8, device=dev)
            rc = lib.dpc_stage2_knapsack(B, L, P, vp(Topt.data_ptr()), vp(I.data_ptr()),
                                         vp(M.data_ptr()), kp, vp(ws.data_ptr()), n, stream)
        assert rc == 0, (static, rc)
        torch.cuda.synchronize()
        out.append((M.cpu().numpy(), None if K is None else K.cpu().numpy()))
    return out


def _same(a, b):
    assert (a[0].view(np.uint32) == b[0].view(np.uint32)).all()
    if a[1] is not None:
        assert (a[1] == b[1]).all()
    assert not np.isnan(a[0]).any()


def test_static_workspace_two_calls_the_second_smaller():
    lib = api.load()
    # first call: 16-row groups, several strips, the device-side choice of shape
    cfg = inputs.CONFIGS[5]
    Topt, I = _tables(cfg, 6, seed=11)
    ref, got = _both(lib, Topt, I, cfg.P)
    _same(ref, got)
    # second call, right after it on the same array: a smaller problem of another shape
    cfg = inputs.CONFIGS[3]
    Topt, I = _tables(cfg, 40, seed=12)
    ref, got = _both(lib, Topt, I, cfg.P)
    _same(ref, got)
    # and a third without back-pointers, smaller still
    cfg = inputs.CONFIGS[1]
    Topt, I = _tables(cfg, 1, seed=13)
    ref, got = _both(lib, Topt, I, cfg.P, store_K=False)
    _same(ref, got)


def test_static_workspace_refuses_what_does_not_fit():
    lib = api.load()
    p = ctypes.c_void_p(256)          # never dereferenced: the checks fail first
    assert lib.dpc_stage2_workspace_bytes(2048, 53, 1000) > api.DPC_STATIC_WORKSPACE_BYTES
    assert lib.dpc_stage2_knapsack_static(2048, 53, 1000, p, p, p, p, None) == -3     # DPC_ERR_WORKSPACE
    assert lib.dpc_stage2_knapsack_static(1, 53, 1000, None, p, p, p, None) == -1     # DPC_ERR_NULL
    assert lib.dpc_stage2_knapsack_static(1, 300, 1000, p, p, p, p, None) == -2       # DPC_ERR_SHAPE
