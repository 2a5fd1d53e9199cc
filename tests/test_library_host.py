"""Host-side checks of libdpc.so that need no GPU: the library loads, exports
every function include/dpc.h declares, and rejects bad arguments before any
device work is queued."""
import ctypes
import os
import re

import pytest

from paper_2301_12187_amd import api

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions(path=os.path.join(ROOT, "include", "dpc.h")):
    text = open(path).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dpc_[a-z0-9_]+)\s*\(", text)))


def test_header_functions_are_exported():
    names = _declared_functions()
    assert set(names) == set(api.EXPORTS), names
    lib = api.load()
    for n in names:
        assert getattr(lib, n) is not None
    # the test hook is exported too, but declared in an internal header only
    hooks = _declared_functions(os.path.join(ROOT, "paper_2301_12187_amd", "csrc", "dpc_hooks.h"))
    assert set(hooks) == set(api.HOOKS)
    for n in hooks:
        assert getattr(lib, n) is not None and n not in names


def test_argument_errors_are_reported_before_any_launch():
    lib = api.load()
    p = ctypes.c_void_p(256)          # never dereferenced: checks fail first
    NULL, SHAPE, WS = -1, -2, -3
    assert lib.dpc_stage1_minplus(1, 4, None, p, p, None) == NULL
    assert lib.dpc_stage1_minplus(1, 4, p, None, p, None) == NULL
    assert lib.dpc_stage1_minplus(0, 4, p, p, p, None) == SHAPE
    assert lib.dpc_stage1_minplus(1, 0, p, p, p, None) == SHAPE
    assert lib.dpc_stage1_minplus(1, 256, p, p, p, None) == SHAPE
    assert lib.dpc_stage2_knapsack(1, 4, 8, None, p, p, p, p, 256, None) == NULL
    assert lib.dpc_stage2_knapsack(1, 4, 8, p, p, p, None, None, 256, None) == NULL
    assert lib.dpc_stage2_knapsack(1, 4, 0, p, p, p, p, p, 256, None) == SHAPE
    assert lib.dpc_stage2_knapsack(1, 300, 8, p, p, p, p, p, 256, None) == SHAPE
    need = lib.dpc_stage2_workspace_bytes(4, 50, 1000)
    assert need >= 1
    assert lib.dpc_stage2_knapsack(4, 50, 1000, p, p, p, p, p, need - 1, None) == WS
    assert lib.dpc_stage2_knapsack(4, 50, 1000, p, p, p, p, ctypes.c_void_p(264), need, None) == WS
    assert lib.dpc_stage2_workspace_bytes(0, 50, 1000) == 0
    args = [p] * 10
    assert lib.dpc_backtrack(1, 4, 8, p, p, p, p, p, -1, *args, None) == SHAPE
    assert lib.dpc_backtrack(1, 4, 8, p, p, p, p, p, 0, *args, None) == 0     # nothing to do
    assert lib.dpc_backtrack(1, 4, 8, None, p, p, p, p, 3, *args, None) == NULL
    assert lib.dpc_backtrack(1, 4, 8, p, p, p, p, None, 3, p, None, *([p] * 8), None) == NULL
    assert lib.dpc_stage2_knapsack_shape(4, 50, 1000, p, p, p, p, p, need, 7, None) == SHAPE
    assert lib.dpc_stage2_knapsack_shape(4, 50, 1000, p, p, p, p, p, need, 37, None) == SHAPE
    assert b"DPC_ERR_NULL" in lib.dpc_status_string(NULL)
    assert lib.dpc_status_string(12345)


def test_argument_errors_of_the_widened_entry_points():
    api._load_ext(), api._load_sweep(), api._load_fused()
    lib = api.load()
    p = ctypes.c_void_p(256)          # never dereferenced: checks fail first
    NULL, SHAPE = -1, -2
    # extended solver
    assert lib.dpc_ext_importance_maxplus(1, 4, None, p, p, None) == NULL
    assert lib.dpc_ext_importance_maxplus(1, 256, p, p, p, None) == SHAPE
    assert lib.dpc_ext_workspace_bytes(1, 127, 100) == 0          # beyond DPC_EXT_MAX_L
    assert lib.dpc_ext_workspace_bytes(1, 126, 100) > 0
    assert lib.dpc_ext_knapsack(1, 127, 100, p, p, p, p, p, 1 << 30, None) == SHAPE
    assert lib.dpc_ext_knapsack(1, 10, 100, p, None, p, p, p, 1 << 30, None) == NULL
    assert lib.dpc_ext_backtrack(1, 10, 100, p, p, p, p, p, -1, *([p] * 12), None) == SHAPE
    assert lib.dpc_ext_backtrack(1, 10, 100, p, p, p, p, None, 2, *([p] * 12), None) == NULL
    # sweep steps
    assert lib.dpc_importance_shift(1, 4, 2, 1, p, p, p, None, None) == SHAPE      # F is 1 or 4
    assert lib.dpc_importance_shift(1, 4, 1, -1, p, p, p, None, None) == SHAPE
    assert lib.dpc_importance_shift(1, 4, 1, 0, None, None, None, None, None) == 0  # nothing to do
    assert lib.dpc_importance_shift(1, 4, 4, 3, p, None, p, None, None) == NULL
    assert lib.dpc_front(1, 4, 8, p, -1, p, p, p, None) == SHAPE
    assert lib.dpc_front(1, 4, 8, None, 4, p, p, p, None) == NULL
    assert lib.dpc_front(1, 4, 8, p, 4, None, p, p, None) == NULL
    assert lib.dpc_front_queries(1, -1, p, p, 4, p, p, p, None) == SHAPE
    assert lib.dpc_front_queries(1, 4, p, p, 4, p, p, None, None) == NULL
    assert lib.dpc_chain_latency(1, 4, p, -1, p, p, p, p, None) == SHAPE
    assert lib.dpc_chain_latency(1, 4, p, 0, None, None, None, None, None) == 0
    assert lib.dpc_chain_latency(1, 4, p, 3, p, None, p, p, None) == NULL
    # shared stage-1 tables
    assert lib.dpc_stage2_knapsack_shared(4, 50, 1000, 0, p, p, p, p, p, 1 << 30, None) == SHAPE
    assert lib.dpc_stage2_knapsack_shared(4, 50, 1000, 2, None, p, p, p, p, 1 << 30, None) == NULL
    assert lib.dpc_backtrack_shared(1, 4, 8, 0, p, p, p, p, p, 3, *([p] * 9), None) == SHAPE
    assert lib.dpc_backtrack_shared(1, 4, 8, 2, p, None, p, p, p, 3, *([p] * 9), None) == NULL
    # single-launch path
    assert lib.dpc_stage12_fused(1, 4, 8, None, p, p, p, p, p, None) == NULL
    assert lib.dpc_stage12_fused(1, 300, 8, p, p, p, p, p, p, None) == SHAPE
    assert lib.dpc_solve_fused(1, 4, 8, p, p, p, p, p, p, -1, *([p] * 9), None) == SHAPE
    assert lib.dpc_solve_fused(1, 4, 8, p, p, p, p, p, p, 2, None, *([p] * 8), None) == NULL
    assert lib.dpc_solve_fused(1, 300, 8, p, p, p, p, p, p, 0, *([None] * 9), None) == SHAPE
    assert lib.dpc_stage12_fused_supported(64, 100) == 0
    assert lib.dpc_stage12_fused_supported(10, 4096) == 0


def test_binding_refuses_cpu_tensors():
    import torch
    T = torch.zeros((1, 5, 5), dtype=torch.int32)
    with pytest.raises(api.DpcError):
        api.dpc_stage1_minplus(T, T.clone(), torch.zeros((1, 5, 5), dtype=torch.uint8))
