"""Thin Python binding over libdpc.so (see include/dpc.h for the contract).

Argument marshalling only: torch provides device memory and streams, every
step of the method runs in the HIP kernels behind the C ABI.  There is no CPU
fallback: if the library is not built, or a tensor is not on the GPU, the call
raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdpc.so")

DPC_INF = 0x3FFFFFFF
DPC_NOARG = 0xFF
DPC_MAX_L = 255
DPC_OK = 0

EXPORTS = (
    "dpc_stage1_minplus", "dpc_stage2_workspace_bytes", "dpc_stage2_knapsack",
    "dpc_stage2_check", "dpc_backtrack", "dpc_status_string",
    "dpc_stage2_knapsack_static",
    "dpc_ext_importance_maxplus", "dpc_ext_workspace_bytes", "dpc_ext_knapsack",
    "dpc_ext_check", "dpc_ext_backtrack",
    "dpc_importance_shift", "dpc_front", "dpc_front_queries", "dpc_chain_latency",
    "dpc_stage2_knapsack_shared", "dpc_backtrack_shared",
    "dpc_stage12_fused_supported", "dpc_stage12_fused", "dpc_solve_fused",
)

# exported for tests and measurements only (csrc/dpc_hooks.h), not part of include/dpc.h
HOOKS = ("dpc_stage2_knapsack_shape",)
SHAPE_ROWS = 1             # one launch per row
SHAPE_WAVE_BASE = 30       # + task shape of the persistent kernel, see csrc/dpc_hooks.h

_lib = None


class DpcError(RuntimeError):
    pass


def load():
    """Load libdpc.so and declare its signatures.  Raises if it is not built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise DpcError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2301_12187_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    i32, vp, sz = ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t
    lib.dpc_stage1_minplus.argtypes = [i32, i32, vp, vp, vp, vp]
    lib.dpc_stage1_minplus.restype = ctypes.c_int
    lib.dpc_stage2_workspace_bytes.argtypes = [i32, i32, i32]
    lib.dpc_stage2_workspace_bytes.restype = sz
    lib.dpc_stage2_knapsack.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.dpc_stage2_knapsack.restype = ctypes.c_int
    lib.dpc_stage2_knapsack_static.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp]
    lib.dpc_stage2_knapsack_static.restype = ctypes.c_int
    lib.dpc_stage2_check.argtypes = [vp, vp]
    lib.dpc_stage2_check.restype = ctypes.c_int
    lib.dpc_backtrack.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, i32, vp, vp,
                                  vp, vp, vp, vp, vp, vp, vp, vp]
    lib.dpc_backtrack.restype = ctypes.c_int
    lib.dpc_status_string.argtypes = [ctypes.c_int]
    lib.dpc_status_string.restype = ctypes.c_char_p
    lib.dpc_stage2_knapsack_shape.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, sz, i32, vp]
    lib.dpc_stage2_knapsack_shape.restype = ctypes.c_int
    _lib = lib
    return lib


def _check(code):
    if code != DPC_OK:
        raise DpcError(load().dpc_status_string(code).decode())


def _dev(t, dtype, shape, name):
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise DpcError(f"{name}: expected a GPU tensor (no CPU fallback)")
    if t.dtype != dtype or tuple(t.shape) != tuple(shape) or not t.is_contiguous():
        raise DpcError(f"{name}: expected contiguous {dtype} {tuple(shape)}, "
                       f"got {t.dtype} {tuple(t.shape)}")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def dpc_stage1_minplus(T, Topt, split, stream=None):
    """T int32 [B][L+1][L+1] -> Topt int32, split uint8 (same shape), in place."""
    B, ld, _ = T.shape
    shp = (B, ld, ld)
    _check(load().dpc_stage1_minplus(
        B, ld - 1, _dev(T, torch.int32, shp, "T"), _dev(Topt, torch.int32, shp, "Topt"),
        _dev(split, torch.uint8, shp, "split"), _stream(stream)))


def dpc_stage2_workspace_bytes(B, L, P):
    return int(load().dpc_stage2_workspace_bytes(B, L, P))


def dpc_stage2_knapsack(Topt, I, M, K, workspace, stream=None, shape=0):
    """Topt int32, I float32 [B][L+1][L+1] -> M float32, K uint8 or None [B][L+1][P].
    shape != 0 goes through the test hook dpc_stage2_knapsack_shape (a fixed kernel shape)."""
    B, ld, _ = Topt.shape
    P = M.shape[2]
    if not (isinstance(workspace, torch.Tensor) and workspace.is_cuda
            and workspace.dtype == torch.uint8 and workspace.is_contiguous()):
        raise DpcError("workspace: expected a contiguous uint8 GPU tensor")
    args = [B, ld - 1, P, _dev(Topt, torch.int32, (B, ld, ld), "Topt"),
            _dev(I, torch.float32, (B, ld, ld), "I"), _dev(M, torch.float32, (B, ld, P), "M"),
            None if K is None else _dev(K, torch.uint8, (B, ld, P), "K"),
            ctypes.c_void_p(workspace.data_ptr()), workspace.numel()]
    if shape:
        _check(load().dpc_stage2_knapsack_shape(*args, int(shape), _stream(stream)))
    else:
        _check(load().dpc_stage2_knapsack(*args, _stream(stream)))


DPC_STATIC_WORKSPACE_BYTES = 48 << 20


def dpc_stage2_knapsack_static(Topt, I, M, K, stream=None):
    """dpc_stage2_knapsack on the library's own fixed workspace (no allocation, no
    workspace argument); shapes that need more than DPC_STATIC_WORKSPACE_BYTES raise."""
    B, ld, _ = Topt.shape
    P = M.shape[2]
    _check(load().dpc_stage2_knapsack_static(
        B, ld - 1, P, _dev(Topt, torch.int32, (B, ld, ld), "Topt"),
        _dev(I, torch.float32, (B, ld, ld), "I"), _dev(M, torch.float32, (B, ld, P), "M"),
        None if K is None else _dev(K, torch.uint8, (B, ld, P), "K"), _stream(stream)))


def dpc_stage2_check(workspace, stream=None):
    _check(load().dpc_stage2_check(ctypes.c_void_p(workspace.data_ptr()), _stream(stream)))


def dpc_backtrack(Topt, split, I, M, K, q_inst, q_T0, A, A_len, S, S_len, obj, lat,
                  status, stream=None):
    B, ld, _ = Topt.shape
    L = ld - 1
    P = M.shape[2]
    Q = q_inst.shape[0]
    if Q == 0:
        return
    _check(load().dpc_backtrack(
        B, L, P, _dev(Topt, torch.int32, (B, ld, ld), "Topt"),
        _dev(split, torch.uint8, (B, ld, ld), "split"),
        _dev(I, torch.float32, (B, ld, ld), "I"), _dev(M, torch.float32, (B, ld, P), "M"),
        None if K is None else _dev(K, torch.uint8, (B, ld, P), "K"), Q,
        _dev(q_inst, torch.int32, (Q,), "q_inst"), _dev(q_T0, torch.int32, (Q,), "q_T0"),
        _dev(A, torch.int32, (Q, L), "A"), _dev(A_len, torch.int32, (Q,), "A_len"),
        _dev(S, torch.int32, (Q, L), "S"), _dev(S_len, torch.int32, (Q,), "S_len"),
        _dev(obj, torch.float32, (Q,), "obj"), _dev(lat, torch.int32, (Q,), "lat"),
        _dev(status, torch.int32, (Q,), "status"), _stream(stream)))


class Buffers:
    """Device buffers for one problem shape, allocated once and reused."""

    def __init__(self, B, L, P, Q, store_K=True, device="cuda:0"):
        self.B, self.L, self.P, self.Q = B, L, P, Q
        ld = L + 1
        dev = torch.device(device)
        self.Topt = torch.empty((B, ld, ld), dtype=torch.int32, device=dev)
        self.split = torch.empty((B, ld, ld), dtype=torch.uint8, device=dev)
        self.M = torch.empty((B, ld, P), dtype=torch.float32, device=dev)
        self.K = torch.empty((B, ld, P), dtype=torch.uint8, device=dev) if store_K else None
        self.workspace = torch.empty(max(dpc_stage2_workspace_bytes(B, L, P), 256),
                                     dtype=torch.uint8, device=dev)
        self.A = torch.empty((Q, L), dtype=torch.int32, device=dev)
        self.S = torch.empty((Q, L), dtype=torch.int32, device=dev)
        self.A_len = torch.empty((Q,), dtype=torch.int32, device=dev)
        self.S_len = torch.empty((Q,), dtype=torch.int32, device=dev)
        self.obj = torch.empty((Q,), dtype=torch.float32, device=dev)
        self.lat = torch.empty((Q,), dtype=torch.int32, device=dev)
        self.status = torch.empty((Q,), dtype=torch.int32, device=dev)


def solve(T, I, q_inst, q_T0, buf: Buffers, stream=None, shape=0):
    """The whole path on device tensors: stage 1, stage 2, set recovery.
    Queues the three calls on `stream` and returns without waiting."""
    dpc_stage1_minplus(T, buf.Topt, buf.split, stream)
    dpc_stage2_knapsack(buf.Topt, I, buf.M, buf.K, buf.workspace, stream, shape)
    dpc_backtrack(buf.Topt, buf.split, I, buf.M, buf.K, q_inst, q_T0, buf.A, buf.A_len,
                  buf.S, buf.S_len, buf.obj, buf.lat, buf.status, stream)


# ---- extended solver (Appendix B of the paper) ----

DPC_EXT_MAX_L = 126
EXT_EXPORTS = ("dpc_ext_importance_maxplus", "dpc_ext_workspace_bytes", "dpc_ext_knapsack",
               "dpc_ext_check", "dpc_ext_backtrack")


def _load_ext():
    lib = load()
    if not getattr(lib, "_ext_ready", False):
        i32, vp, sz = ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t
        lib.dpc_ext_importance_maxplus.argtypes = [i32, i32, vp, vp, vp, vp]
        lib.dpc_ext_importance_maxplus.restype = ctypes.c_int
        lib.dpc_ext_workspace_bytes.argtypes = [i32, i32, i32]
        lib.dpc_ext_workspace_bytes.restype = sz
        lib.dpc_ext_knapsack.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, sz, vp]
        lib.dpc_ext_knapsack.restype = ctypes.c_int
        lib.dpc_ext_check.argtypes = [i32, i32, i32, vp, vp]
        lib.dpc_ext_check.restype = ctypes.c_int
        lib.dpc_ext_backtrack.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, i32] + [vp] * 13
        lib.dpc_ext_backtrack.restype = ctypes.c_int
        lib._ext_ready = True
    return lib


def dpc_ext_importance_maxplus(I4, Iopt, bsplit, stream=None):
    B, ld = I4.shape[0], I4.shape[1]
    shp = (B, ld, ld, 2, 2)
    _check(_load_ext().dpc_ext_importance_maxplus(
        B, ld - 1, _dev(I4, torch.float32, shp, "I4"), _dev(Iopt, torch.float32, shp, "Iopt"),
        _dev(bsplit, torch.uint8, shp, "bsplit"), _stream(stream)))


def dpc_ext_workspace_bytes(B, L, P):
    return int(_load_ext().dpc_ext_workspace_bytes(B, L, P))


def dpc_ext_knapsack(Topt, Iopt, D, Kx, workspace, stream=None):
    B, ld, _ = Topt.shape
    L, P = ld - 1, D.shape[2]
    V = 2 * L + 3
    _check(_load_ext().dpc_ext_knapsack(
        B, L, P, _dev(Topt, torch.int32, (B, ld, ld), "Topt"),
        _dev(Iopt, torch.float32, (B, ld, ld, 2, 2), "Iopt"),
        _dev(D, torch.float32, (B, V, P), "D"), _dev(Kx, torch.uint8, (B, V, P), "Kx"),
        ctypes.c_void_p(workspace.data_ptr()), workspace.numel(), _stream(stream)))


def dpc_ext_check(B, L, P, workspace, stream=None):
    _check(_load_ext().dpc_ext_check(B, L, P, ctypes.c_void_p(workspace.data_ptr()),
                                     _stream(stream)))


def dpc_ext_backtrack(Topt, split, bsplit, D, Kx, q_inst, q_T0, A, A_len, S, S_len, Bs, B_len,
                      obj, lat, a_last, status, stream=None):
    B, ld, _ = Topt.shape
    L, P, Q = ld - 1, D.shape[2], q_inst.shape[0]
    V = 2 * L + 3
    if Q == 0:
        return
    i32 = torch.int32
    _check(_load_ext().dpc_ext_backtrack(
        B, L, P, _dev(Topt, i32, (B, ld, ld), "Topt"), _dev(split, torch.uint8, (B, ld, ld), "split"),
        _dev(bsplit, torch.uint8, (B, ld, ld, 2, 2), "bsplit"),
        _dev(D, torch.float32, (B, V, P), "D"), _dev(Kx, torch.uint8, (B, V, P), "Kx"), Q,
        _dev(q_inst, i32, (Q,), "q_inst"), _dev(q_T0, i32, (Q,), "q_T0"),
        _dev(A, i32, (Q, L), "A"), _dev(A_len, i32, (Q,), "A_len"),
        _dev(S, i32, (Q, L), "S"), _dev(S_len, i32, (Q,), "S_len"),
        _dev(Bs, i32, (Q, L), "Bs"), _dev(B_len, i32, (Q,), "B_len"),
        _dev(obj, torch.float32, (Q,), "obj"), _dev(lat, i32, (Q,), "lat"),
        _dev(a_last, i32, (Q,), "a_last"), _dev(status, i32, (Q,), "status"), _stream(stream)))


class ExtBuffers:
    """Device buffers of the extended solver for one problem shape."""

    def __init__(self, B, L, P, Q, device="cuda:0"):
        self.B, self.L, self.P, self.Q = B, L, P, Q
        ld, V = L + 1, 2 * L + 3
        dev = torch.device(device)
        e = lambda shape, dt: torch.empty(shape, dtype=dt, device=dev)  # noqa: E731
        self.Topt, self.split = e((B, ld, ld), torch.int32), e((B, ld, ld), torch.uint8)
        self.Iopt, self.bsplit = e((B, ld, ld, 2, 2), torch.float32), e((B, ld, ld, 2, 2), torch.uint8)
        self.D, self.Kx = e((B, V, P), torch.float32), e((B, V, P), torch.uint8)
        self.workspace = e((max(dpc_ext_workspace_bytes(B, L, P), 256),), torch.uint8)
        self.A, self.S, self.Bs = (e((Q, L), torch.int32) for _ in range(3))
        self.A_len, self.S_len, self.B_len, self.lat, self.a_last, self.status = (
            e((Q,), torch.int32) for _ in range(6))
        self.obj = e((Q,), torch.float32)


def ext_solve(T, I4, q_inst, q_T0, buf: ExtBuffers, stream=None):
    """The extended path on device tensors: Algorithm 1, Algorithm 3,
    Algorithm 4 and set recovery, queued on `stream` without waiting."""
    dpc_stage1_minplus(T, buf.Topt, buf.split, stream)
    dpc_ext_importance_maxplus(I4, buf.Iopt, buf.bsplit, stream)
    dpc_ext_knapsack(buf.Topt, buf.Iopt, buf.D, buf.Kx, buf.workspace, stream)
    dpc_ext_backtrack(buf.Topt, buf.split, buf.bsplit, buf.D, buf.Kx, q_inst, q_T0, buf.A,
                      buf.A_len, buf.S, buf.S_len, buf.Bs, buf.B_len, buf.obj, buf.lat,
                      buf.a_last, buf.status, stream)


# ---- steps around the solver in a sweep over hyper-parameters ----

def _load_sweep():
    lib = load()
    if not getattr(lib, "_sweep_ready", False):
        i32, vp = ctypes.c_int32, ctypes.c_void_p
        lib.dpc_importance_shift.argtypes = [i32, i32, i32, i32, vp, vp, vp, vp, vp]
        lib.dpc_importance_shift.restype = ctypes.c_int
        lib.dpc_front.argtypes = [i32, i32, i32, vp, i32, vp, vp, vp, vp]
        lib.dpc_front.restype = ctypes.c_int
        lib.dpc_front_queries.argtypes = [i32, i32, vp, vp, i32, vp, vp, vp, vp]
        lib.dpc_front_queries.restype = ctypes.c_int
        lib.dpc_chain_latency.argtypes = [i32, i32, vp, i32, vp, vp, vp, vp, vp]
        lib.dpc_chain_latency.restype = ctypes.c_int
        sz = ctypes.c_size_t
        lib.dpc_stage2_knapsack_shared.argtypes = [i32, i32, i32, i32, vp, vp, vp, vp, vp, sz, vp]
        lib.dpc_stage2_knapsack_shared.restype = ctypes.c_int
        lib.dpc_backtrack_shared.argtypes = [i32, i32, i32, i32, vp, vp, vp, vp, vp, i32] + [vp] * 10
        lib.dpc_backtrack_shared.restype = ctypes.c_int
        lib._sweep_ready = True
    return lib


def dpc_stage2_knapsack_shared(share, Topt, I, M, K, workspace, stream=None):
    """Stage 2 for B = I.shape[0] instances, instance x reading table x // share of Topt
    (int32 [ceil(B/share)][L+1][L+1])."""
    B, ld, _ = I.shape
    P = M.shape[2]
    nt = (B + share - 1) // share
    _check(_load_sweep().dpc_stage2_knapsack_shared(
        B, ld - 1, P, int(share), _dev(Topt, torch.int32, (nt, ld, ld), "Topt"),
        _dev(I, torch.float32, (B, ld, ld), "I"), _dev(M, torch.float32, (B, ld, P), "M"),
        None if K is None else _dev(K, torch.uint8, (B, ld, P), "K"),
        ctypes.c_void_p(workspace.data_ptr()), workspace.numel(), _stream(stream)))


def dpc_backtrack_shared(share, Topt, split, I, M, K, q_inst, q_T0, A, A_len, S, S_len, obj, lat,
                         status, stream=None):
    """dpc_backtrack with the stage-1 tables of network x // share serving instance x."""
    B, ld, _ = I.shape
    L, P, Q = ld - 1, M.shape[2], q_inst.shape[0]
    nt = (B + share - 1) // share
    if Q == 0:
        return
    i32 = torch.int32
    _check(_load_sweep().dpc_backtrack_shared(
        B, L, P, int(share), _dev(Topt, i32, (nt, ld, ld), "Topt"),
        _dev(split, torch.uint8, (nt, ld, ld), "split"), _dev(I, torch.float32, (B, ld, ld), "I"),
        _dev(M, torch.float32, (B, ld, P), "M"),
        None if K is None else _dev(K, torch.uint8, (B, ld, P), "K"), Q,
        _dev(q_inst, i32, (Q,), "q_inst"), _dev(q_T0, i32, (Q,), "q_T0"),
        _dev(A, i32, (Q, L), "A"), _dev(A_len, i32, (Q,), "A_len"),
        _dev(S, i32, (Q, L), "S"), _dev(S_len, i32, (Q,), "S_len"),
        _dev(obj, torch.float32, (Q,), "obj"), _dev(lat, i32, (Q,), "lat"),
        _dev(status, i32, (Q,), "status"), _stream(stream)))


def dpc_importance_shift(I_raw, alpha, I_out, mean_out=None, stream=None):
    """I_raw float32 [B][L+1][L+1] or [B][L+1][L+1][2][2], alpha float32 [n_alpha]
    -> I_out float32 [B*n_alpha][...] (table b*n_alpha+a), mean_out float64 [B] or None."""
    B, ld = I_raw.shape[0], I_raw.shape[1]
    tail = tuple(I_raw.shape[1:])
    if tail not in ((ld, ld), (ld, ld, 2, 2)):
        raise DpcError(f"I_raw: expected [B][L+1][L+1] or [B][L+1][L+1][2][2], got {tuple(I_raw.shape)}")
    F = 1 if len(tail) == 2 else 4
    n_alpha = alpha.shape[0]
    _check(_load_sweep().dpc_importance_shift(
        B, ld - 1, F, n_alpha, _dev(I_raw, torch.float32, (B,) + tail, "I_raw"),
        _dev(alpha, torch.float32, (n_alpha,), "alpha"),
        _dev(I_out, torch.float32, (B * n_alpha,) + tail, "I_out"),
        None if mean_out is None else _dev(mean_out, torch.float64, (B,), "mean_out"),
        _stream(stream)))


def dpc_front(M, front_t, front_obj, front_len, stream=None):
    """M float32 [B][rows][P] (last row read) -> front_t int32 / front_obj float32 [B][cap],
    front_len int32 [B]."""
    B, rows, P = M.shape
    cap = front_t.shape[1]
    _check(_load_sweep().dpc_front(
        B, rows - 1, P, _dev(M, torch.float32, (B, rows, P), "M"), cap,
        _dev(front_t, torch.int32, (B, cap), "front_t"),
        _dev(front_obj, torch.float32, (B, cap), "front_obj"),
        _dev(front_len, torch.int32, (B,), "front_len"), _stream(stream)))


def dpc_front_queries(front_t, front_len, q_inst, q_T0, q_count, stream=None):
    """front_t int32 [B][cap], front_len int32 [B] -> q_inst, q_T0 int32 [qcap], q_count int32 [1]."""
    B, cap = front_t.shape
    qcap = q_inst.shape[0]
    _check(_load_sweep().dpc_front_queries(
        B, cap, _dev(front_t, torch.int32, (B, cap), "front_t"),
        _dev(front_len, torch.int32, (B,), "front_len"), qcap,
        _dev(q_inst, torch.int32, (qcap,), "q_inst"), _dev(q_T0, torch.int32, (qcap,), "q_T0"),
        _dev(q_count, torch.int32, (1,), "q_count"), _stream(stream)))


def dpc_chain_latency(T, q_inst, X, X_len, lat, stream=None):
    """T int32 [B][L+1][L+1]; X int32 [Q][L] ascending sets with lengths X_len -> lat int32 [Q]."""
    B, ld, _ = T.shape
    L = ld - 1
    Q = q_inst.shape[0]
    if Q == 0:
        return
    _check(_load_sweep().dpc_chain_latency(
        B, L, _dev(T, torch.int32, (B, ld, ld), "T"), Q,
        _dev(q_inst, torch.int32, (Q,), "q_inst"), _dev(X, torch.int32, (Q, L), "X"),
        _dev(X_len, torch.int32, (Q,), "X_len"), _dev(lat, torch.int32, (Q,), "lat"),
        _stream(stream)))


# ---- small instances: stage 1 and stage 2 in one launch ----

def _load_fused():
    lib = load()
    if not getattr(lib, "_fused_ready", False):
        i32, vp = ctypes.c_int32, ctypes.c_void_p
        lib.dpc_stage12_fused_supported.argtypes = [i32, i32]
        lib.dpc_stage12_fused_supported.restype = ctypes.c_int
        lib.dpc_stage12_fused.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, vp, vp]
        lib.dpc_stage12_fused.restype = ctypes.c_int
        lib.dpc_solve_fused.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, vp, i32] + [vp] * 10
        lib.dpc_solve_fused.restype = ctypes.c_int
        lib._fused_ready = True
    return lib


def dpc_stage12_fused_supported(L, P):
    return bool(_load_fused().dpc_stage12_fused_supported(L, P))


def dpc_stage12_fused(T, I, Topt, split, M, K, stream=None):
    """T int32, I float32 [B][L+1][L+1] -> Topt, split, M, K (or None), one launch."""
    B, ld, _ = T.shape
    P = M.shape[2]
    shp = (B, ld, ld)
    _check(_load_fused().dpc_stage12_fused(
        B, ld - 1, P, _dev(T, torch.int32, shp, "T"), _dev(I, torch.float32, shp, "I"),
        _dev(Topt, torch.int32, shp, "Topt"), _dev(split, torch.uint8, shp, "split"),
        _dev(M, torch.float32, (B, ld, P), "M"),
        None if K is None else _dev(K, torch.uint8, (B, ld, P), "K"), _stream(stream)))


def dpc_solve_fused(T, I, Topt, split, M, K, q_inst, q_T0, A, A_len, S, S_len, obj, lat, status,
                    stream=None):
    """Stage 1, stage 2 and set recovery in one launch (small instances)."""
    B, ld, _ = T.shape
    L, P, Q = ld - 1, M.shape[2], q_inst.shape[0]
    shp = (B, ld, ld)
    i32 = torch.int32
    _check(_load_fused().dpc_solve_fused(
        B, L, P, _dev(T, i32, shp, "T"), _dev(I, torch.float32, shp, "I"),
        _dev(Topt, i32, shp, "Topt"), _dev(split, torch.uint8, shp, "split"),
        _dev(M, torch.float32, (B, ld, P), "M"),
        None if K is None else _dev(K, torch.uint8, (B, ld, P), "K"), Q,
        _dev(q_inst, i32, (Q,), "q_inst"), _dev(q_T0, i32, (Q,), "q_T0"),
        _dev(A, i32, (Q, L), "A"), _dev(A_len, i32, (Q,), "A_len"),
        _dev(S, i32, (Q, L), "S"), _dev(S_len, i32, (Q,), "S_len"),
        _dev(obj, torch.float32, (Q,), "obj"), _dev(lat, i32, (Q,), "lat"),
        _dev(status, i32, (Q,), "status"), _stream(stream)))


# queries per instance up to which the single launch beats a separate dpc_backtrack
ONE_LAUNCH_QUERIES_PER_INSTANCE = 32


def solve_fused(T, I, q_inst, q_T0, buf: "Buffers", stream=None, one_launch=None):
    """The small-instance path into the buffers of `buf`: one launch (dpc_solve_fused)
    when there are few queries per instance, else dpc_stage12_fused + dpc_backtrack.
    one_launch: True / False to force either."""
    Q = q_inst.shape[0]
    if one_launch is None:
        one_launch = 0 < Q <= ONE_LAUNCH_QUERIES_PER_INSTANCE * T.shape[0]
    if one_launch and Q > 0:
        dpc_solve_fused(T, I, buf.Topt, buf.split, buf.M, buf.K, q_inst, q_T0, buf.A, buf.A_len,
                        buf.S, buf.S_len, buf.obj, buf.lat, buf.status, stream)
        return
    dpc_stage12_fused(T, I, buf.Topt, buf.split, buf.M, buf.K, stream)
    dpc_backtrack(buf.Topt, buf.split, I, buf.M, buf.K, q_inst, q_T0, buf.A, buf.A_len, buf.S,
                  buf.S_len, buf.obj, buf.lat, buf.status, stream)
