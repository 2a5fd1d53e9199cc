"""The stage-2 wave-window kernels compiled for the host (tests/host_emu) and
run under AddressSanitizer / UBSan, one workgroup at a time, one host thread
per lane: the kernels' own index arithmetic is exercised on the CPU, where an
out-of-bounds access is a test failure instead of a GPU fault, and the result
is compared bit for bit with the oracle.  (What the emulation cannot show:
anything that depends on the GPU's timing or on the inline assembly.)"""
import os
import shutil
import subprocess

import numpy as np
import pytest

import oracle
from helpers import rand_tables

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
EMU_DIR = os.path.join(HERE, "host_emu")


def _build(tmp_path_factory, main_cpp, name):
    if shutil.which("g++") is None:
        pytest.skip("no host compiler")
    exe = str(tmp_path_factory.mktemp(name) / name)
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-pthread",
           "-I", EMU_DIR, "-I", os.path.join(ROOT, "include"),
           "-I", os.path.join(ROOT, "paper_2301_12187_amd", "csrc"),
           "-x", "c++", "-o", exe, os.path.join(EMU_DIR, main_cpp)]
    subprocess.run(cmd, check=True)
    return exe


@pytest.fixture(scope="module")
def emu(tmp_path_factory):
    return _build(tmp_path_factory, "emu_main.cpp", "dpc_emu")


@pytest.fixture(scope="module")
def emu_fused(tmp_path_factory):
    return _build(tmp_path_factory, "emu_fused_main.cpp", "dpc_emu_fused")


def _run(emu, tmp_path, T, I, P, shape):
    B, ld, _ = T.shape
    Topt, split, M, K = oracle.solve_batch(T, I, P, want_K=True, threads=4)
    fin, fout = str(tmp_path / "in.bin"), str(tmp_path / "out.bin")
    with open(fin, "wb") as f:
        np.array([B, ld - 1, P, shape], np.int32).tofile(f)
        Topt.astype(np.int32).tofile(f)
        I.astype(np.float32).tofile(f)
    r = subprocess.run([emu, fin, fout], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-4000:]
    raw = np.fromfile(fout, np.uint8)
    n = B * ld * P
    Me = raw[:4 * n].view(np.float32).reshape(B, ld, P)
    Ke = raw[4 * n:].reshape(B, ld, P)
    assert (Me.view(np.uint32) == M.view(np.uint32)).all()
    assert (Ke == K).all()


# shape: 1 = groups of 8 rows, 4 waves; 5 = groups of 16 rows, 4 waves; 3 = 8 rows, 2 waves
@pytest.mark.parametrize("shape", [1, 5, 3])
def test_whole_groups_several_strips_ragged_tail(emu, tmp_path, shape):
    rng = np.random.default_rng(501)
    B, L, P = 2, 21, 1291                  # P not a multiple of 4, partial last group
    T, I = zip(*[rand_tables(rng, L, tmax=12, inf_frac=0.3, ikind="neg", span=9) for _ in range(B)])
    _run(emu, tmp_path, np.stack(T), np.stack(I), P, shape)


@pytest.mark.parametrize("shape", [1, 5])
def test_row_by_row_groups_and_missing_candidates(emu, tmp_path, shape):
    rng = np.random.default_rng(502)
    B, L, P = 2, 11, 1100
    Ts, Is = [], []
    for b in range(B):
        T, I = rand_tables(rng, L, tmax=5, ikind="mixed")
        ii, jj = np.triu_indices(L + 1, k=1)
        jump = rng.random(ii.size) < 0.3     # wildly different shifts: spreads beyond the window
        T[ii[jump], jj[jump]] = rng.integers(0, 1500, size=int(jump.sum()))
        Ts.append(T)
        Is.append(I)
    _run(emu, tmp_path, np.stack(Ts), np.stack(Is), P, shape)


@pytest.mark.parametrize("L,P", [(70, 260), (255, 40)])
def test_pairs_of_predecessors_long_chain(emu, tmp_path, L, P):
    """Groups of 16 rows with many rows below them (the five ring slots wrap
    many times, odd and even counts, the largest table of pair operands), with
    integer importances: exact ties inside and between pairs."""
    rng = np.random.default_rng(504 + L)
    T, I = rand_tables(rng, L, tmax=3, inf_frac=0.2, ikind="int")
    _run(emu, tmp_path, T[None], I[None], P, 5)


def _additive_tables(rng, B, L, lo, hi):
    """Latencies that add up along the chain (block latency about the sum of its
    layers), so that the shifts of one predecessor into a group of rows spread
    over several hundred columns."""
    Ts, Is = [], []
    for _ in range(B):
        T, I = rand_tables(rng, L, tmax=5, ikind="neg")
        base = rng.integers(lo, hi + 1, L)
        for i in range(L + 1):
            for j in range(i + 1, L + 1):
                T[i, j] = max(1, int(rng.uniform(0.7, 1.1) * base[i:j].sum()))
        Ts.append(T)
        Is.append(I)
    return np.stack(Ts), np.stack(Is)


# spreads of about 300 (three copies per window, two rows ahead), 600 (four
# copies, one row ahead) and beyond 764 (row by row) for groups of 8 rows;
# twice that for groups of 16
# (a table wider than a task also needs ghost columns, at most half a task:
#  the widest windows are reached with P = 1000, one task per group)
@pytest.mark.parametrize("shape,lo,hi,P", [(1, 35, 45, 1400), (1, 70, 90, 1000), (1, 55, 65, 1400),
                                           (5, 15, 22, 1400), (5, 35, 45, 1000), (2, 70, 90, 2100),
                                           (1, 120, 160, 1400)])
def test_windows_wider_than_the_smallest_ring_slot(emu, tmp_path, shape, lo, hi, P):
    rng = np.random.default_rng(503 + lo)
    T, I = _additive_tables(rng, 2, 19, lo, hi)
    _run(emu, tmp_path, T, I, P, shape)


# ---- the single-launch kernel for small instances (stage 1 + stage 2) ----

def _run_fused(emu_fused, tmp_path, T, I, P, lds_limit):
    """Stage 1, stage 2 and, in the same launch, set recovery at four budgets per
    instance plus one query that names no instance."""
    B, ld, _ = T.shape
    L = ld - 1
    Topt, split, M, K = oracle.solve_batch(T, I, P, want_K=True, threads=4)
    qi = np.concatenate([np.repeat(np.arange(B, dtype=np.int32), 4), [-1]]).astype(np.int32)
    qt = np.concatenate([np.tile(np.array([0, P // 3, P // 2, P - 1], np.int32), B), [0]]).astype(np.int32)
    Q = len(qi)
    fin, fout = str(tmp_path / "fin.bin"), str(tmp_path / "fout.bin")
    with open(fin, "wb") as f:
        np.array([B, L, P, lds_limit, Q], np.int32).tofile(f)
        T.astype(np.int32).tofile(f)
        I.astype(np.float32).tofile(f)
        qi.tofile(f)
        qt.tofile(f)
    r = subprocess.run([emu_fused, fin, fout], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-4000:]
    raw = np.fromfile(fout, np.uint8)
    n2, n = B * ld * ld, B * ld * P
    o = 0
    Te = raw[o:o + 4 * n2].view(np.int32).reshape(B, ld, ld); o += 4 * n2
    Se = raw[o:o + n2].reshape(B, ld, ld); o += n2
    Me = raw[o:o + 4 * n].view(np.float32).reshape(B, ld, P); o += 4 * n
    Ke = raw[o:o + n].reshape(B, ld, P); o += n
    assert (Te == Topt).all() and (Se == split).all()
    assert (Me.view(np.uint32) == M.view(np.uint32)).all()
    assert (Ke == K).all()
    Ae = raw[o:o + 4 * Q * L].view(np.int32).reshape(Q, L); o += 4 * Q * L
    Sse = raw[o:o + 4 * Q * L].view(np.int32).reshape(Q, L); o += 4 * Q * L
    small = raw[o:o + 16 * Q].view(np.int32).reshape(4, Q); o += 16 * Q
    obj = raw[o:o + 4 * Q].view(np.float32)
    for q in range(Q - 1):
        b = int(qi[q])
        ref = oracle.backtrack(Topt[b], split[b], I[b], M[b], K[b], int(qt[q]))
        assert small[3, q] == ref["status"] and small[0, q] == ref["A_len"] and small[1, q] == ref["S_len"]
        assert small[2, q] == ref["lat"]
        assert obj[q:q + 1].view(np.uint32)[0] == np.array([ref["obj"]], np.float32).view(np.uint32)[0]
        if ref["status"] == 0:
            assert list(Ae[q][:ref["A_len"]]) == list(ref["A"])
            assert list(Sse[q][:ref["S_len"]]) == list(ref["S"])
    assert small[3, Q - 1] == 2 and small[0, Q - 1] == -1 and small[2, Q - 1] == -1     # bad query


# lds_limit: 160 KB keeps every row of these shapes in LDS; the small limits
# leave room for a few rows only (4 and 1 resident rows plus the ring of three,
# then 20 resident rows, then 2 resident rows, two columns per thread and several batches per row), the rest
# is read back from the output array
@pytest.mark.parametrize("L,P,lds_limit", [(1, 1, 163840), (7, 100, 163840), (21, 333, 163840),
                                           (21, 333, 8 * 22 * 22 + 7 * 334 * 4),
                                           (13, 1291, 8 * 14 * 14 + 4 * 1292 * 4),
                                           (40, 70, 8 * 41 * 41 + 41 * 41 * 4),
                                           (63, 1291, 8 * 64 * 64 + 5 * 1292 * 4),
                                           (63, 130, 163840)])
def test_fused_small_kernel(emu_fused, tmp_path, L, P, lds_limit):
    rng = np.random.default_rng(600 + L + P)
    B = 2
    T, I = zip(*[rand_tables(rng, L, tmax=12, inf_frac=0.3, ikind="neg", span=9) for _ in range(B)])
    T, I = np.stack(T), np.stack(I)
    if L >= 7:
        T[1, 0, 3] = 5000                    # a shift beyond every budget
        I[1, 2, 5] = -np.inf                 # an excluded block
    _run_fused(emu_fused, tmp_path, T, I, P, lds_limit)
