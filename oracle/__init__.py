"""CPU oracle -- TEST INFRASTRUCTURE ONLY (ctypes front end of sagnn_oracle.c).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this package.
It does not import, and is not imported by, the GPU package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sagnn_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.run(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                        "-fvisibility=hidden", "-o", _LIB, _SRC, "-lm"], check=True)
    return _LIB


_lib = None


def _declare(L):
    """Argument and result types of the library's entry points."""
    i64, i32, vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p
    L.oracle_needed_rows.restype = i64
    L.oracle_needed_rows.argtypes = [vp, vp, i64, i64, vp, i32, vp, vp, vp]
    L.oracle_pack_rows.restype = None
    L.oracle_pack_rows.argtypes = [vp, i64, i32, vp, i64, vp, i64]
    L.oracle_spmm.restype = None
    L.oracle_spmm.argtypes = [vp, vp, vp, i64, vp, i64, i32, vp, i64, i32, vp]
    L.oracle_gemm.restype = None
    L.oracle_gemm.argtypes = [vp, i64, i32, vp, i64, i32, i64, i64, i64, i32, vp, i64, vp, vp]
    L.oracle_gcn_layer_fwd.restype = None
    L.oracle_gcn_layer_fwd.argtypes = [vp, vp, vp, i64, vp, i64, i32, vp, i32, i32, i32,
                                       vp, vp, vp, vp, vp]
    L.oracle_gcn_layer_bwd.restype = None
    L.oracle_gcn_layer_bwd.argtypes = [vp, vp, vp, i64, vp, i32, vp, i32, vp, vp, i32,
                                       vp, vp, vp, vp, vp, vp]
    L.oracle_bf16_round.restype = ctypes.c_float
    L.oracle_bf16_round.argtypes = [ctypes.c_float]
    L.oracle_max_threads.restype = i32
    return L


def _L():
    global _lib
    if _lib is None:
        build()
        _lib = _declare(ctypes.CDLL(_LIB))
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dt):
    a = np.ascontiguousarray(a, dtype=dt)
    return a


def max_threads() -> int:
    return int(_L().oracle_max_threads())


def needed_rows(rowptr, colidx, n, colblk, want_compact=True):
    """NnzCols for every column block of a row block.  Returns (needed, blk_off, compact)."""
    rowptr, colidx = _c(rowptr, np.int32), _c(colidx, np.int32)
    colblk = _c(colblk, np.int64)
    m, nb = rowptr.size - 1, colblk.size - 1
    needed = np.empty(max(n, 1), dtype=np.int32)
    blk_off = np.empty(nb + 1, dtype=np.int64)
    compact = np.empty(max(colidx.size, 1), dtype=np.int32) if want_compact else None
    N = _L().oracle_needed_rows(_p(rowptr), _p(colidx), m, n, _p(colblk), nb, _p(needed),
                                _p(blk_off), _p(compact))
    if N < 0:
        raise ValueError(f"oracle_needed_rows failed ({N})")
    return needed[:N].copy(), blk_off, (compact[:colidx.size] if want_compact else None)


def pack_rows(H, rows):
    H = _c(H, np.float32)
    rows = _c(rows, np.int32)
    f = H.shape[1]
    out = np.empty((rows.size, f), dtype=np.float32)
    _L().oracle_pack_rows(_p(H), H.shape[1], f, _p(rows), rows.size, _p(out), f)
    return out


def spmm(rowptr, colidx, val, B, C=None, want_abs=False):
    """C (+)= A*B, fp64 accumulate.  Returns C or (C, Cabs)."""
    rowptr, colidx, val = _c(rowptr, np.int32), _c(colidx, np.int32), _c(val, np.float32)
    B = _c(B, np.float32)
    m, f = rowptr.size - 1, B.shape[1]
    acc = C is not None
    out = np.array(C, dtype=np.float32, order="C", copy=True) if acc else np.empty((m, f), np.float32)
    assert out.shape == (m, f)
    ab = np.empty((m, f), dtype=np.float64) if want_abs else None
    _L().oracle_spmm(_p(rowptr), _p(colidx), _p(val), m, _p(B), f, f, _p(out), f, int(acc), _p(ab))
    return (out, ab) if want_abs else out


def gemm(X, W, bf16=False, transX=False, transW=False, Xabs=None, want_abs=False):
    X, W = _c(X, np.float32), _c(W, np.float32)
    m, k = (X.shape[1], X.shape[0]) if transX else X.shape
    n = W.shape[0] if transW else W.shape[1]
    assert (W.shape[1] if transW else W.shape[0]) == k
    Z = np.empty((m, n), dtype=np.float32)
    ab = np.empty((m, n), dtype=np.float64) if want_abs else None
    if Xabs is not None:
        Xabs = _c(Xabs, np.float64)
        assert Xabs.shape == X.shape
    _L().oracle_gemm(_p(X), X.shape[1], int(transX), _p(W), W.shape[1], int(transW), m, k, n,
                     int(bf16), _p(Z), n, _p(Xabs), _p(ab))
    return (Z, ab) if want_abs else Z


def gcn_layer_fwd(rowptr, colidx, val, H, W, act=1, bf16=False):
    """Returns dict(T, Z, H, Tabs, Zabs)."""
    rowptr, colidx, val = _c(rowptr, np.int32), _c(colidx, np.int32), _c(val, np.float32)
    H, W = _c(H, np.float32), _c(W, np.float32)
    m, fi, fo = rowptr.size - 1, H.shape[1], W.shape[1]
    assert W.shape[0] == fi
    T = np.empty((m, fi), np.float32)
    Z = np.empty((m, fo), np.float32)
    Ho = np.empty((m, fo), np.float32)
    Tabs = np.empty((m, fi), np.float64)
    Zabs = np.empty((m, fo), np.float64)
    _L().oracle_gcn_layer_fwd(_p(rowptr), _p(colidx), _p(val), m, _p(H), fi, fi, _p(W), fo,
                              int(act), int(bf16), _p(T), _p(Z), _p(Ho), _p(Tabs), _p(Zabs))
    return dict(T=T, Z=Z, H=Ho, Tabs=Tabs, Zabs=Zabs)


def gcn_layer_bwd(rowptr, colidx, val, G, W, Zprev, Hprev, bf16=False, want_gprev=True):
    """Returns dict(S, Gprev, Y, Sabs, Gabs, Yabs).  W is f_in x f_out, G is m x f_out."""
    rowptr, colidx, val = _c(rowptr, np.int32), _c(colidx, np.int32), _c(val, np.float32)
    G, W, Hprev = _c(G, np.float32), _c(W, np.float32), _c(Hprev, np.float32)
    m, fo = G.shape
    fi = W.shape[0]
    assert W.shape[1] == fo and Hprev.shape == (m, fi)
    Zp = None if Zprev is None else _c(Zprev, np.float32)
    assert Zp is None or Zp.shape == (m, fi)
    S = np.empty((m, fo), np.float32)
    Gp = np.empty((m, fi), np.float32) if want_gprev else None
    Y = np.empty((fi, fo), np.float32)
    Sabs = np.empty((m, fo), np.float64)
    Gabs = np.empty((m, fi), np.float64) if want_gprev else None
    Yabs = np.empty((fi, fo), np.float64)
    _L().oracle_gcn_layer_bwd(_p(rowptr), _p(colidx), _p(val), m, _p(G), fo, _p(W), fi, _p(Zp),
                              _p(Hprev), int(bf16), _p(S), _p(Gp), _p(Y), _p(Sabs), _p(Gabs),
                              _p(Yabs))
    return dict(S=S, Gprev=Gp, Y=Y, Sabs=Sabs, Gabs=Gabs, Yabs=Yabs)


def bf16_round(x):
    x = np.asarray(x, dtype=np.float32)
    out = np.empty_like(x)
    flat_in, flat_out = x.reshape(-1), out.reshape(-1)
    L = _L()
    for i in range(flat_in.size):
        flat_out[i] = L.oracle_bf16_round(float(flat_in[i]))
    return out


# ---------------------------------------------------------------------------------------------
# 1.5D stage loop, sparsity-oblivious plan and volume statistics (plain numpy / Python)

def needed_rows_oblivious(colidx, n, colblk):
    """Plan of the sparsity-oblivious algorithm (Sec. 4.1: a process transfers its whole block
    row of H): every column is needed.  Returns (needed, blk_off, compact) like needed_rows."""
    colblk = np.asarray(colblk, dtype=np.int64)
    return (np.arange(n, dtype=np.int32), colblk.copy(),
            np.array(colidx, dtype=np.int32, copy=True))


def split_colblocks(rowptr, colidx, val, bounds):
    """The column blocks A_iq of a row block (Sec. 4.2): for every q the CSR of the entries
    with bounds[q] <= column < bounds[q+1], columns made relative to bounds[q], stored order
    kept.  Returns a list of (rowptr_q, colidx_q, val_q)."""
    rowptr = np.asarray(rowptr, dtype=np.int64)
    colidx = np.asarray(colidx, dtype=np.int64)
    val = np.asarray(val, dtype=np.float32)
    bounds = np.asarray(bounds, dtype=np.int64)
    m = rowptr.size - 1
    row_of = np.repeat(np.arange(m, dtype=np.int64), np.diff(rowptr))
    out = []
    for q in range(bounds.size - 1):
        sel = (colidx >= bounds[q]) & (colidx < bounds[q + 1])     # boolean mask keeps order
        cnt = np.bincount(row_of[sel], minlength=m)
        rp = np.zeros(m + 1, dtype=np.int32)
        rp[1:] = np.cumsum(cnt)
        out.append((rp, (colidx[sel] - bounds[q]).astype(np.int32), val[sel].copy()))
    return out


def stage_loop(blocks, rows_per_stage, H, m, want_abs=False):
    """Alg. 2, loop over the stages of one rank: for each stage take the rows NnzCols(i,q) of
    H (here: pack them), then Z^ <- Z^ + SpMM(A_iq, H^).  `blocks[k]` = (rowptr, colidx, val)
    with column ids = positions in stage k's packed rows; `rows_per_stage[k]` = those rows.
    Returns Z (float32) or (Z, Zabs) with Zabs = sum over stages of |A_iq| |H^|."""
    f = np.asarray(H).shape[1]
    Z = np.zeros((m, f), dtype=np.float32)
    Zabs = np.zeros((m, f), dtype=np.float64)
    for (rp, ci, va), rows in zip(blocks, rows_per_stage):
        T = pack_rows(H, rows)
        if want_abs:
            Z, ab = spmm(rp, ci, va, T, C=Z, want_abs=True)
            Zabs += ab
        else:
            Z = spmm(rp, ci, va, T, C=Z)
    return (Z, Zabs) if want_abs else Z


def volume_stats(counts, f, elem_bytes=4):
    """Data moved by one SpMM (Sec. 4.1 cost paragraph, Sec. 5 / Table 2).  counts[i][q] =
    |NnzCols(i,q)|: rows of H_q that P(i) receives; the diagonal is local.  A process's volume
    is what it receives (or sends) from all others; imbalance % = (max / average - 1) * 100;
    cut_P = largest off-diagonal count."""
    c = np.array(counts, dtype=np.float64)
    P = c.shape[0]
    off = c.copy()
    np.fill_diagonal(off, 0.0)
    row_bytes = float(f) * float(elem_bytes)
    recv = off.sum(axis=1) * row_bytes
    send = off.sum(axis=0) * row_bytes
    total = recv.sum()
    avg = total / P
    imb = lambda mx: (mx / avg - 1.0) * 100.0 if avg > 0 else 0.0
    return {"total_bytes": total, "avg_bytes": avg, "max_recv_bytes": recv.max(),
            "recv_imbalance_pct": imb(recv.max()), "max_send_bytes": send.max(),
            "send_imbalance_pct": imb(send.max()), "cut_rows": off.max(),
            "cut_bytes": off.max() * row_bytes}


def transpose_csr(rowptr, colidx, val, n):
    """CSR of A^T (Sec. 2.1: the forward pass uses A^T, the backward pass A).  Entry (r, c, v) of
    A becomes entry (c, r, v); inside a row of A^T the entries are ordered by r, entries of one
    row of A that repeat a column keep their stored order.  That is a stable sort of the entries
    by column (library sort as the step), the row ids and values carried along."""
    rowptr = np.asarray(rowptr, dtype=np.int64)
    colidx = np.asarray(colidx, dtype=np.int64)
    val = np.asarray(val, dtype=np.float32)
    m = rowptr.size - 1
    row_of = np.repeat(np.arange(m, dtype=np.int64), np.diff(rowptr))
    perm = np.argsort(colidx, kind="stable")
    rpt = np.zeros(n + 1, dtype=np.int64)
    rpt[1:] = np.cumsum(np.bincount(colidx, minlength=n)[:n])
    return rpt.astype(np.int32), row_of[perm].astype(np.int32), val[perm].copy()


def perm_from_labels(labels, n_parts):
    """Renumbering by partition label (Sec. 5, Sec. 6.1): the vertices of part 0 first, then
    part 1, ...; inside a part the old order is kept (a stable sort, library sort as the step).
    Returns (perm, inv, part_off): perm[i] = old id of new vertex i, inv[v] = new id of v."""
    labels = np.asarray(labels, dtype=np.int64)
    n = labels.size
    perm = np.argsort(labels, kind="stable")
    inv = np.empty(n, dtype=np.int64)
    inv[perm] = np.arange(n, dtype=np.int64)
    off = np.zeros(n_parts + 1, dtype=np.int64)
    off[1:] = np.cumsum(np.bincount(labels, minlength=n_parts)[:n_parts])
    return perm.astype(np.int32), inv.astype(np.int32), off


def permute_symmetric(rowptr, colidx, val, inv):
    """B = P A P^T for a square CSR matrix: entry (r, c, v) of A becomes entry (inv[r], inv[c], v)
    of B; the entries of B are listed by row, inside a row by column, entries that repeat a
    position in their stored order (a stable sort of the relabelled coordinate list)."""
    rowptr = np.asarray(rowptr, dtype=np.int64)
    colidx = np.asarray(colidx, dtype=np.int64)
    val = np.asarray(val, dtype=np.float32)
    inv = np.asarray(inv, dtype=np.int64)
    n = rowptr.size - 1
    row_of = np.repeat(np.arange(n, dtype=np.int64), np.diff(rowptr))
    nr, nc = inv[row_of], inv[colidx]
    order = np.lexsort((nc, nr))                      # by new row, then new column; stable
    rpp = np.zeros(n + 1, dtype=np.int64)
    rpp[1:] = np.cumsum(np.bincount(nr, minlength=n)[:n])
    return rpp.astype(np.int32), nc[order].astype(np.int32), val[order].copy()
