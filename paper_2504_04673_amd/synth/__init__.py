"""Seeded synthetic workloads (host side, numpy + a small C helper library).

Only *inputs* are produced here: CSR graphs with GCN-normalised values and dense
matrices.  Nothing in this module implements the method under test; the CPU oracle and
the GPU library both consume these arrays.

The graphs take the shapes of the datasets in the paper's Table 3 and of the five
benchmark configurations; they contain no dataset content.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gen.c")
_LIB = os.path.join(_HERE, "libsynth.so")

# stream ids: one independent random stream per kind of input
STREAM_GRAPH, STREAM_H, STREAM_W, STREAM_G, STREAM_PERM = 1, 2, 3, 4, 5
INVALID = np.uint64(0xFFFFFFFFFFFFFFFF)


def build(force: bool = False) -> str:
    """Compile gen.c into libsynth.so (gcc, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-fopenmp", "-fPIC", "-shared", "-fvisibility=hidden",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _L():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        u64, i64, i32, u32, dbl, vp = (ctypes.c_uint64, ctypes.c_int64, ctypes.c_int32,
                                       ctypes.c_uint32, ctypes.c_double, ctypes.c_void_p)
        L.synth_ctr64.restype = u64
        L.synth_ctr64.argtypes = [u64, u64, u64]
        L.synth_uniform_f32.argtypes = [u64, u64, u64, i64, dbl, dbl, vp]
        L.synth_normal_f32.argtypes = [u64, u64, u64, i64, dbl, vp]
        L.synth_normal_rows_f32.argtypes = [u64, u64, vp, i64, i32, dbl, vp]
        L.synth_uniform_pairs.argtypes = [u64, u64, u64, i64, u32, vp]
        L.synth_relabel.restype = u32
        L.synth_relabel.argtypes = [u32, i32, u64]
        L.synth_rmat_pairs.argtypes = [u64, u64, u64, i64, i32, dbl, dbl, dbl, u32, u64, vp]
        L.synth_rmat_rowblock.restype = i64
        L.synth_rmat_rowblock.argtypes = [u64, u64, u64, i64, i32, dbl, dbl, dbl, u32, u64,
                                          u32, u32, vp, vp, i64]
        L.synth_sbm_pairs.argtypes = [u64, u64, u32, u32, dbl, dbl, i32, vp]
        L.synth_gcn_values.argtypes = [vp, vp, i64, i64, vp, vp]
        L.synth_keys_to_csr.argtypes = [vp, i64, i64, u32, vp, vp]
        for f in ("synth_uniform_f32", "synth_normal_f32", "synth_normal_rows_f32",
                  "synth_uniform_pairs", "synth_rmat_pairs", "synth_sbm_pairs",
                  "synth_gcn_values", "synth_keys_to_csr"):
            getattr(L, f).restype = None
        _lib = L
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


# --------------------------------------------------------------------------- dense inputs

def uniform(shape, seed: int, stream: int, lo=-1.0, hi=1.0) -> np.ndarray:
    out = np.empty(shape, dtype=np.float32)
    _L().synth_uniform_f32(seed, stream, 0, out.size, lo, hi, _p(out))
    return out


def normal(shape, seed: int, stream: int, scale=1.0) -> np.ndarray:
    out = np.empty(shape, dtype=np.float32)
    _L().synth_normal_f32(seed, stream, 0, out.size, scale, _p(out))
    return out


def normal_rows(rows: np.ndarray, f: int, seed: int, stream: int, scale=1.0) -> np.ndarray:
    """Rows `rows` of a virtual row-major N(0,1) matrix of width f (never stored whole)."""
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    out = np.empty((rows.size, f), dtype=np.float32)
    _L().synth_normal_rows_f32(seed, stream, _p(rows), rows.size, f, scale, _p(out))
    return out


# --------------------------------------------------------------------------- graphs

@dataclass
class CSR:
    """Row block of a sparse matrix: rows [row0, row0+m) of an n-column matrix."""
    m: int
    n: int
    rowptr: np.ndarray          # int32, m+1
    colidx: np.ndarray          # int32, nnz, ascending inside each row
    val: np.ndarray             # float32, nnz
    row0: int = 0
    meta: dict = field(default_factory=dict)

    @property
    def nnz(self) -> int:
        return int(self.rowptr[-1])

    def row_block(self, r0: int, r1: int) -> "CSR":
        s, e = int(self.rowptr[r0]), int(self.rowptr[r1])
        return CSR(r1 - r0, self.n, (self.rowptr[r0:r1 + 1] - s).astype(np.int32),
                   self.colidx[s:e].copy(), self.val[s:e].copy(), self.row0 + r0, dict(self.meta))


def block_offsets(n: int, parts: int) -> np.ndarray:
    """Contiguous block boundaries off[i] = floor(i*n/parts) (1D block distribution)."""
    return np.array([(i * n) // parts for i in range(parts + 1)], dtype=np.int64)


def _csr_from_undirected(und: np.ndarray, n: int, meta: dict) -> CSR:
    """und: unique keys (u<<32|v), u<v.  Symmetrise, add self loops, sort, normalise."""
    und = np.ascontiguousarray(und, dtype=np.uint64)
    u = und >> np.uint64(32)
    v = und & np.uint64(0xFFFFFFFF)
    diag = np.arange(n, dtype=np.uint64)
    keys = np.concatenate([und, (v << np.uint64(32)) | u, (diag << np.uint64(32)) | diag])
    del u, v, diag
    keys.sort()
    return _csr_from_directed_sorted(keys, n, n, 0, None, meta)


def _csr_from_directed_sorted(keys, m, n, row0, deg, meta) -> CSR:
    nnz = keys.size
    assert nnz < 2**31
    rowptr = np.empty(m + 1, dtype=np.int32)
    colidx = np.empty(nnz, dtype=np.int32)
    _L().synth_keys_to_csr(_p(keys), nnz, m, row0, _p(rowptr), _p(colidx))
    if deg is None:
        assert m == n and row0 == 0
        deg = np.diff(rowptr).astype(np.int32)
    val = np.empty(nnz, dtype=np.float32)
    _L().synth_gcn_values(_p(rowptr), _p(colidx), m, row0, _p(deg), _p(val))
    return CSR(m, n, rowptr, colidx, val, row0, meta)


def er_graph(n: int, avg_deg: float, seed: int) -> CSR:
    """Erdos-Renyi G(n, M) with M = n*avg_deg/2 distinct undirected edges, symmetrised,
    self loops added, GCN-normalised."""
    target = int(n * avg_deg / 2)
    keys = np.empty(0, dtype=np.uint64)
    start, batch = 0, max(1024, 2 * target)
    while True:
        b = np.empty(batch, dtype=np.uint64)
        _L().synth_uniform_pairs(seed, STREAM_GRAPH, start, batch, n, _p(b))
        start += batch
        keys = np.concatenate([keys, b[b != INVALID]])
        uniq, first = np.unique(keys, return_index=True)
        if uniq.size >= target:
            # keep the `target` pairs that were drawn first
            keep = np.sort(first)[:target]
            und = np.sort(keys[keep])
            break
    return _csr_from_undirected(und, n, {"kind": "er", "seed": seed})


def rmat_graph(n: int, target_nnz: int, seed: int, a=0.57, b=0.19, c=0.19,
               batch: int = 1 << 26) -> CSR:
    """R-MAT (a,b,c,d=1-a-b-c) on 2^scale >= n vertices with a seeded bijective relabel;
    draws with an endpoint >= n or u == v are rejected.  Draws are taken in batches until
    the number of distinct undirected edges reaches (target_nnz - n)/2.  If the last batch
    overshoots, the surplus is removed by dropping the edges with the largest hashed key
    (a seeded pseudo-random subset, so no vertex range is favoured).  Then: symmetrise,
    add self loops, GCN-normalise."""
    scale = max(1, int(np.ceil(np.log2(n))))
    want = max(0, (target_nnz - n) // 2)
    rk = int(_L().synth_ctr64(seed, STREAM_PERM, 0))
    und = np.empty(0, dtype=np.uint64)
    start = 0
    batch = int(min(batch, max(1 << 16, want)))
    while und.size < want:
        buf = np.empty(batch, dtype=np.uint64)
        _L().synth_rmat_pairs(seed, STREAM_GRAPH, start, batch, scale, a, b, c, n, rk, _p(buf))
        start += batch
        buf = np.unique(buf[buf != INVALID])
        und = np.union1d(und, buf) if und.size else buf
        if start > 400 * max(want, 1):
            break  # saturated (tiny n): accept what exists
    if und.size > want:
        mixed = _mix_np(und ^ np.uint64((seed * 0x9E3779B97F4A7C15) & 0xFFFFFFFFFFFFFFFF))
        keep = np.argpartition(mixed, want - 1)[:want] if want > 0 else np.empty(0, np.int64)
        und = np.sort(und[keep])
    return _csr_from_undirected(und, n, {"kind": "rmat", "seed": seed, "scale": scale,
                                         "draws": start})


def _mix_np(z: np.ndarray) -> np.ndarray:
    z = z.astype(np.uint64, copy=True)
    with np.errstate(over="ignore"):
        z += np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
    return z ^ (z >> np.uint64(31))


def rmat_rowblock(n: int, total_draws: int, r0: int, r1: int, seed: int,
                  a=0.57, b=0.19, c=0.19, chunk: int = 1 << 26, with_degrees=True) -> CSR:
    """Rows [r0,r1) of an R-MAT graph on n vertices that is never stored whole: the draws
    are streamed, only entries whose row is in the block are kept, and draw-level degrees
    of all n vertices are counted for the normalisation (duplicates outside the block are
    not removed from those degrees; the values only need to be positive and fixed)."""
    scale = max(1, int(np.ceil(np.log2(n))))
    rk = int(_L().synth_ctr64(seed, STREAM_PERM, 0))
    deg = np.zeros(n, dtype=np.int32) if with_degrees else None
    parts = []
    start = 0
    frac = min(1.0, 4.0 * (r1 - r0) / max(n, 1))
    while start < total_draws:
        cnt = int(min(chunk, total_draws - start))
        cap = int(max(1 << 16, 2 * cnt * frac))
        out = np.empty(cap, dtype=np.uint64)
        got = _L().synth_rmat_rowblock(seed, STREAM_GRAPH, start, cnt, scale, a, b, c, n, rk,
                                       r0, r1, None if deg is None else _p(deg), _p(out), cap)
        if got < 0:
            raise RuntimeError("rmat_rowblock: output capacity exceeded")
        parts.append(np.unique(out[:got]))
        start += cnt
    keys = np.unique(np.concatenate(parts)) if parts else np.empty(0, np.uint64)
    m = r1 - r0
    diag = np.arange(r0, r1, dtype=np.uint64)
    keys = np.union1d(keys, (diag << np.uint64(32)) | diag)
    if deg is None:
        deg = np.ones(n, dtype=np.int32)
    else:
        deg += 1  # the self loop
    return _csr_from_directed_sorted(np.ascontiguousarray(keys), m, n, r0, deg,
                                     {"kind": "rmat_rowblock", "seed": seed, "scale": scale,
                                      "draws": total_draws})


def sbm_graph(n: int, ncomm: int, mean_in: float, mean_out: float, seed: int,
              order: str = "community") -> CSR:
    """Stochastic block model with `ncomm` equal planted communities.

    order="community": vertices sorted by community label (what a partitioner would
    deliver); order="random": the same graph under a seeded random vertex permutation."""
    kmax = int(max(mean_in, mean_out) / 2 + 8 * np.sqrt(max(mean_in, mean_out) / 2) + 8)
    keys = np.empty(n * 2 * kmax, dtype=np.uint64)
    _L().synth_sbm_pairs(seed, STREAM_GRAPH, n, ncomm, mean_in, mean_out, kmax, _p(keys))
    keys = keys[keys != INVALID]
    und = np.unique(keys)
    del keys
    meta = {"kind": "sbm", "seed": seed, "order": order, "ncomm": ncomm}
    if order == "community":
        return _csr_from_undirected(und, n, meta)
    perm = random_permutation(n, seed)          # new id of vertex v is perm[v]
    u = perm[(und >> np.uint64(32)).astype(np.int64)].astype(np.uint64)
    v = perm[(und & np.uint64(0xFFFFFFFF)).astype(np.int64)].astype(np.uint64)
    lo, hi = np.minimum(u, v), np.maximum(u, v)
    und = np.sort((lo << np.uint64(32)) | hi)
    g = _csr_from_undirected(und, n, meta)
    g.meta["perm"] = perm
    return g


def sbm_labels(g: CSR) -> np.ndarray:
    """Community label of every vertex of an sbm_graph, in the graph's own vertex numbering
    (what a partitioner would hand back: the input of the reordering step)."""
    n, ncomm = g.n, int(g.meta["ncomm"])
    planted = (np.arange(n, dtype=np.int64) // (n // ncomm)).astype(np.int32)
    if g.meta.get("order") == "community":
        return planted
    labels = np.empty(n, dtype=np.int32)
    labels[g.meta["perm"]] = planted            # vertex v of the planted order became perm[v]
    return labels


def random_permutation(n: int, seed: int) -> np.ndarray:
    """Seeded permutation of [0,n): rank of a counter-based hash (ties broken by index)."""
    h = _mix_np(np.arange(n, dtype=np.uint64) ^ np.uint64(int(_L().synth_ctr64(seed, STREAM_PERM, 1))))
    order = np.argsort(h, kind="stable")
    perm = np.empty(n, dtype=np.int64)
    perm[order] = np.arange(n, dtype=np.int64)
    return perm


def ring_graph(n: int, d: int) -> CSR:
    """d-regular ring (d even): vertex i adjacent to i±1..i±d/2, unit values, no self loops."""
    assert d % 2 == 0 and d < n
    offs = np.array([k for k in range(-(d // 2), d // 2 + 1) if k != 0], dtype=np.int64)
    cols = (np.arange(n, dtype=np.int64)[:, None] + offs[None, :]) % n
    cols.sort(axis=1)
    rowptr = (np.arange(n + 1, dtype=np.int64) * d).astype(np.int32)
    return CSR(n, n, rowptr, cols.reshape(-1).astype(np.int32),
               np.ones(n * d, dtype=np.float32), 0, {"kind": "ring", "d": d})
