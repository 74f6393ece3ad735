"""The five benchmark configurations as seeded synthetic inputs (host arrays).

Each stands in for a dataset of the paper's Table 3 (same vertex count / density class, no
dataset content): cfg2 ~ Reddit-shaped, cfg3 ~ a products-scale power-law graph, cfg4 ~ one
rank's share of a Papers-sized graph, cfg5 ~ a partitioned graph (planted communities).
`scale` < 1 shrinks vertex and entry counts proportionally for tests.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

from . import synth


@dataclass
class Workload:
    name: str
    g: synth.CSR                 # the row block this GPU owns (all columns)
    colblk: np.ndarray           # column-block boundaries for the needed-row plan
    f: int
    H: np.ndarray = None         # n x f dense input (None when virtual, see H_rows)
    W: np.ndarray = None
    extra: dict = field(default_factory=dict)

    def H_rows(self, rows: np.ndarray) -> np.ndarray:
        """Rows of the (possibly virtual) dense input."""
        if self.H is not None:
            return self.H[rows]
        return synth.normal_rows(rows, self.f, self.extra["seed"], synth.STREAM_H)


def cfg1(seed=0) -> Workload:
    g = synth.er_graph(4096, 8, seed)
    H = synth.uniform((4096, 16), seed, synth.STREAM_H)
    return Workload("cfg1", g, synth.block_offsets(4096, 4), 16, H, None, {"P": 4, "seed": seed})


def cfg2(seed=0, scale=1.0, f=128) -> Workload:
    n = max(64, int(232_965 * scale))
    nnz = max(n, int(114_000_000 * scale))
    g = synth.rmat_graph(n, nnz, seed)
    H = synth.normal((n, f), seed, synth.STREAM_H)
    W = synth.normal((f, f), seed, synth.STREAM_W, scale=1 / np.sqrt(f))
    return Workload("cfg2", g, np.array([0, n], np.int64), f, H, W, {"seed": seed})


def cfg3(seed=0, scale=1.0, f=128) -> Workload:
    n = max(64, int(2_450_000 * scale))
    nnz = max(n, int(124_000_000 * scale))
    g = synth.rmat_graph(n, nnz, seed)
    H = synth.normal((n, f), seed, synth.STREAM_H)
    W = synth.normal((f, f), seed, synth.STREAM_W, scale=1 / np.sqrt(f))
    return Workload("cfg3", g, np.array([0, n], np.int64), f, H, W, {"seed": seed})


def cfg4(seed=0, scale=1.0, f=128) -> Workload:
    """Rank 0 of P=64: rows [0, n/64) x all columns of an R-MAT graph with n = 111,059,956
    vertices and ~0.8e9 undirected edges; 16 column blocks; H is virtual (rows on demand)."""
    n = max(4096, int(111_059_956 * scale))
    und_target = int(0.8e9 * scale)
    sc = int(np.ceil(np.log2(n)))
    accept = (n / 2.0 ** sc) ** 2
    draws = int(und_target / accept)
    r1 = n // 64
    g = synth.rmat_rowblock(n, draws, 0, r1, seed)
    return Workload("cfg4", g, synth.block_offsets(n, 16), f, None, None,
                    {"seed": seed, "P": 64, "c": 4, "draws": draws})


def cfg5(seed=0, scale=1.0, f=256, order="community") -> Workload:
    """Planted-partition graph, 16 communities; `order` = "random" (before reordering) or
    "community" (after).  g is the WHOLE graph; rank 0's block is g.row_block(0, n/16)."""
    n = max(1600, int(2_000_000 * scale)) // 16 * 16
    g = synth.sbm_graph(n, 16, 40, 2, seed, order=order)
    H = synth.normal((n, f), seed, synth.STREAM_H)
    W1 = synth.normal((f, f), seed, synth.STREAM_W, scale=1 / np.sqrt(f))
    W2 = synth.normal((f, f), seed + 1, synth.STREAM_W, scale=1 / np.sqrt(f))
    G2 = synth.normal((n, f), seed, synth.STREAM_G)
    return Workload("cfg5", g, synth.block_offsets(n, 16), f, H, W1,
                    {"seed": seed, "W2": W2, "G2": G2, "order": order})


def byte_models(m, n, nnz, N, f, f_out, nb=1):
    """Algorithmic bytes / flops of each step for one pass (what the method itself must move)."""
    plan = nnz * 4 + nnz * 4 + N * 4 + 2 * ((n + 7) // 8)
    pack = N * f * 4 * 2 + N * 4
    spmm = nnz * 8 + (m + 1) * 4 + N * f * 4 + m * f * 4
    gemm = m * f * 4 + f * f_out * 4 + m * f_out * 4
    return {"plan_bytes": plan, "pack_bytes": pack, "spmm_bytes": spmm, "gemm_bytes": gemm,
            "spmm_flops": 2 * nnz * f, "gemm_flops": 2 * m * f * f_out,
            "spmm_gather_bytes": nnz * f * 4}
