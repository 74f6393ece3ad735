"""Pins of the CPU oracle against things other than itself: brute force on tiny inputs,
closed forms, invariants, and library routines on special cases (CPU only)."""
import math

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from paper_2504_04673_amd import synth


def random_csr(m, n, density, rng, sort=True, dup=False):
    """Directed random CSR with arbitrary float values (NOT symmetric)."""
    rows = []
    rowptr = [0]
    for _ in range(m):
        k = rng.binomial(n, density)
        cols = rng.choice(n, size=k, replace=dup) if k else np.empty(0, np.int64)
        if sort:
            cols = np.sort(cols)
        rows.append(cols)
        rowptr.append(rowptr[-1] + k)
    colidx = np.concatenate(rows).astype(np.int32) if rowptr[-1] else np.empty(0, np.int32)
    val = rng.standard_normal(rowptr[-1]).astype(np.float32)
    return np.array(rowptr, np.int32), colidx, val


def dense_of(rowptr, colidx, val, n):
    m = rowptr.size - 1
    D = [[0.0] * n for _ in range(m)]
    for r in range(m):
        for e in range(rowptr[r], rowptr[r + 1]):
            D[r][int(colidx[e])] += float(val[e])
    return D


# ----------------------------------------------------------------------------- SpMM

@pytest.mark.parametrize("m,n,f,seed", [(1, 1, 1, 0), (7, 5, 3, 1), (33, 64, 17, 2), (64, 40, 8, 3)])
def test_spmm_bruteforce_dense(m, n, f, seed):
    """Definition of the product written as pure-Python loops over a dense copy of A.
    A is rectangular, non-symmetric and has duplicate entries in a row, so a transposed
    operand, a wrong index or a dropped duplicate would show."""
    rng = np.random.default_rng(seed)
    rowptr, colidx, val = random_csr(m, n, 0.3, rng, sort=False, dup=True)
    B = rng.standard_normal((n, f)).astype(np.float32)
    D = dense_of(rowptr, colidx, val, n)
    ref = np.zeros((m, f))
    for r in range(m):
        for c in range(f):
            ref[r, c] = math.fsum(D[r][k] * float(B[k, c]) for k in range(n))
    got, gabs = oracle.spmm(rowptr, colidx, val, B, want_abs=True)
    assert np.all(np.abs(got - ref) <= 1e-6 * gabs + 1e-30)
    # magnitude companion: sum |a||b|
    aref = np.abs(np.array(D))  # duplicates may cancel in D; bound from below only
    assert np.all(gabs + 1e-12 >= aref @ np.abs(B.astype(np.float64)) - 1e-9)


def test_spmm_identity_bit_exact():
    n, f = 257, 19
    rowptr = np.arange(n + 1, dtype=np.int32)
    colidx = np.arange(n, dtype=np.int32)
    val = np.ones(n, np.float32)
    H = synth.normal((n, f), 7, synth.STREAM_H)
    Z = oracle.spmm(rowptr, colidx, val, H)
    assert Z.tobytes() == H.tobytes()


@pytest.mark.parametrize("n,d,f", [(50, 2, 4), (101, 6, 5), (4096, 8, 16)])
def test_spmm_regular_ring_all_ones(n, d, f):
    """d-regular ring with unit weights times the all-ones matrix: every entry equals d."""
    g = synth.ring_graph(n, d)
    Z = oracle.spmm(g.rowptr, g.colidx, g.val, np.ones((n, f), np.float32))
    assert np.all(Z == np.float32(d))


def test_spmm_accumulate_adds_old_value():
    rng = np.random.default_rng(5)
    rowptr, colidx, val = random_csr(20, 30, 0.2, rng)
    B = rng.standard_normal((30, 6)).astype(np.float32)
    C0 = rng.standard_normal((20, 6)).astype(np.float32)
    Z = oracle.spmm(rowptr, colidx, val, B)
    Zacc = oracle.spmm(rowptr, colidx, val, B, C=C0)
    A = sp.csr_matrix((val.astype(np.float64), colidx, rowptr), shape=(20, 30))
    ref = C0.astype(np.float64) + A @ B.astype(np.float64)
    assert np.allclose(Zacc, ref, rtol=0, atol=1e-6)
    assert not np.allclose(Zacc, Z)


@pytest.mark.parametrize("kind", ["er", "rmat", "sbm"])
def test_spmm_gcn_eigenvector(kind):
    """For A = D^-1/2 (B+I) D^-1/2 the vector sqrt(d) is an eigenvector with eigenvalue 1.
    Holds at any size, so it also pins the generators' normalisation."""
    if kind == "er":
        g = synth.er_graph(4096, 8, 0)
    elif kind == "rmat":
        g = synth.rmat_graph(30000, 1_500_000, 3)
    else:
        g = synth.sbm_graph(32000, 16, 40, 2, 4, order="random")
    d = np.diff(g.rowptr).astype(np.float64)
    x = np.sqrt(d).astype(np.float32)
    X = np.stack([x, 2 * x, -x], axis=1).copy()
    Z, Zabs = oracle.spmm(g.rowptr, g.colidx, g.val, X, want_abs=True)
    assert np.all(np.abs(Z - X.astype(np.float64)) <= 4e-7 * Zabs)


def test_spmm_symmetry_and_scipy():
    g = synth.rmat_graph(5000, 200_000, 11)
    A = sp.csr_matrix((g.val.astype(np.float64), g.colidx, g.rowptr), shape=(g.m, g.n))
    assert abs(A - A.T).max() == 0.0          # generator gives a symmetric matrix
    X = synth.normal((g.n, 9), 1, synth.STREAM_H)
    Z, Zabs = oracle.spmm(g.rowptr, g.colidx, g.val, X, want_abs=True)
    ref = A @ X.astype(np.float64)
    assert np.all(np.abs(Z - ref) <= 2e-7 * Zabs + 1e-30)
    absref = abs(A) @ np.abs(X.astype(np.float64))
    assert np.allclose(Zabs, absref, rtol=1e-12)
    # x^T (A y) == y^T (A x)
    x, y = X[:, 0].astype(np.float64), X[:, 1].astype(np.float64)
    assert math.isclose(x @ Z[:, 1].astype(np.float64), y @ Z[:, 0].astype(np.float64), rel_tol=1e-5)


# ----------------------------------------------------------------------------- needed rows

def brute_nnzcols(rowptr, colidx, colblk):
    cols = set(int(c) for c in colidx[rowptr[0]:rowptr[-1]])
    out = []
    for q in range(len(colblk) - 1):
        out.append(sorted(c for c in cols if colblk[q] <= c < colblk[q + 1]))
    return out


@pytest.mark.parametrize("seed,m,n,nb", [(0, 10, 37, 1), (1, 25, 64, 4), (2, 40, 130, 7), (3, 5, 9, 9)])
def test_needed_rows_bruteforce(seed, m, n, nb):
    rng = np.random.default_rng(seed)
    rowptr, colidx, _ = random_csr(m, n, 0.08, rng, sort=False, dup=True)
    cuts = np.sort(rng.choice(np.arange(1, n), size=nb - 1, replace=False)) if nb > 1 else []
    colblk = np.array([0, *cuts, n], dtype=np.int64)
    needed, blk_off, compact = oracle.needed_rows(rowptr, colidx, n, colblk)
    ref = brute_nnzcols(rowptr, colidx, colblk)
    assert list(needed) == [c for blk in ref for c in blk]
    assert list(blk_off) == list(np.cumsum([0] + [len(b) for b in ref]))
    assert np.array_equal(needed[compact], colidx)


def test_needed_rows_empty_and_full():
    # no entries at all
    needed, blk_off, compact = oracle.needed_rows(np.zeros(4, np.int32), np.empty(0, np.int32), 10,
                                                  np.array([0, 5, 10]))
    assert needed.size == 0 and list(blk_off) == [0, 0, 0] and compact.size == 0
    # a full row: every column needed
    needed, blk_off, _ = oracle.needed_rows(np.array([0, 6], np.int32), np.arange(6, dtype=np.int32)[::-1].copy(),
                                            6, np.array([0, 2, 6]))
    assert list(needed) == [0, 1, 2, 3, 4, 5] and list(blk_off) == [0, 2, 6]


def test_needed_rows_cfg1_invariants_and_expectation(cfg1):
    """Configuration 1, P = 4 row blocks x 4 column blocks.  Invariants, plus the closed-form
    expectation for G(n,M): an off-diagonal 1024x1024 block holds ~Poisson(2) entries per
    column, so 1024*(1-exp(-2)) ~ 885 columns are non-empty; diagonal blocks contain the
    self loops, so all 1024 columns are needed."""
    g, _ = cfg1
    off = synth.block_offsets(g.n, 4)
    exp_off = 1024 * (1 - math.exp(-2.0))
    sd = math.sqrt(1024 * math.exp(-2.0) * (1 - math.exp(-2.0)))
    for i in range(4):
        blk = g.row_block(int(off[i]), int(off[i + 1]))
        needed, blk_off, compact = oracle.needed_rows(blk.rowptr, blk.colidx, g.n, off)
        assert np.all(np.diff(needed) > 0)
        assert set(needed.tolist()) == set(blk.colidx.tolist())
        assert np.array_equal(needed[compact], blk.colidx)
        for q in range(4):
            cnt = int(blk_off[q + 1] - blk_off[q])
            seg = needed[blk_off[q]:blk_off[q + 1]]
            assert np.all((seg >= off[q]) & (seg < off[q + 1]))
            if q == i:
                assert cnt == 1024
            else:
                assert abs(cnt - exp_off) < 5 * sd, (i, q, cnt)


def test_needed_rows_sbm_expectation():
    """Planted partition: needed-row count of the rank-0 block before / after reordering by
    community, against the Poisson closed forms (scaled-down configuration 5)."""
    n, k = 64000, 16
    blk = n // k
    for order, expect in (("random", n * (1 - math.exp(-(40 + 2) / k)) + 0.0),
                          ("community", None)):
        g = synth.sbm_graph(n, k, 40, 2, 0, order=order).row_block(0, blk)
        needed, blk_off, _ = oracle.needed_rows(g.rowptr, g.colidx, n, synth.block_offsets(n, k))
        if order == "random":
            # each column: self loop if inside the block, else hit by ~Poisson(42/16) entries
            e = blk + (n - blk) * (1 - math.exp(-42.0 / k))
            assert abs(needed.size - e) < 0.01 * e
        else:
            # own community: all needed; others: Poisson(2 * blk/(n-blk)) entries per column
            e = blk + (n - blk) * (1 - math.exp(-2.0 * blk / (n - blk)))
            assert abs(needed.size - e) < 0.02 * e
            assert blk_off[1] - blk_off[0] == blk


# ----------------------------------------------------------------------------- pack + packed path

def test_pack_rows_is_fancy_indexing(cfg1):
    g, H = cfg1
    rows = np.array([5, 5, 0, 4095, 17], np.int32)
    assert oracle.pack_rows(H, rows).tobytes() == H[rows].tobytes()
    assert oracle.pack_rows(H, np.empty(0, np.int32)).shape == (0, 16)


def test_packed_blocks_sum_to_one_shot(cfg1):
    """Sum over column blocks of A_iq * H[NnzCols(i,q)] (compact indices) equals A_i * H
    (block-sum equation of the 1D algorithm)."""
    g, H = cfg1
    off = synth.block_offsets(g.n, 4)
    for i in range(4):
        blk = g.row_block(int(off[i]), int(off[i + 1]))
        one_shot, zabs = oracle.spmm(blk.rowptr, blk.colidx, blk.val, H, want_abs=True)
        needed, blk_off, compact = oracle.needed_rows(blk.rowptr, blk.colidx, g.n, off)
        # single product through the compact buffer: identical summation order => identical bits
        Hn = oracle.pack_rows(H, needed)
        via = oracle.spmm(blk.rowptr, compact, blk.val, Hn)
        assert via.tobytes() == one_shot.tobytes()
        # block by block with accumulation
        Z = np.zeros_like(one_shot)
        for q in range(4):
            keep = (blk.colidx >= off[q]) & (blk.colidx < off[q + 1])
            rp = np.concatenate([[0], np.cumsum(np.add.reduceat(keep.astype(np.int64), blk.rowptr[:-1]) *
                                            (np.diff(blk.rowptr) > 0))]).astype(np.int32)
            ci = (compact[keep] - blk_off[q]).astype(np.int32)
            Hq = oracle.pack_rows(H, needed[blk_off[q]:blk_off[q + 1]])
            Z = oracle.spmm(rp, ci, blk.val[keep], Hq, C=Z)
        assert np.all(np.abs(Z - one_shot) <= 1e-6 * zabs + 1e-30)


# ----------------------------------------------------------------------------- GEMM, bf16

@pytest.mark.parametrize("m,k,n", [(1, 1, 1), (5, 7, 3), (33, 16, 48)])
@pytest.mark.parametrize("tx,tw", [(False, False), (False, True), (True, False)])
def test_gemm_vs_numpy_fp64(m, k, n, tx, tw):
    rng = np.random.default_rng(m * 100 + k)
    X = rng.standard_normal((k, m) if tx else (m, k)).astype(np.float32)
    W = rng.standard_normal((n, k) if tw else (k, n)).astype(np.float32)
    Xe = X.T if tx else X
    We = W.T if tw else W
    ref = Xe.astype(np.float64) @ We.astype(np.float64)
    Z, Zabs = oracle.gemm(X, W, transX=tx, transW=tw, want_abs=True)
    assert np.all(np.abs(Z - ref) <= 1e-7 * Zabs + 1e-30)
    assert np.allclose(Zabs, np.abs(Xe.astype(np.float64)) @ np.abs(We.astype(np.float64)), rtol=1e-12)


@pytest.mark.parametrize("tx,tw", [(False, False), (False, True), (True, False), (True, True)])
def test_gemm_magnitude_companion_with_given_scale(tx, tw):
    """The scale of the rounding-error bound can be handed down from an earlier product: with
    Xabs given, Zabs = op(Xabs) |op(W)| (numpy fp64, an independent evaluation), whatever X holds;
    without it, |op(X)| |op(W)|.  Non-square shapes so that a transposed index cannot pass."""
    rng = np.random.default_rng(17 + 2 * tx + tw)
    m, k, n = 6, 11, 4
    X = rng.standard_normal((k, m) if tx else (m, k)).astype(np.float32)
    W = rng.standard_normal((n, k) if tw else (k, n)).astype(np.float32)
    A = rng.random(X.shape) * 5.0 + 0.5                      # a scale unrelated to |X|
    Ae = A.T if tx else A
    We = np.abs((W.T if tw else W).astype(np.float64))
    Z, Zabs = oracle.gemm(X, W, transX=tx, transW=tw, Xabs=A, want_abs=True)
    assert np.allclose(Zabs, Ae @ We, rtol=1e-13, atol=0)
    Z0, Zabs0 = oracle.gemm(X, W, transX=tx, transW=tw, want_abs=True)
    assert np.array_equal(Z, Z0)                             # the scale never touches the product
    assert np.allclose(Zabs0, np.abs((X.T if tx else X).astype(np.float64)) @ We, rtol=1e-13, atol=0)
    assert not np.allclose(Zabs, Zabs0, rtol=1e-3)
    # bfloat16 mode: the handed-down scale multiplies the magnitudes of the ROUNDED weights
    _, Zb = oracle.gemm(X, W, bf16=True, transX=tx, transW=tw, Xabs=A, want_abs=True)
    Wb = np.abs(oracle.bf16_round(W).astype(np.float64))
    assert np.allclose(Zb, Ae @ (Wb.T if tw else Wb), rtol=1e-13, atol=0)


def test_layer_magnitude_companions_propagate_the_spmm_scale():
    """Tabs = |A||H|; Zabs = Tabs |W|; Sabs = |A||G|; Gabs = Sabs |W^T|; Yabs = |Hprev^T| |S| --
    each checked against dense numpy fp64 on a rectangular-feature, non-symmetric case."""
    rng = np.random.default_rng(33)
    n, fi, fo = 19, 7, 5
    rowptr, colidx, val = random_csr(n, n, 0.25, rng)
    A = np.abs(np.array(dense_of(rowptr, colidx, val, n)))
    H = rng.standard_normal((n, fi)).astype(np.float32)
    W = rng.standard_normal((fi, fo)).astype(np.float32)
    G = rng.standard_normal((n, fo)).astype(np.float32)
    Zp = rng.standard_normal((n, fi)).astype(np.float32)
    aW = np.abs(W.astype(np.float64))
    fwd = oracle.gcn_layer_fwd(rowptr, colidx, val, H, W, act=1)
    Tabs = A @ np.abs(H.astype(np.float64))
    assert np.allclose(fwd["Tabs"], Tabs, rtol=1e-13, atol=0)
    assert np.allclose(fwd["Zabs"], Tabs @ aW, rtol=1e-13, atol=0)
    assert not np.allclose(fwd["Zabs"], np.abs(fwd["T"].astype(np.float64)) @ aW, rtol=1e-3)
    bwd = oracle.gcn_layer_bwd(rowptr, colidx, val, G, W, Zp, H)
    Sabs = A @ np.abs(G.astype(np.float64))
    assert np.allclose(bwd["Sabs"], Sabs, rtol=1e-13, atol=0)
    assert np.allclose(bwd["Gabs"], Sabs @ aW.T, rtol=1e-13, atol=0)
    assert np.allclose(bwd["Yabs"], np.abs(H.astype(np.float64)).T @ np.abs(bwd["S"].astype(np.float64)),
                       rtol=1e-13, atol=0)


def test_bf16_round_known_values_and_torch():
    """bfloat16 keeps 8 significand bits; ties go to even."""
    one = np.float32(1.0)
    cases = {
        1.0: 1.0,
        1.0 + 2.0 ** -8: 1.0,                      # tie -> even (1.0)
        1.0 + 2.0 ** -8 + 2.0 ** -20: 1.0 + 2.0 ** -7,
        1.0 + 3 * 2.0 ** -8: 1.0 + 2.0 ** -6,      # tie -> even
        -(1.0 + 2.0 ** -7): -(1.0 + 2.0 ** -7),
        0.0: 0.0,
        3.3895313892515355e38: 3.3895313892515355e38,   # the largest finite bfloat16
        3.4028234663852886e38: float("inf"),             # largest float32: rounds up to inf
    }
    for x, y in cases.items():
        assert float(oracle.bf16_round(np.float32(x))) == y, x
    import torch
    v = synth.normal((4096,), 3, synth.STREAM_W, scale=37.0)
    ref = torch.from_numpy(v).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(oracle.bf16_round(v), ref)
    assert one == 1.0


def test_gemm_bf16_rounds_operands():
    rng = np.random.default_rng(0)
    X = rng.standard_normal((9, 20)).astype(np.float32)
    W = rng.standard_normal((20, 6)).astype(np.float32)
    Z = oracle.gemm(X, W, bf16=True)
    ref = oracle.bf16_round(X).astype(np.float64) @ oracle.bf16_round(W).astype(np.float64)
    assert np.allclose(Z, ref, rtol=1e-6, atol=1e-6)
    assert not np.allclose(Z, X.astype(np.float64) @ W.astype(np.float64), rtol=1e-6, atol=1e-6)


# ----------------------------------------------------------------------------- GCN layer

def test_gcn_layer_fwd_against_dense_numpy():
    rng = np.random.default_rng(9)
    rowptr, colidx, val = random_csr(24, 24, 0.2, rng)
    H = rng.standard_normal((24, 10)).astype(np.float32)
    W = rng.standard_normal((10, 7)).astype(np.float32)
    A = np.array(dense_of(rowptr, colidx, val, 24))
    out = oracle.gcn_layer_fwd(rowptr, colidx, val, H, W, act=1)
    T = A @ H.astype(np.float64)
    Z = T @ W.astype(np.float64)
    assert np.allclose(out["T"], T, atol=1e-5)
    assert np.allclose(out["Z"], Z, atol=1e-4)
    assert np.array_equal(out["H"], np.maximum(out["Z"], 0))
    assert np.array_equal(oracle.gcn_layer_fwd(rowptr, colidx, val, H, W, act=0)["H"], out["Z"])


def test_gcn_backward_finite_differences():
    """Two layers on a tiny NON-symmetric graph.  Loss L = <G2, Z2>.  The oracle's backward
    (given the transposed CSR, as the backward equation multiplies by the other orientation
    of the adjacency matrix) must match central finite differences of a dense fp64 forward."""
    rng = np.random.default_rng(21)
    n, f0, f1, f2 = 14, 5, 6, 4
    rowptr, colidx, val = random_csr(n, n, 0.3, rng)
    M = np.array(dense_of(rowptr, colidx, val, n))          # forward multiplies by M
    Mt = sp.csr_matrix(M.T)
    Mt.sort_indices()
    H0 = rng.standard_normal((n, f0)).astype(np.float32)
    W1 = rng.standard_normal((f0, f1)).astype(np.float32)
    W2 = rng.standard_normal((f1, f2)).astype(np.float32)
    G2 = rng.standard_normal((n, f2)).astype(np.float32)

    def loss(H0_, W1_, W2_):
        Z1 = M @ H0_ @ W1_
        H1 = np.maximum(Z1, 0)
        Z2 = M @ H1 @ W2_
        return float(np.sum(G2.astype(np.float64) * Z2))

    l1 = oracle.gcn_layer_fwd(rowptr, colidx, val, H0, W1, act=1)
    l2 = oracle.gcn_layer_fwd(rowptr, colidx, val, l1["H"], W2, act=0)
    tp, tc, tv = Mt.indptr.astype(np.int32), Mt.indices.astype(np.int32), Mt.data.astype(np.float32)
    b2 = oracle.gcn_layer_bwd(tp, tc, tv, G2, W2, l1["Z"], l1["H"])
    b1 = oracle.gcn_layer_bwd(tp, tc, tv, b2["Gprev"], W1, None, H0)

    def fd(arg, shape):
        g = np.zeros(shape)
        base = [H0.astype(np.float64), W1.astype(np.float64), W2.astype(np.float64)]
        eps = 1e-5
        for idx in np.ndindex(*shape):
            p = [b.copy() for b in base]
            q = [b.copy() for b in base]
            p[arg][idx] += eps
            q[arg][idx] -= eps
            g[idx] = (loss(*p) - loss(*q)) / (2 * eps)
        return g

    assert np.allclose(b2["Y"], fd(2, W2.shape), rtol=2e-4, atol=2e-4)
    assert np.allclose(b1["Y"], fd(1, W1.shape), rtol=2e-4, atol=2e-4)
    assert np.allclose(b1["Gprev"], fd(0, H0.shape), rtol=2e-4, atol=2e-4)
    _ = l2
