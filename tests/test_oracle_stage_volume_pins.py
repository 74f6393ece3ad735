"""Pins of the oracle's 1.5D stage loop, column-block split, sparsity-oblivious plan and volume
statistics (CPU only): the figures printed in the paper's Table 2, hand-computed tiny cases,
pure-Python brute force and the dense product."""
import os

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from tests.test_oracle_pins import dense_of, random_csr

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def table2_rows():
    rows = []
    for line in open(os.path.join(GOLDEN, "table2_amazon_metis.txt")):
        line = line.strip()
        if line and not line.startswith("#"):
            p, avg, mx, imb = line.split()
            rows.append((int(p), float(avg), float(mx), float(imb)))
    return rows


@pytest.mark.parametrize("p,avg_mb,max_mb,imb", table2_rows())
def test_volume_imbalance_matches_table2(p, avg_mb, max_mb, imb):
    """Table 2 prints average MB, max MB and imbalance % for f = 300.  Build a count matrix
    whose per-process received volumes have exactly that average and maximum (process 0 gets
    the maximum, the others share the rest) and check that the oracle reports the printed
    imbalance (within the rounding of the printed one-decimal figures)."""
    f, eb = 300, 4
    row_b = f * eb
    max_rows = int(round(max_mb * 1e6 / row_b))
    rest_rows = int(round((avg_mb * p - max_mb) * 1e6 / row_b / (p - 1)))
    counts = np.zeros((p, p), dtype=np.int64)
    counts[0, 1] = max_rows                       # everything process 0 receives comes from P(1)
    for i in range(1, p):
        counts[i, (i + 1) % p if (i + 1) % p != i else 0] = rest_rows
    counts[np.arange(p), np.arange(p)] = 123456   # diagonal must not count
    st = oracle.volume_stats(counts, f, eb)
    assert abs(st["avg_bytes"] / 1e6 - avg_mb) < 0.06
    assert abs(st["max_recv_bytes"] / 1e6 - max_mb) < 0.06
    # one-decimal rounding of avg and max moves the ratio by up to ~0.05/avg + 0.05/max relative
    slack = 100.0 * (max_mb / avg_mb) * (0.05 / avg_mb + 0.05 / max_mb) + 0.06
    assert abs(st["recv_imbalance_pct"] - imb) <= slack


def test_volume_stats_hand_case():
    """3 processes, f = 2, 4-byte elements (8 bytes per row), counted by hand:
    received rows: P0 = 1+2 = 3, P1 = 4+0 = 4, P2 = 5+6 = 11; sent rows: P0 = 4+5 = 9,
    P1 = 1+6 = 7, P2 = 2+0 = 2; total 18 rows = 144 B; average 48 B; cut = 6 rows."""
    counts = [[9, 1, 2], [4, 9, 0], [5, 6, 9]]
    st = oracle.volume_stats(counts, 2, 4)
    assert st["total_bytes"] == 144 and st["avg_bytes"] == 48
    assert st["max_recv_bytes"] == 88 and st["max_send_bytes"] == 72
    assert st["recv_imbalance_pct"] == pytest.approx((88 / 48 - 1) * 100)
    assert st["send_imbalance_pct"] == pytest.approx(50.0)
    assert st["cut_rows"] == 6 and st["cut_bytes"] == 48
    z = oracle.volume_stats(np.diag([5, 5]), 16)
    assert z["total_bytes"] == 0 and z["recv_imbalance_pct"] == 0 and z["cut_rows"] == 0


def test_volume_counts_from_plan_equal_bruteforce_sets():
    """counts[i][q] taken from the plan's block offsets equal the sizes of brute-force sets."""
    rng = np.random.default_rng(5)
    n, P = 60, 4
    rowptr, colidx, val = random_csr(n, n, 0.05, rng)
    blk = np.array([0, 13, 13, 40, 60], dtype=np.int64)   # ragged, one empty block
    counts = np.zeros((P, P), dtype=np.int64)
    for i in range(P):
        a, b = rowptr[blk[i]], rowptr[blk[i + 1]]
        rp = (rowptr[blk[i]:blk[i + 1] + 1] - a).astype(np.int32)
        _, off, _ = oracle.needed_rows(rp, colidx[a:b], n, blk)
        counts[i] = np.diff(off)
        for q in range(P):
            brute = {int(c) for c in colidx[a:b] if blk[q] <= c < blk[q + 1]}
            assert counts[i, q] == len(brute)
    ob = oracle.volume_stats(np.tile(np.diff(blk), (P, 1)), 8)   # oblivious: whole blocks
    aw = oracle.volume_stats(counts, 8)
    assert aw["total_bytes"] <= ob["total_bytes"]


def test_oblivious_plan_is_identity():
    colidx = np.array([3, 0, 3, 5], dtype=np.int32)
    needed, off, compact = oracle.needed_rows_oblivious(colidx, 7, [0, 2, 7])
    assert needed.tolist() == list(range(7)) and off.tolist() == [0, 2, 7]
    assert compact.tolist() == colidx.tolist()


@pytest.mark.parametrize("seed,sort", [(0, True), (1, False)])
def test_split_colblocks_bruteforce(seed, sort):
    """Pure-Python scan of every entry: block membership, relative column, stable order."""
    rng = np.random.default_rng(seed)
    m, n = 23, 50
    rowptr, colidx, val = random_csr(m, n, 0.3, rng, sort=sort, dup=True)
    bounds = [5, 5, 17, 30, 44]          # drops columns < 5 and >= 44; one empty block
    blocks = oracle.split_colblocks(rowptr, colidx, val, bounds)
    assert len(blocks) == 4
    for q, (rp, ci, va) in enumerate(blocks):
        exp_rp, exp_ci, exp_va = [0], [], []
        for r in range(m):
            for e in range(rowptr[r], rowptr[r + 1]):
                if bounds[q] <= colidx[e] < bounds[q + 1]:
                    exp_ci.append(int(colidx[e]) - bounds[q])
                    exp_va.append(val[e])
            exp_rp.append(len(exp_ci))
        assert rp.tolist() == exp_rp and ci.tolist() == exp_ci
        assert np.array_equal(va, np.array(exp_va, dtype=np.float32))


def test_stage_loop_equals_dense_product_of_selected_blocks():
    """Alg. 2's partial sum over the stages q of A_iq H_q equals the dense product with the
    columns of the other blocks zeroed (Eq. for the 1.5D partial sum)."""
    rng = np.random.default_rng(11)
    m, n, f = 19, 64, 5
    rowptr, colidx, val = random_csr(m, n, 0.2, rng, sort=True)
    H = rng.standard_normal((n, f)).astype(np.float32)
    colblk = np.array([0, 16, 30, 30, 51, 64], dtype=np.int64)
    needed, off, compact = oracle.needed_rows(rowptr, colidx, n, colblk)
    blocks = oracle.split_colblocks(rowptr, compact, val, off)
    stages = [1, 3, 4]                                   # a rank's share of the column blocks
    rows = [needed[off[q]:off[q + 1]] for q in stages]
    Z, Zabs = oracle.stage_loop([blocks[q] for q in stages], rows, H, m, want_abs=True)
    D = np.array(dense_of(rowptr, colidx, val, n))
    keep = np.zeros(n, dtype=bool)
    for q in stages:
        keep[colblk[q]:colblk[q + 1]] = True
    ref = (D * keep[None, :]) @ H.astype(np.float64)
    assert np.all(np.abs(Z - ref) <= 1e-6 * Zabs + 1e-30)
    full = oracle.stage_loop(blocks, [needed[off[q]:off[q + 1]] for q in range(5)], H, m)
    assert np.allclose(full, D @ H.astype(np.float64), rtol=0, atol=1e-5)


@pytest.mark.parametrize("seed,sort,dup", [(0, True, False), (1, False, True), (2, False, False)])
def test_transpose_bruteforce_and_scipy(seed, sort, dup):
    """Entry-by-entry definition in pure Python (rows ascending, stored order inside a row), the
    dense transpose, and scipy's CSR->CSC conversion where the matrix has no duplicates."""
    rng = np.random.default_rng(seed)
    m, n = 17, 29
    rowptr, colidx, val = random_csr(m, n, 0.25, rng, sort=sort, dup=dup)
    rpt, cit, vat = oracle.transpose_csr(rowptr, colidx, val, n)
    exp = [[] for _ in range(n)]
    for r in range(m):
        for e in range(rowptr[r], rowptr[r + 1]):
            exp[int(colidx[e])].append((r, val[e]))
    assert rpt.tolist() == [0] + list(np.cumsum([len(x) for x in exp]))
    assert cit.tolist() == [r for x in exp for r, _ in x]
    assert np.array_equal(vat, np.array([v for x in exp for _, v in x], dtype=np.float32))
    D = np.array(dense_of(rowptr, colidx, val, n))
    Dt = np.array(dense_of(rpt, cit, vat, m))
    assert np.array_equal(Dt, D.T)
    if not dup:
        A = sp.csr_matrix((val, colidx, rowptr), shape=(m, n))
        T = A.tocsc()                       # CSC of A = CSR of A^T, row ids ascending per column
        T.sort_indices()
        assert np.array_equal(T.indptr, rpt) and np.array_equal(T.indices, cit) and np.array_equal(T.data, vat)


def test_transpose_twice_is_identity_for_sorted_rows():
    rng = np.random.default_rng(4)
    rowptr, colidx, val = random_csr(40, 33, 0.2, rng, sort=True)
    rpt, cit, vat = oracle.transpose_csr(rowptr, colidx, val, 33)
    rp2, ci2, va2 = oracle.transpose_csr(rpt, cit, vat, 40)
    assert np.array_equal(rp2, rowptr) and np.array_equal(ci2, colidx) and np.array_equal(va2, val)
    empty = oracle.transpose_csr(np.zeros(4, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32), 5)
    assert empty[0].tolist() == [0] * 6 and empty[1].size == 0


# ----------------------------------------------------------------------------- reordering

@pytest.mark.parametrize("n,n_parts,seed", [(1, 1, 0), (13, 3, 1), (40, 7, 2), (64, 64, 3)])
def test_perm_from_labels_bruteforce(n, n_parts, seed):
    """Renumbering by part label, written out as Python loops: part 0's vertices first in their
    old order, then part 1's, ...  (Sec. 5 / 6.1: every part owns a contiguous range)."""
    rng = np.random.default_rng(seed)
    labels = rng.integers(0, n_parts, size=n)
    perm, inv, off = oracle.perm_from_labels(labels, n_parts)
    expect = [v for q in range(n_parts) for v in range(n) if labels[v] == q]
    assert list(perm) == expect
    assert all(inv[perm[i]] == i for i in range(n))
    assert list(off) == [sum(1 for v in range(n) if labels[v] < q) for q in range(n_parts + 1)]


@pytest.mark.parametrize("seed,dup", [(0, False), (1, True), (2, False)])
def test_permute_symmetric_against_dense_and_product(seed, dup):
    """B = P A P^T: dense copies agree entry by entry (B[i][j] = A[perm[i]][perm[j]]), rows come
    out ascending, the product commutes with the renumbering ((P A P^T)(P x) = P (A x)) and the
    inverse permutation gives A back bit for bit.  A is non-symmetric, so a transposed result or
    perm used in place of inv fails."""
    rng = np.random.default_rng(seed)
    n = 23
    rowptr, colidx, val = random_csr(n, n, 0.2, rng, sort=True, dup=dup)
    if dup:                                          # duplicates adjacent, as a sorted row stores them
        for r in range(n):
            colidx[rowptr[r]:rowptr[r + 1]].sort()
    labels = rng.integers(0, 4, size=n)
    perm, inv, _ = oracle.perm_from_labels(labels, 4)
    rpp, cip, vap = oracle.permute_symmetric(rowptr, colidx, val, inv)
    A = np.array(dense_of(rowptr, colidx, val, n))
    B = np.array(dense_of(rpp, cip, vap, n))
    for i in range(n):
        for j in range(n):
            assert B[i][j] == pytest.approx(A[perm[i]][perm[j]], abs=1e-12)
        assert np.all(np.diff(cip[rpp[i]:rpp[i + 1]]) >= 0)
    assert rpp[-1] == rowptr[-1]
    x = rng.standard_normal((n, 3)).astype(np.float32)
    lhs = oracle.spmm(rpp, cip, vap, x[perm])
    rhs = oracle.spmm(rowptr, colidx, val, x)[perm]
    assert np.allclose(lhs, rhs, rtol=1e-6, atol=1e-6)
    # undo: permuting B with the inverse map (old id of new vertex i is perm[i]) restores A
    rp2, ci2, va2 = oracle.permute_symmetric(rpp, cip, vap, perm)
    assert np.array_equal(rp2, rowptr) and np.array_equal(ci2, colidx) and va2.tobytes() == val.tobytes()
    # stored values travel with their entries (not re-derived): multiset of values per new row
    for i in range(n):
        old = perm[i]
        assert sorted(vap[rpp[i]:rpp[i + 1]].tolist()) == sorted(val[rowptr[old]:rowptr[old + 1]].tolist())
