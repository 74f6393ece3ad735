"""GPU parity of the entry points around the 1.5D stage loop: sparsity-oblivious plan,
column-block split, stage loop (one and two streams) and volume statistics, against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2504_04673_amd as sagnn
from paper_2504_04673_amd import synth
from tests.test_oracle_pins import random_csr
from tests.util import assert_close, dev

pytestmark = pytest.mark.gpu

RTOL_SPMM = 1e-5


def row_block(g, i, P=4):
    off = synth.block_offsets(g.n, P)
    return g.row_block(int(off[i]), int(off[i + 1])), off


def test_oblivious_plan_cfg1(cfg1):
    g, H = cfg1
    blk, off = row_block(g, 1)
    rp, ci, v = dev(blk.rowptr), dev(blk.colidx), dev(blk.val)
    plan = sagnn.spmm_plan_needed_rows(rp, ci, g.n, off, oblivious=True, validate=True)
    needed, blk_off, compact = oracle.needed_rows_oblivious(blk.colidx, g.n, off)
    assert np.array_equal(plan.blk_off, blk_off)
    assert np.array_equal(plan.needed.cpu().numpy(), needed)
    assert np.array_equal(plan.colidx_compact.cpu().numpy(), compact)
    # the oblivious path moves every row and computes the same product
    Hd = dev(H)
    T = sagnn.spmm_pack_rows(Hd, plan.needed)
    assert T.cpu().numpy().tobytes() == H.tobytes()
    Z = sagnn.spmm_csr_tallskinny(rp, plan.colidx_compact, v, T)
    ref, zabs = oracle.spmm(blk.rowptr, blk.colidx, blk.val, H, want_abs=True)
    assert_close(Z, ref, zabs, RTOL_SPMM, "oblivious Z")


def check_split(rowptr, colidx, val, bounds):
    got = sagnn.spmm_split_colblocks(dev(rowptr), dev(colidx), dev(val), bounds)
    torch.cuda.synchronize()
    exp = oracle.split_colblocks(rowptr, colidx, val, bounds)
    off = np.concatenate([[0], np.cumsum([b[1].size for b in exp])])
    assert np.array_equal(got.nnz_off, off)
    for q, (rp, ci, va) in enumerate(exp):
        grp, gci, gva = got.block(q)
        assert np.array_equal(grp.cpu().numpy(), rp), q
        assert np.array_equal(gci.cpu().numpy(), ci), q
        assert gva.cpu().numpy().tobytes() == va.tobytes(), q
    return got


@pytest.mark.parametrize("case", ["cfg1_global", "cfg1_compact", "unsorted_dup_ragged", "many_blocks",
                                  "hub_row", "empty"])
def test_split_colblocks(case, cfg1):
    g, _ = cfg1
    rng = np.random.default_rng(3)
    if case == "cfg1_global":
        check_split(g.rowptr, g.colidx, g.val, synth.block_offsets(g.n, 4))
    elif case == "cfg1_compact":
        blk, off = row_block(g, 2)
        needed, blk_off, compact = oracle.needed_rows(blk.rowptr, blk.colidx, g.n, off)
        check_split(blk.rowptr, compact, blk.val, blk_off)
    elif case == "unsorted_dup_ragged":
        rowptr, colidx, val = random_csr(300, 500, 0.1, rng, sort=False, dup=True)
        check_split(rowptr, colidx, val, [7, 7, 100, 101, 333, 480])      # drops both ends
    elif case == "many_blocks":
        rowptr, colidx, val = random_csr(257, 4000, 0.05, rng, sort=False)
        check_split(rowptr, colidx, val, np.linspace(0, 4000, 201).astype(np.int64))   # 200 blocks
    elif case == "hub_row":
        # one row of 5000 entries spanning several 64-entry steps per block, then short rows
        hub = np.sort(rng.choice(20000, size=5000, replace=False))
        rows = [hub] + [np.sort(rng.choice(20000, size=3, replace=False)) for _ in range(40)]
        rowptr = np.concatenate([[0], np.cumsum([r.size for r in rows])]).astype(np.int32)
        colidx = np.concatenate(rows).astype(np.int32)
        val = rng.standard_normal(colidx.size).astype(np.float32)
        check_split(rowptr, colidx, val, [0, 5000, 10000, 15000, 20000])
    else:
        z = np.zeros(0, dtype=np.int32)
        got = sagnn.spmm_split_colblocks(dev(np.zeros(6, np.int32)), dev(z), dev(z.astype(np.float32)),
                                         [0, 10, 20])
        assert got.nnz_off.tolist() == [0, 0, 0] and int(got.rowptr_blk.abs().sum()) == 0


def stage_inputs(blk, n, colblk, H, stages, prepare):
    rp, ci, v = dev(blk.rowptr), dev(blk.colidx), dev(blk.val)
    plan = sagnn.spmm_plan_needed_rows(rp, ci, n, colblk)
    cb = sagnn.spmm_split_colblocks(rp, plan.colidx_compact, v, plan.blk_off)
    needed, off, compact = oracle.needed_rows(blk.rowptr, blk.colidx, n, colblk)
    assert np.array_equal(plan.blk_off, off)
    oblocks = oracle.split_colblocks(blk.rowptr, compact, blk.val, off)
    glist, olist, orows = [], [], []
    for q in stages:
        brp, bci, bva = cb.block(q)
        rows = plan.needed[int(off[q]):int(off[q + 1])]
        st = {"rowptr": brp, "colidx": bci, "val": bva, "rows": rows}
        if prepare and bci.numel():
            st["ws"] = sagnn.spmm_csr_prepare(brp, bci, bva, rows.numel(), H.shape[1])
        glist.append(st)
        olist.append(oblocks[q])
        orows.append(needed[off[q]:off[q + 1]])
    cap = max(int(np.diff(off).max()), 1)
    return glist, olist, orows, cap


@pytest.mark.parametrize("two_streams", [False, True])
@pytest.mark.parametrize("stages,prepare", [([0, 1, 2, 3], False), ([1, 3], True), ([2], False), ([], False)])
def test_stage_loop_cfg1(cfg1, stages, prepare, two_streams):
    """Row block 0 of configuration 1 (P = 4): partial sums over a rank's stages (Alg. 2)."""
    g, H = cfg1
    blk, off = row_block(g, 0)
    f = H.shape[1]
    glist, olist, orows, cap = stage_inputs(blk, g.n, off, H, stages, prepare)
    Hd = dev(H)
    T0 = torch.empty((cap, f), dtype=torch.float32, device="cuda")
    T1 = torch.empty((cap, f), dtype=torch.float32, device="cuda")
    Z = torch.full((blk.m, f), 7.0, dtype=torch.float32, device="cuda")
    side = torch.cuda.Stream() if two_streams else None
    sagnn.spmm_stage_loop(glist, blk.m, Hd, T0, T1, Z, accumulate_first=False, pack_stream=side)
    torch.cuda.synchronize()
    if not stages:
        assert float(Z.min()) == 7.0 and float(Z.max()) == 7.0      # nothing to do: Z untouched
        return
    ref, zabs = oracle.stage_loop(olist, orows, H, blk.m, want_abs=True)
    assert_close(Z, ref, zabs, RTOL_SPMM, f"stage loop {stages}")
    # accumulate_first = 1 adds to what Z holds
    Z2 = torch.full((blk.m, f), 0.5, dtype=torch.float32, device="cuda")
    sagnn.spmm_stage_loop(glist, blk.m, Hd, T0, T1, Z2, accumulate_first=True, pack_stream=side)
    torch.cuda.synchronize()
    assert_close(Z2, ref.astype(np.float64) + 0.5, zabs + 0.5, RTOL_SPMM, "stage loop accumulate")


def test_stage_loop_with_empty_block_and_capacity_error():
    rng = np.random.default_rng(8)
    m, n, f = 200, 1000, 64
    rowptr, colidx, val = random_csr(m, n, 0.02, rng)
    colidx = np.where((colidx >= 250) & (colidx < 500), colidx + 250, colidx).astype(np.int32)  # block 1 empty
    order = np.argsort(np.repeat(np.arange(m), np.diff(rowptr)) * n + colidx, kind="stable")
    colidx, val = colidx[order], val[order]
    H = rng.standard_normal((n, f)).astype(np.float32)

    class B:  # minimal stand-in for a CSR block
        pass
    blk = B()
    blk.rowptr, blk.colidx, blk.val, blk.m = rowptr, colidx, val, m
    colblk = np.array([0, 250, 500, 750, 1000], dtype=np.int64)
    glist, olist, orows, cap = stage_inputs(blk, n, colblk, H, [0, 1, 2, 3], False)
    assert orows[1].size == 0
    Hd = dev(H)
    T0 = torch.empty((cap, f), dtype=torch.float32, device="cuda")
    T1 = torch.empty((cap, f), dtype=torch.float32, device="cuda")
    Z = torch.empty((m, f), dtype=torch.float32, device="cuda")
    sagnn.spmm_stage_loop(glist, m, Hd, T0, T1, Z, pack_stream=torch.cuda.Stream())
    torch.cuda.synchronize()
    ref, zabs = oracle.stage_loop(olist, orows, H, m, want_abs=True)
    assert_close(Z, ref, zabs, RTOL_SPMM, "stage loop with an empty block")
    with pytest.raises(sagnn.SagnnError) as e:
        sagnn.spmm_stage_loop(glist, m, Hd, T0[:1], T1[:1], Z)
    assert e.value.code == -2


def test_volume_stats_cfg1_all_row_blocks(cfg1):
    """Counts |NnzCols(i,q)| of all P = 4 row blocks from the GPU plan; statistics from the
    library against the oracle's, sparsity-aware and sparsity-oblivious."""
    g, _ = cfg1
    P = 4
    counts = np.zeros((P, P), dtype=np.int64)
    ocounts = np.zeros((P, P), dtype=np.int64)
    for i in range(P):
        blk, off = row_block(g, i)
        plan = sagnn.spmm_plan_needed_rows(dev(blk.rowptr), dev(blk.colidx), g.n, off, want_compact=False)
        counts[i] = np.diff(plan.blk_off)
        ocounts[i] = np.diff(oracle.needed_rows(blk.rowptr, blk.colidx, g.n, off, want_compact=False)[1])
    assert np.array_equal(counts, ocounts)
    for c in (counts, np.tile(np.diff(off), (P, 1))):
        got = sagnn.spmm_volume_stats(c, 16)
        exp = oracle.volume_stats(c, 16)
        for k, v in exp.items():
            assert got[k] == pytest.approx(v, rel=1e-12), k
    aware, obl = sagnn.spmm_volume_stats(counts, 16), sagnn.spmm_volume_stats(np.tile(np.diff(off), (P, 1)), 16)
    assert aware["total_bytes"] < obl["total_bytes"] and aware["cut_rows"] <= 1024


def check_transpose(rowptr, colidx, val, n):
    rpt, cit, vat = sagnn.spmm_csr_transpose(dev(rowptr), dev(colidx), dev(val), n)
    torch.cuda.synchronize()
    erp, eci, eva = oracle.transpose_csr(rowptr, colidx, val, n)
    assert np.array_equal(rpt.cpu().numpy(), erp)
    assert np.array_equal(cit.cpu().numpy(), eci)
    assert vat.cpu().numpy().tobytes() == eva.tobytes()
    return rpt, cit, vat


@pytest.mark.parametrize("case", ["cfg1", "rect_unsorted_dup", "hub_and_empty", "three_passes", "four_passes",
                                  "one_column", "empty"])
def test_csr_transpose(case, cfg1):
    g, _ = cfg1
    rng = np.random.default_rng(12)
    if case == "cfg1":
        rpt, cit, vat = check_transpose(g.rowptr, g.colidx, g.val, g.n)
        # the normalised adjacency matrix is symmetric: its transpose is itself
        assert np.array_equal(rpt.cpu().numpy(), g.rowptr) and np.array_equal(cit.cpu().numpy(), g.colidx)
    elif case == "rect_unsorted_dup":
        rowptr, colidx, val = random_csr(700, 300, 0.05, rng, sort=False, dup=True)
        check_transpose(rowptr, colidx, val, 300)
    elif case == "hub_and_empty":
        hub = np.sort(rng.choice(60000, size=9000, replace=False))
        rows = [np.empty(0, np.int64), hub, np.empty(0, np.int64)] + \
               [np.sort(rng.choice(60000, size=5, replace=False)) for _ in range(3000)]
        rowptr = np.concatenate([[0], np.cumsum([r.size for r in rows])]).astype(np.int32)
        colidx = np.concatenate(rows).astype(np.int32)
        val = rng.standard_normal(colidx.size).astype(np.float32)
        check_transpose(rowptr, colidx, val, 60000)
    elif case in ("three_passes", "four_passes"):
        n = 5_000_000 if case == "three_passes" else 20_000_000        # 23 and 25 column bits
        nnz = 300_000
        cols = rng.integers(0, n, size=nnz)
        cols[:3] = [0, n - 1, n - 1]
        cuts = np.sort(rng.integers(0, nnz + 1, size=999))
        rowptr = np.array([0, *cuts, nnz], dtype=np.int32)
        check_transpose(rowptr, cols.astype(np.int32), rng.standard_normal(nnz).astype(np.float32), n)
    elif case == "one_column":
        rowptr = np.arange(0, 5001, dtype=np.int32)
        check_transpose(rowptr, np.zeros(5000, np.int32), rng.standard_normal(5000).astype(np.float32), 1)
    else:
        z = np.zeros(0, dtype=np.int32)
        rpt, cit, vat = sagnn.spmm_csr_transpose(dev(np.zeros(8, np.int32)), dev(z), dev(z.astype(np.float32)), 11)
        assert rpt.cpu().numpy().tolist() == [0] * 12
        bad = np.array([0, 5, 11], dtype=np.int32)           # column 11 is outside [0, 11)
        with pytest.raises(sagnn.SagnnError) as e:
            sagnn.spmm_csr_transpose(dev(np.array([0, 3], np.int32)), dev(bad), dev(np.ones(3, np.float32)), 11)
        assert e.value.code == -3


def test_directed_graph_layer_uses_both_orientations():
    """Directed graph: the forward product runs on A^T (Sec. 2.1 forward equation), the backward
    product on A.  A^T comes from the device transpose; both layer calls against the oracle."""
    rng = np.random.default_rng(21)
    n, f_in, f_out = 900, 64, 32
    rowptr, colidx, val = random_csr(n, n, 0.02, rng, sort=True)
    H = rng.standard_normal((n, f_in)).astype(np.float32)
    W = (rng.standard_normal((f_in, f_out)) / 8).astype(np.float32)
    G = rng.standard_normal((n, f_out)).astype(np.float32)
    rp, ci, va = dev(rowptr), dev(colidx), dev(val)
    rpt, cit, vat = sagnn.spmm_csr_transpose(rp, ci, va, n)
    T, Z, Ho = sagnn.gcn_layer_fwd(rpt, cit, vat, dev(H), dev(W), act=sagnn.ACT_RELU)
    ot = oracle.transpose_csr(rowptr, colidx, val, n)
    of = oracle.gcn_layer_fwd(ot[0], ot[1], ot[2], H, W, act=1)
    assert_close(T, of["T"], of["Tabs"], RTOL_SPMM, "directed T")
    assert_close(Z, of["Z"], of["Zabs"], 1e-5, "directed Z")
    assert_close(Ho, of["H"], of["Zabs"], 1e-5, "directed H'")
    Zprev = rng.standard_normal((n, f_in)).astype(np.float32)     # stand-in for Z^{l-1} (mask source)
    S, Gp, Y = sagnn.gcn_layer_bwd(rp, ci, va, dev(G), dev(W), dev(Zprev), dev(H))
    ob = oracle.gcn_layer_bwd(rowptr, colidx, val, G, W, Zprev, H)
    assert_close(S, ob["S"], ob["Sabs"], RTOL_SPMM, "directed S")
    assert_close(Gp, ob["Gprev"], ob["Gabs"], 1e-5, "directed Gprev")
    assert_close(Y, ob["Y"], ob["Yabs"], 1e-5, "directed Y")


# ------------------------------------------------------------------------------------ reordering

@pytest.mark.parametrize("case", ["cfg1_random_labels", "sbm_communities", "unsorted_dup", "one_part", "tiny"])
def test_reorder_by_labels_and_permute_symmetric(case, cfg1):
    """Renumbering by partition labels and the symmetric permutation of A (Sec. 5 / 6.1), bit for
    bit against the oracle; then the product in the new numbering, moved back with the inverse
    row gather, against the oracle's product in the old numbering."""
    rng = np.random.default_rng(len(case))
    if case == "cfg1_random_labels":
        g, _ = cfg1
        rowptr, colidx, val, n, parts = g.rowptr, g.colidx, g.val, g.n, 4
        labels = rng.integers(0, parts, size=n).astype(np.int32)
    elif case == "sbm_communities":
        g = synth.sbm_graph(8000, 16, 20, 2, 5, order="random")
        rowptr, colidx, val, n, parts = g.rowptr, g.colidx, g.val, g.n, 16
        labels = synth.sbm_labels(g)
    elif case == "unsorted_dup":
        n, parts = 3001, 7
        rowptr, colidx, val = random_csr(n, n, 0.004, rng, sort=False, dup=True)
        labels = rng.integers(0, parts, size=n).astype(np.int32)
        labels[labels == 3] = 4                       # an empty part
    elif case == "one_part":
        n, parts = 513, 1
        rowptr, colidx, val = random_csr(n, n, 0.02, rng)
        labels = np.zeros(n, np.int32)
    else:
        n, parts = 1, 1
        rowptr, colidx, val = np.array([0, 1], np.int32), np.array([0], np.int32), np.array([2.0], np.float32)
        labels = np.zeros(1, np.int32)
    perm, inv, off = sagnn.spmm_perm_from_labels(dev(labels), parts)
    operm, oinv, ooff = oracle.perm_from_labels(labels, parts)
    assert np.array_equal(perm.cpu().numpy(), operm) and np.array_equal(inv.cpu().numpy(), oinv)
    assert np.array_equal(off, ooff)
    rp, ci, v = dev(rowptr), dev(colidx), dev(val)
    rpp, cip, vap = sagnn.spmm_csr_permute_symmetric(rp, ci, v, inv)
    torch.cuda.synchronize()
    orp, oci, ova = oracle.permute_symmetric(rowptr, colidx, val, oinv)
    assert np.array_equal(rpp.cpu().numpy(), orp)
    assert np.array_equal(cip.cpu().numpy(), oci)
    assert vap.cpu().numpy().tobytes() == ova.tobytes()
    # product in the new numbering, moved back: Z_old = pack(Z_new, inv), H_new = pack(H, perm)
    f = 32
    H = synth.normal((n, f), 3, synth.STREAM_H)
    Hn = sagnn.spmm_pack_rows(dev(H), perm)
    Zn = sagnn.spmm_csr_tallskinny(rpp, cip, vap, Hn)
    Z = sagnn.spmm_pack_rows(Zn, inv)
    torch.cuda.synchronize()
    ref, zabs = oracle.spmm(rowptr, colidx, val, H, want_abs=True)
    assert_close(Z, ref, zabs, RTOL_SPMM, f"reordered product {case}")


def test_reorder_rejects_bad_labels_and_maps():
    labels = dev(np.array([0, 1, 2, 5, 1], np.int32))
    with pytest.raises(sagnn.SagnnError) as ei:
        sagnn.spmm_perm_from_labels(labels, 3)
    assert ei.value.code == -3
    rowptr, colidx, val = random_csr(6, 6, 0.5, np.random.default_rng(0))
    for bad in ([0, 1, 2, 3, 4, 4], [0, 1, 2, 3, 4, 6], [0, 1, 2, 3, 4, -1]):
        with pytest.raises(sagnn.SagnnError) as ei:
            sagnn.spmm_csr_permute_symmetric(dev(rowptr), dev(colidx), dev(val), dev(np.array(bad, np.int32)))
        assert ei.value.code == -3
    ok = dev(np.array([5, 4, 3, 2, 1, 0], np.int32))
    badcol = colidx.copy()
    badcol[0] = 6
    with pytest.raises(sagnn.SagnnError) as ei:
        sagnn.spmm_csr_permute_symmetric(dev(rowptr), dev(badcol), dev(val), ok)
    assert ei.value.code == -3
    sagnn.spmm_csr_permute_symmetric(dev(rowptr), dev(colidx), dev(val), ok)
