"""GPU parity: every step of the hot path, called through the C ABI, element by element against
the CPU oracle on the same seeded inputs.  Integer results bit-exact; fp32 SpMM within
1e-5 * sum|terms|; bf16 GEMM within 1e-2 * sum|terms|."""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2504_04673_amd as sagnn
from paper_2504_04673_amd import synth
from tests.util import assert_close, csr_dev, dev

pytestmark = pytest.mark.gpu

RTOL_SPMM = 1e-5
RTOL_GEMM_FP32 = 1e-5
RTOL_BF16 = 1e-2


def random_csr(m, n, avg, rng, empty_frac=0.0, hubs=(), dup=False):
    deg = rng.poisson(avg, size=m)
    if empty_frac:
        deg[rng.random(m) < empty_frac] = 0
    for r, d in hubs:
        deg[r] = d
    rowptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)
    nnz = int(rowptr[-1])
    colidx = rng.integers(0, n, size=nnz).astype(np.int32)
    if not dup:
        # sort inside rows (duplicates may remain; both sides sum them)
        for r in range(m):
            colidx[rowptr[r]:rowptr[r + 1]].sort()
    val = rng.standard_normal(nnz).astype(np.float32)
    return rowptr, colidx, val


# ------------------------------------------------------------------------------------ pack

@pytest.mark.parametrize("n,f,N,ld", [(4096, 16, 3700, 16), (1000, 4, 1, 4), (1000, 20, 333, 24),
                                      (5000, 128, 4097, 128), (3000, 256, 1025, 260), (2000, 300, 777, 300),
                                      (10, 64, 0, 64)])
def test_pack_rows(n, f, N, ld):
    rng = np.random.default_rng(n + f)
    Hfull = synth.normal((n, ld), 1, synth.STREAM_H)
    rows = np.sort(rng.choice(n, size=N, replace=False)).astype(np.int32)
    Hd = dev(Hfull)[:, :f]          # strided view: leading dimension ld
    got = torch.empty((N, f), device="cuda")
    L = sagnn.lib()
    import ctypes
    rc = L.spmm_pack_rows(ctypes.c_void_p(Hd.data_ptr()), n, ld, f, ctypes.c_void_p(dev(rows).data_ptr()) if N else None,
                          N, ctypes.c_void_p(got.data_ptr()) if N else None, f,
                          ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == 0
    torch.cuda.synchronize()
    ref = oracle.pack_rows(np.ascontiguousarray(Hfull[:, :f]), rows)
    assert got.cpu().numpy().tobytes() == ref.tobytes()


def test_pack_rows_out_of_range_ids_give_zero_rows():
    H = dev(synth.normal((100, 32), 2, synth.STREAM_H))
    rows = dev(np.array([5, -1, 100, 99, 2 ** 31 - 1], np.int32))
    out = sagnn.spmm_pack_rows(H, rows).cpu().numpy()
    Hh = H.cpu().numpy()
    assert np.array_equal(out[0], Hh[5]) and np.array_equal(out[3], Hh[99])
    assert not out[1].any() and not out[2].any() and not out[4].any()


def test_pack_rows_offsets_beyond_4gib():
    """H larger than 2^32 bytes: element offsets must be 64-bit."""
    n, f = 9_000_000, 128                       # 4.6 GB
    H = torch.empty((n, f), device="cuda")
    rows_h = np.array([0, 1, 4_194_304, 8_388_607, 8_388_608, 8_999_999], np.int32)
    vals = synth.normal_rows(rows_h, f, 3, synth.STREAM_H)
    H[torch.from_numpy(rows_h.astype(np.int64)).cuda()] = dev(vals)
    out = sagnn.spmm_pack_rows(H, dev(rows_h)).cpu().numpy()
    assert out.tobytes() == vals.tobytes()
    del H


# ------------------------------------------------------------------------------------ plan

def small_block(m, n, nnz, nb):
    """the shapes the library plans with one workgroup in one launch"""
    return n <= 262144 and m <= 262144 and nnz <= 65536 and nb <= 16


def check_plan(rowptr, colidx, n, colblk):
    """Against the oracle; small blocks through both the one-launch and the general path."""
    needed, blk_off, compact = oracle.needed_rows(rowptr, colidx, n, colblk)
    modes = (False, True) if small_block(rowptr.size - 1, n, colidx.size, len(colblk) - 1) else (False,)
    for multipass in modes:
        plan = sagnn.spmm_plan_needed_rows(dev(rowptr), dev(colidx), n, colblk, multipass=multipass)
        torch.cuda.synchronize()
        assert np.array_equal(plan.blk_off, blk_off), multipass
        assert np.array_equal(plan.needed.cpu().numpy(), needed), multipass
        if colidx.size:
            assert np.array_equal(plan.colidx_compact.cpu().numpy(), compact), multipass
    return plan


@pytest.mark.parametrize("m,n,nnz,nb,seed", [(4096, 262_144, 65_536, 16, 0), (262_144, 262_144, 65_536, 1, 1),
                                             (4096, 262_145, 65_536, 16, 2), (4096, 262_144, 65_537, 16, 3),
                                             (4096, 262_144, 65_536, 17, 4), (300, 129, 5000, 7, 5),
                                             (10, 64, 64, 2, 6), (7, 1, 40, 1, 7), (2000, 200_000, 3, 16, 8)])
def test_plan_small_blocks_one_launch_and_its_limits(m, n, nnz, nb, seed):
    """Shapes at and just beyond the limits of the one-launch path (columns, entries, blocks), tiny
    and nearly empty ones; unsorted columns with duplicates, columns on both sides of every 64-column
    word edge in use and of the last column, block boundaries that coincide and that cut inside a word.
    Capacity: exactly N succeeds; N - 1 is refused with the required size reported and nothing written."""
    rng = np.random.default_rng(seed)
    cols = rng.integers(0, n, size=nnz)
    edge = [0, n - 1, 63, 64, 65, 127, 128, n // 2, (n - 1) // 64 * 64, max((n - 1) // 64 * 64 - 1, 0)]
    k = min(len(edge), nnz)
    cols[:k] = [min(max(c, 0), n - 1) for c in edge[:k]]
    if nnz > 200:
        cols[100:200] = cols[0]                                   # a run of duplicates
    cuts = np.sort(rng.integers(0, nnz + 1, size=m - 1))
    rowptr = np.array([0, *cuts, nnz], dtype=np.int32)
    colidx = cols.astype(np.int32)
    bc = np.sort(rng.integers(0, n + 1, size=nb - 1))
    if nb > 3:
        bc[1] = bc[0]                                             # an empty block
    colblk = np.array([0, *bc, n], dtype=np.int64)
    plan = check_plan(rowptr, colidx, n, colblk)
    N = plan.N
    for multipass in ((False, True) if small_block(m, n, nnz, nb) else (False,)):
        exact = sagnn.spmm_plan_needed_rows(dev(rowptr), dev(colidx), n, colblk, needed_cap=N, multipass=multipass)
        assert exact.N == N and torch.equal(exact.needed, plan.needed)
        if N > 0:
            ws, needed, compact = sagnn.plan_buffers(m, n, nnz, nb, torch.device("cuda"), N - 1, True)
            needed.fill_(-7)
            compact.fill_(-7)
            with pytest.raises(sagnn.SagnnError) as ei:
                sagnn.spmm_plan_needed_rows(dev(rowptr), dev(colidx), n, colblk, needed_cap=N - 1,
                                            bufs=(ws, needed, compact), multipass=multipass)
            assert ei.value.code == -2
            torch.cuda.synchronize()
            assert bool((needed == -7).all()) and bool((compact == -7).all())
        # validation: a negative column, a column equal to n, a row pointer that steps back
        for bad_at, bad_val in ((0, -1), (nnz - 1, n)):
            badc = colidx.copy()
            badc[bad_at] = bad_val
            with pytest.raises(sagnn.SagnnError) as ei:
                sagnn.spmm_plan_needed_rows(dev(rowptr), dev(badc), n, colblk, validate=True, multipass=multipass)
            assert ei.value.code == -3
            lax = sagnn.spmm_plan_needed_rows(dev(rowptr), dev(badc), n, colblk, multipass=multipass)
            assert int(lax.colidx_compact[bad_at]) == -1            # not validated: skipped and flagged
        if m >= 3 and rowptr[1] < nnz:
            badrp = rowptr.copy()
            badrp[1] = badrp[2] + 1
            with pytest.raises(sagnn.SagnnError) as ei:
                sagnn.spmm_plan_needed_rows(dev(badrp), dev(colidx), n, colblk, validate=True, multipass=multipass)
            assert ei.value.code == -3
        sagnn.spmm_plan_needed_rows(dev(rowptr), dev(colidx), n, colblk, validate=True, multipass=multipass)


def test_plan_cfg1_all_blocks(cfg1):
    g, _ = cfg1
    off = synth.block_offsets(g.n, 4)
    for i in range(4):
        blk = g.row_block(int(off[i]), int(off[i + 1]))
        check_plan(blk.rowptr, blk.colidx, g.n, off)
    check_plan(g.rowptr, g.colidx, g.n, np.array([0, g.n]))


@pytest.mark.parametrize("m,n,nb,avg,seed", [(1, 1, 1, 1, 0), (50, 63, 3, 2, 1), (64, 64, 1, 3, 2),
                                             (1000, 65, 5, 1, 3), (3000, 100_003, 16, 9, 4),
                                             (20000, 5_000_001, 7, 4, 5), (10, 1_000_000, 64, 0.3, 6),
                                             (30000, 20_000_003, 9, 6, 7), (5, 33_554_432, 3, 2, 8)])
def test_plan_random_ragged(m, n, nb, avg, seed):
    rng = np.random.default_rng(seed)
    rowptr, colidx, _ = random_csr(m, n, avg, rng, dup=True)
    cuts = np.sort(rng.integers(0, n + 1, size=nb - 1))       # ragged, possibly empty blocks
    colblk = np.array([0, *cuts, n], dtype=np.int64)
    check_plan(rowptr, colidx, n, colblk)


@pytest.mark.parametrize("n,nnz,misalign", [(1_000_000, 4_300_000, 0), (1_245_185, 4_200_003, 1),
                                            (2_700_001, 4_500_001, 3), (4_980_736, 4_194_304, 0),
                                            (500_000, 4_300_000, 0), (100_000, 4_300_003, 0),
                                            (100_001, 4_300_001, 1),
                                            # wider than four LDS ranges: entries partitioned by range first
                                            (4_980_737, 4_200_000, 0), (6_225_921, 4_300_003, 1),
                                            (20_000_003, 4_500_001, 3), (111_059_956, 5_000_000, 0),
                                            (318_767_104, 4_194_304, 0)])
def test_plan_large_entry_counts_lds_marking(n, nnz, misalign):
    """Entry counts above 2^22 with at most ~5 M columns take the LDS-bitmap marking path
    (1 to 4 column ranges); beyond that, up to 2048 ranges of 155,648 columns (318.8 M columns), the
    entries are partitioned by range first and every range is marked from its bucket; the column array is also given at a 4-byte-but-not-16-byte aligned
    address.  Power-law-like columns (squared uniform) plus the last column of every range.
    With eight or more entries per column the marking pass also writes the identity remap in
    advance: the 500 k-column case leaves columns unused (the advance copy must be replaced by
    the real remap), the 100 k-column cases use every column (it is the result)."""
    rng = np.random.default_rng(n % 97)
    m = 5000
    cols = (rng.random(nnz) ** 2 * n).astype(np.int64)
    cols[:8] = [0, n - 1, min(n - 1, 1_245_183), min(n - 1, 1_245_184), min(n - 1, 2_490_367),
                min(n - 1, 2_490_368), min(n - 1, 3_735_552), n // 2]
    if n > 4_980_736:
        # first and last column of the ranges around the middle and at the end; a uniform share so that
        # the far ranges are not empty
        r = 1_245_184
        mid, last = (n // 2) // r, (n - 1) // r
        edge = [mid * r - 1, mid * r, mid * r + r - 1, last * r - 1, last * r, n - 2, 155_647, 155_648,
                (n - 1) // 155_648 * 155_648 - 1, (n - 1) // 155_648 * 155_648]
        cols[8:8 + len(edge)] = [min(max(c, 0), n - 1) for c in edge]
        cols[100:100 + nnz // 4] = rng.integers(0, n, size=nnz // 4)
    cuts = np.sort(rng.integers(0, nnz + 1, size=m - 1))
    rowptr = np.array([0, *cuts, nnz], dtype=np.int32)
    colidx = cols.astype(np.int32)
    colblk = np.array([0, n // 3, n // 3, n - 5, n], dtype=np.int64)
    buf = torch.empty(nnz + 4, dtype=torch.int32, device="cuda")
    ci = buf[misalign:misalign + nnz]
    ci.copy_(torch.from_numpy(colidx))
    plan = sagnn.spmm_plan_needed_rows(dev(rowptr), ci, n, colblk, validate=True)
    torch.cuda.synchronize()
    needed, blk_off, compact = oracle.needed_rows(rowptr, colidx, n, colblk)
    assert np.array_equal(plan.blk_off, blk_off)
    assert np.array_equal(plan.needed.cpu().numpy(), needed)
    assert np.array_equal(plan.colidx_compact.cpu().numpy(), compact)
    if n == 500_000:
        assert plan.N < n
    if n in (100_000, 100_001):
        assert plan.N == n
    ci[12345] = n                                           # out of range: validation must see it
    with pytest.raises(sagnn.SagnnError) as ei:
        sagnn.spmm_plan_needed_rows(dev(rowptr), ci, n, colblk, validate=True)
    assert ei.value.code == -3
    ci[12345] = -2                                          # negative: likewise
    with pytest.raises(sagnn.SagnnError) as ei:
        sagnn.spmm_plan_needed_rows(dev(rowptr), ci, n, colblk, validate=True)
    assert ei.value.code == -3


def test_plan_empty_matrix_and_capacity_and_validate():
    rp = np.zeros(6, np.int32)
    plan = sagnn.spmm_plan_needed_rows(dev(rp), torch.empty(0, dtype=torch.int32, device="cuda"), 100,
                                       np.array([0, 50, 100]))
    assert plan.N == 0 and list(plan.blk_off) == [0, 0, 0]
    rng = np.random.default_rng(0)
    rowptr, colidx, _ = random_csr(100, 1000, 5, rng)
    with pytest.raises(sagnn.SagnnError) as ei:
        sagnn.spmm_plan_needed_rows(dev(rowptr), dev(colidx), 1000, np.array([0, 1000]), needed_cap=3)
    assert ei.value.code == -2
    bad = colidx.copy()
    bad[7] = 1000
    with pytest.raises(sagnn.SagnnError) as ei:
        sagnn.spmm_plan_needed_rows(dev(rowptr), dev(bad), 1000, np.array([0, 1000]), validate=True)
    assert ei.value.code == -3
    badrp = rowptr.copy()
    badrp[10] = badrp[11] + 1
    with pytest.raises(sagnn.SagnnError) as ei:
        sagnn.spmm_plan_needed_rows(dev(badrp), dev(colidx), 1000, np.array([0, 1000]), validate=True)
    assert ei.value.code == -3
    # without validation the bad column is skipped and flagged -1 in the remap
    plan = sagnn.spmm_plan_needed_rows(dev(rowptr), dev(bad), 1000, np.array([0, 1000]))
    assert int(plan.colidx_compact[7]) == -1
    sagnn.spmm_plan_needed_rows(dev(rowptr), dev(colidx), 1000, np.array([0, 1000]), validate=True)
    # every column needed (the remap is then the identity) and one column out of range
    n = 777
    rp2 = np.arange(0, n + 2, dtype=np.int32)
    ci2 = np.concatenate([rng.permutation(n), [n + 3]]).astype(np.int32)
    plan = sagnn.spmm_plan_needed_rows(dev(rp2), dev(ci2), n, np.array([0, 100, n]))
    assert plan.N == n and np.array_equal(plan.needed.cpu().numpy(), np.arange(n))
    assert np.array_equal(plan.colidx_compact.cpu().numpy(), np.concatenate([ci2[:-1], [-1]]))


# ------------------------------------------------------------------------------------ SpMM

def run_spmm(rowptr, colidx, val, B, use_ws, C0=None, expect_mode=None):
    rp, ci, v = dev(rowptr), dev(colidx), dev(val)
    ws = sagnn.spmm_csr_prepare(rp, ci, v, B.shape[0], B.shape[1]) if use_ws else None
    if expect_mode is not None:
        assert ws.info()["mode"] == expect_mode, ws.info()
    C = None if C0 is None else dev(C0)
    out = sagnn.spmm_csr_tallskinny(rp, ci, v, dev(B), C=C, accumulate=C0 is not None, ws=ws)
    torch.cuda.synchronize()
    return out


@pytest.mark.parametrize("f", [4, 16, 20, 32, 48, 64, 100, 128, 192, 256, 320])
@pytest.mark.parametrize("use_ws", [True, False])
def test_spmm_random_widths(f, use_ws):
    rng = np.random.default_rng(f)
    m, n = 3001, 2500
    rowptr, colidx, val = random_csr(m, n, 12, rng, empty_frac=0.15, hubs=[(7, 3000), (1500, 777), (3000, 300)],
                                     dup=True)
    B = synth.normal((n, f), f, synth.STREAM_H)
    ref, zabs = oracle.spmm(rowptr, colidx, val, B, want_abs=True)
    got = run_spmm(rowptr, colidx, val, B, use_ws)
    assert_close(got, ref, zabs, RTOL_SPMM, f"spmm f={f} ws={use_ws}")
    C0 = synth.normal((m, f), f + 1, synth.STREAM_G)
    ref2, zabs2 = oracle.spmm(rowptr, colidx, val, B, C=C0, want_abs=True)
    got2 = run_spmm(rowptr, colidx, val, B, use_ws, C0=C0)
    assert_close(got2, ref2, zabs2, RTOL_SPMM, f"spmm accumulate f={f} ws={use_ws}")


@pytest.fixture(params=["short_rows_by_nonzero_splitting", "short_rows_swept_whole"])
def force_sweep(request, monkeypatch):
    """Force the slab-sweep schedule on small matrices (the heuristic reserves it for big ones)
    with tiny pieces and many slabs, so that split rows, staggered starts and the short-row
    path are all exercised -- the short rows once through the nonzero-splitting kernel on their
    compacted CSR, once as whole-row wavefronts of the sweep (where the width has that form)."""
    monkeypatch.setenv("SAGNN_SWEEP_SHORT_ROWS", "-1" if request.param == "short_rows_by_nonzero_splitting" else "1")
    monkeypatch.setenv("SAGNN_SWEEP", "1")
    monkeypatch.setenv("SAGNN_SWEEP_MINDEG", "16")
    monkeypatch.setenv("SAGNN_SWEEP_PIECE", "1024")
    monkeypatch.setenv("SAGNN_SWEEP_SLAB_MB", "0")
    monkeypatch.setenv("SAGNN_SWEEP_GROUPS", "2")      # lane-group kernels at f = 128 / 64 even with little reuse


@pytest.mark.parametrize("f", [16, 32, 64, 128, 192, 256, 320])
def test_spmm_slab_sweep_schedule(f, force_sweep):
    rng = np.random.default_rng(100 + f)
    m, n = 5003, 40_000
    rowptr, colidx, val = random_csr(m, n, 20, rng, empty_frac=0.1,
                                     hubs=[(3, 9000), (7, 3000), (2500, 1024), (2501, 1025), (5002, 17), (11, 16)])
    B = synth.normal((n, f), f, synth.STREAM_H)
    ref, zabs = oracle.spmm(rowptr, colidx, val, B, want_abs=True)
    got = run_spmm(rowptr, colidx, val, B, True, expect_mode=1)
    assert_close(got, ref, zabs, RTOL_SPMM, f"sweep f={f}")
    got_again = run_spmm(rowptr, colidx, val, B, True)
    assert torch.equal(got, got_again)                       # reproducible across preparations
    C0 = synth.normal((m, f), f + 1, synth.STREAM_G)
    ref2, zabs2 = oracle.spmm(rowptr, colidx, val, B, C=C0, want_abs=True)
    got2 = run_spmm(rowptr, colidx, val, B, True, C0=C0)
    assert_close(got2, ref2, zabs2, RTOL_SPMM, f"sweep accumulate f={f}")


@pytest.mark.parametrize("f", [64, 128, 192, 256])
@pytest.mark.parametrize("groups", [1, 2])
def test_spmm_sweep_short_rows_as_whole_rows(f, groups, monkeypatch):
    """Option short_rows: the rows below the long-row threshold are swept as whole rows, 16 per
    wavefront, instead of going through the nonzero-splitting kernel (no compacted short-row CSR is
    left).  Most rows of this matrix are short, their columns are not sorted and may repeat; long
    rows are ascending as the sweep requires; hubs are cut into pieces; some rows are empty."""
    monkeypatch.setenv("SAGNN_SWEEP", "1")
    monkeypatch.setenv("SAGNN_SWEEP_PIECE", "1024")
    monkeypatch.setenv("SAGNN_SWEEP_SLAB_MB", "0")
    monkeypatch.setenv("SAGNN_SWEEP_MINDEG", "64")
    monkeypatch.setenv("SAGNN_SWEEP_GROUPS", str(groups))
    rng = np.random.default_rng(300 + f + groups)
    m, n = 7001, 30_000
    rowptr, colidx, val = random_csr(m, n, 22, rng, empty_frac=0.1, dup=True,
                                     hubs=[(3, 9000), (7, 3000), (2500, 1025), (5002, 64), (11, 63), (12, 1),
                                           (7000, 200)])
    for r in range(m):
        a, b = rowptr[r], rowptr[r + 1]
        if b - a >= 64:
            o = np.argsort(colidx[a:b], kind="stable")
            colidx[a:b], val[a:b] = colidx[a:b][o], val[a:b][o]
    B = synth.normal((n, f), f, synth.STREAM_H)
    ref, zabs = oracle.spmm(rowptr, colidx, val, B, want_abs=True)
    rp, ci, v = dev(rowptr), dev(colidx), dev(val)
    ws = sagnn.spmm_csr_prepare(rp, ci, v, n, f)
    info = ws.info()
    assert info["mode"] == 1 and info["chunk_rows"] == 0 and info["chunk_entries"] == 0, info
    assert info["split_rows"] >= 3 and info["has_empty_rows"] == 1
    C0 = torch.full((m, f), float("nan"), device="cuda")
    got = sagnn.spmm_csr_tallskinny(rp, ci, v, dev(B), C=C0, ws=ws)
    torch.cuda.synchronize()
    assert_close(got, ref, zabs, RTOL_SPMM, f"whole-row sweep f={f} groups={groups}")
    Cacc = synth.normal((m, f), f + 1, synth.STREAM_G)
    ref2, zabs2 = oracle.spmm(rowptr, colidx, val, B, C=Cacc, want_abs=True)
    got2 = sagnn.spmm_csr_tallskinny(rp, ci, v, dev(B), C=dev(Cacc), accumulate=True, ws=ws)
    torch.cuda.synchronize()
    assert_close(got2, ref2, zabs2, RTOL_SPMM, f"whole-row sweep accumulate f={f} groups={groups}")
    if f in (64, 128, 256):
        # every row ends in a wavefront of the sweep: the layer takes the sweep-epilogue form
        fout = 96
        W = synth.normal((f, fout), 5, synth.STREAM_W, scale=1 / np.sqrt(f))
        for prec in (0, 1, 2):
            assert sagnn.gcn_layer_fwd_form(ws, f, fout, prec) == 2
            o = oracle.gcn_layer_fwd(rowptr, colidx, val, B, W, act=1, bf16=(prec == 1))
            Z0 = torch.full((m, fout), float("nan"), device="cuda")
            H0 = torch.full((m, fout), float("nan"), device="cuda")
            _, Z, Ho = sagnn.gcn_layer_fwd(rp, ci, v, dev(B), dev(W), act=sagnn.ACT_RELU, prec=prec, ws=ws,
                                           want_t=False, out=(None, Z0, H0))
            torch.cuda.synchronize()
            rtol = RTOL_BF16 if prec == 1 else RTOL_GEMM_FP32
            assert_close(Z, o["Z"], o["Zabs"], rtol, f"whole-row sweep layer Z f={f} prec={prec}")
            assert_close(Ho, o["H"], o["Zabs"], rtol, f"whole-row sweep layer H' f={f} prec={prec}")


@pytest.mark.parametrize("variant", ["sixteen_pieces_per_wavefront", "many_small_windows", "snake_dealing",
                                     "one_window_long_threshold_64", "one_row_per_instruction"])
def test_spmm_slab_sweep_planner_variants(variant, force_sweep, monkeypatch):
    """The planner's alternatives (pieces per wavefront, dealing windows, dealing order,
    thresholds) all have to give the same product; small inputs take them through the
    environment overrides the experiments use."""
    if variant == "sixteen_pieces_per_wavefront":
        monkeypatch.setenv("SAGNN_SWEEP_MIN_WAVES", "1")
    elif variant == "many_small_windows":
        monkeypatch.setenv("SAGNN_SWEEP_MIN_WAVES", "64")
        monkeypatch.setenv("SAGNN_SWEEP_WINDOW_PCT", "1")
    elif variant == "snake_dealing":
        monkeypatch.setenv("SAGNN_SWEEP_MIN_WAVES", "1")
        monkeypatch.setenv("SAGNN_SWEEP_LPT", "0")
        monkeypatch.setenv("SAGNN_SWEEP_GROUPS", "1")   # snake dealing exists for one stream per wavefront
    elif variant == "one_row_per_instruction":
        monkeypatch.setenv("SAGNN_SWEEP_GROUPS", "1")
    else:
        monkeypatch.setenv("SAGNN_SWEEP_MINDEG", "64")
        monkeypatch.setenv("SAGNN_SWEEP_WINDOW_PCT", "0")
        monkeypatch.setenv("SAGNN_SWEEP_SLAB_MB", "1")
    f = 128
    rng = np.random.default_rng(77)
    m, n = 9001, 50_000
    rowptr, colidx, val = random_csr(m, n, 30, rng, empty_frac=0.05,
                                     hubs=[(0, 20000), (1, 4097), (4500, 2048), (9000, 700), (17, 64), (18, 63)])
    B = synth.normal((n, f), 3, synth.STREAM_H)
    ref, zabs = oracle.spmm(rowptr, colidx, val, B, want_abs=True)
    got = run_spmm(rowptr, colidx, val, B, True, expect_mode=1)
    assert_close(got, ref, zabs, RTOL_SPMM, f"sweep planner variant {variant}")
    C0 = synth.normal((m, f), 4, synth.STREAM_G)
    ref2, zabs2 = oracle.spmm(rowptr, colidx, val, B, C=C0, want_abs=True)
    assert_close(run_spmm(rowptr, colidx, val, B, True, C0=C0), ref2, zabs2, RTOL_SPMM, f"{variant} accumulate")


@pytest.mark.parametrize("f", [128, 64, 256])
def test_spmm_sweep_planner_balances_streams(f, monkeypatch):
    """The device planner deals pieces longest-first to the shortest stream in batches; its longest
    stream must be as short as the one of the sequential piece-by-piece rule, computed here with a
    heap on the sizes the planner cuts (rows of >= 64 entries in pieces of <= 4096, strided).
    Heavy-tailed degrees make the rule matter: dealing in whole rounds would leave the streams
    that got the largest pieces first ~30 % longer than the average."""
    import heapq
    monkeypatch.setenv("SAGNN_SWEEP", "1")
    monkeypatch.setenv("SAGNN_SWEEP_MINDEG", "64")
    monkeypatch.setenv("SAGNN_SWEEP_MIN_WAVES", "1")          # all 16 slots of a wavefront
    monkeypatch.setenv("SAGNN_SWEEP_SHORT_ROWS", "-1")        # the streams of the long rows only
    rng = np.random.default_rng(9)
    m, n = 30_000, 200_000
    deg = np.minimum((64 / rng.random(m) ** 0.8).astype(np.int64), 30_000)   # heavy tail from 64 up
    deg[rng.random(m) < 0.3] = 5                                              # some short rows
    rowptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)
    nnz = int(rowptr[-1])
    colidx = np.empty(nnz, np.int32)
    for r in range(m):
        colidx[rowptr[r]:rowptr[r + 1]] = np.sort(rng.integers(0, n, size=deg[r]))
    val = np.ones(nnz, np.float32)
    ws = sagnn.spmm_csr_prepare(dev(rowptr), dev(colidx), dev(val), n, f)
    info = ws.info()
    assert info["mode"] == 1 and info["sweep_entries"] + info["chunk_entries"] == nnz
    R = info["groups"]
    sizes = []
    for d in deg[deg >= 64]:
        p = -(-int(d) // 4096)
        sizes += [(int(d) - j + p - 1) // p for j in range(p)]
    sizes.sort(reverse=True)
    assert info["sweep_entries"] == sum(sizes)
    n_waves = -(-len(sizes) // 16)        # as few wavefronts as the 16 slots allow (the launch rounds up to 4)
    assert n_waves <= info["sweep_waves"] < n_waves + 4
    units, per_unit = n_waves * R, 16 // R
    heap = [(0, u) for u in range(units)]
    used = [0] * units
    longest = 0
    for sz in sizes:
        load, u = heapq.heappop(heap)
        load += sz
        used[u] += 1
        longest = max(longest, load)
        if used[u] < per_unit:
            heapq.heappush(heap, (load, u))
    # the library counts steps of wavefronts (the longer of a wavefront's group streams, in whole
    # batches of 8): allow that rounding and 3 % on top
    assert info["longest_stream_steps"] <= 1.03 * longest + 8, (info, longest, sum(sizes) / units)
    # and the product is right
    B = synth.normal((n, f), 5, synth.STREAM_H)
    rows = rng.choice(m, size=200, replace=False)
    got = sagnn.spmm_csr_tallskinny(dev(rowptr), dev(colidx), dev(val), dev(B), ws=ws)
    torch.cuda.synchronize()
    rows.sort()
    sub_deg = deg[rows]
    sub_rowptr = np.concatenate([[0], np.cumsum(sub_deg)]).astype(np.int32)
    sub_idx = np.concatenate([np.arange(rowptr[r], rowptr[r + 1]) for r in rows])
    ref, zabs = oracle.spmm(sub_rowptr, colidx[sub_idx], val[sub_idx], B, want_abs=True)
    assert_close(got[torch.from_numpy(rows).cuda()], ref, zabs, RTOL_SPMM, f"balanced planner f={f}")


@pytest.mark.parametrize("f", [192, 256, 320])
def test_spmm_sweep_wide_operand_as_128_wide_slabs(f, force_sweep, monkeypatch):
    """Operands wider than 128 taken as 128-wide column slabs (plus a 64-wide rest) by the kernels
    that fetch two rows of B per load: same product."""
    monkeypatch.setenv("SAGNN_SWEEP_SLAB_WIDTH", "128")
    rng = np.random.default_rng(f + 1)
    m, n = 6001, 40_000
    rowptr, colidx, val = random_csr(m, n, 25, rng, empty_frac=0.1,
                                     hubs=[(4, 7000), (9, 2049), (3000, 1024), (6000, 33)])
    B = synth.normal((n, f), f, synth.STREAM_H)
    ref, zabs = oracle.spmm(rowptr, colidx, val, B, want_abs=True)
    rp, ci, v = dev(rowptr), dev(colidx), dev(val)
    ws = sagnn.spmm_csr_prepare(rp, ci, v, n, f)
    info = ws.info()
    assert info["mode"] == 1 and info["groups"] == 2
    got = sagnn.spmm_csr_tallskinny(rp, ci, v, dev(B), ws=ws)
    torch.cuda.synchronize()
    assert_close(got, ref, zabs, RTOL_SPMM, f"128-wide slabs f={f}")
    C0 = synth.normal((m, f), f + 2, synth.STREAM_G)
    ref2, zabs2 = oracle.spmm(rowptr, colidx, val, B, C=C0, want_abs=True)
    got2 = sagnn.spmm_csr_tallskinny(rp, ci, v, dev(B), C=dev(C0), accumulate=True, ws=ws)
    torch.cuda.synchronize()
    assert_close(got2, ref2, zabs2, RTOL_SPMM, f"128-wide slabs accumulate f={f}")
    # a narrower call on the same workspace (the streams serve 128- and 64-wide launches)
    B64 = synth.normal((n, 64), 3, synth.STREAM_H)
    ref3, zabs3 = oracle.spmm(rowptr, colidx, val, B64, want_abs=True)
    got3 = sagnn.spmm_csr_tallskinny(rp, ci, v, dev(B64), ws=ws)
    torch.cuda.synchronize()
    assert_close(got3, ref3, zabs3, RTOL_SPMM, f"128-wide slabs prepared {f}, called 64")


def test_spmm_sweep_workspace_prepared_for_wider_f(force_sweep):
    """A workspace prepared for f = 128 (two lane groups) or 256 also serves narrower calls."""
    rng = np.random.default_rng(31)
    m, n = 3000, 30_000
    rowptr, colidx, val = random_csr(m, n, 25, rng, hubs=[(2, 6000), (1500, 1500)])
    rp, ci, v = dev(rowptr), dev(colidx), dev(val)
    for f_prep, f_call in ((128, 64), (256, 128), (256, 64), (192, 128)):
        ws = sagnn.spmm_csr_prepare(rp, ci, v, n, f_prep)
        assert ws.info()["mode"] == 1
        B = synth.normal((n, f_call), f_prep + f_call, synth.STREAM_H)
        ref, zabs = oracle.spmm(rowptr, colidx, val, B, want_abs=True)
        got = sagnn.spmm_csr_tallskinny(rp, ci, v, dev(B), ws=ws)
        torch.cuda.synchronize()
        assert_close(got, ref, zabs, RTOL_SPMM, f"prepared {f_prep}, called {f_call}")


def test_spmm_slab_sweep_falls_back_on_unsorted_rows(force_sweep):
    rng = np.random.default_rng(5)
    m, n, f = 2000, 30_000, 128
    rowptr, colidx, val = random_csr(m, n, 40, rng, hubs=[(5, 5000)], dup=True)   # unsorted rows
    B = synth.normal((n, f), 1, synth.STREAM_H)
    ref, zabs = oracle.spmm(rowptr, colidx, val, B, want_abs=True)
    assert_close(run_spmm(rowptr, colidx, val, B, True, expect_mode=0), ref, zabs, RTOL_SPMM, "unsorted fallback")
    bad = colidx.copy()
    rowptr2, colidx2, val2 = random_csr(m, n, 40, rng, hubs=[(5, 5000)])
    colidx2[rowptr2[5] + 4999] = n + 7                        # out-of-range column in a long row
    ref, zabs = oracle.spmm(rowptr2, np.minimum(colidx2, n - 1), val2, B, want_abs=True)
    assert_close(run_spmm(rowptr2, colidx2, val2, B, True, expect_mode=0), ref, zabs, RTOL_SPMM, "clamped column")
    _ = bad


def _strided(a, pad, fill):
    """Device matrix whose rows are `pad` floats apart wider than a's: returns (view, whole)."""
    m, f = a.shape
    whole = torch.full((m, f + pad), fill, dtype=torch.float32, device="cuda")
    whole[:, :f] = dev(a)
    return whole[:, :f], whole


@pytest.mark.parametrize("schedule", ["no_workspace", "nonzero_splitting", "sweep", "sweep_one_row_per_load"])
@pytest.mark.parametrize("f", [16, 32, 48, 64, 100, 128, 192, 256, 320])
def test_spmm_leading_dimensions_wider_than_f(f, schedule, monkeypatch):
    """B and C as column slices of wider matrices (ldb = f + 4, ldc = f + 8), overwrite and
    accumulate; the padding columns of C must come back untouched."""
    if schedule.startswith("sweep"):
        if f not in (16, 32, 64, 128, 192, 256, 320) or (schedule == "sweep_one_row_per_load" and f < 64):
            pytest.skip("no such kernel at this width")
        monkeypatch.setenv("SAGNN_SWEEP", "1")
        monkeypatch.setenv("SAGNN_SWEEP_MINDEG", "16")
        monkeypatch.setenv("SAGNN_SWEEP_PIECE", "1024")
        monkeypatch.setenv("SAGNN_SWEEP_SLAB_MB", "0")
        monkeypatch.setenv("SAGNN_SWEEP_GROUPS", "1" if schedule == "sweep_one_row_per_load" else "2")
    else:
        monkeypatch.setenv("SAGNN_SWEEP", "0")
    rng = np.random.default_rng(1000 + f)
    m, n = 4001, 30_000
    rowptr, colidx, val = random_csr(m, n, 18, rng, empty_frac=0.1,
                                     hubs=[(3, 7000), (9, 2049), (2000, 1024), (4000, 100), (17, 16)])
    B = synth.normal((n, f), f, synth.STREAM_H)
    C0 = synth.normal((m, f), f + 1, synth.STREAM_G)
    rp, ci, v = dev(rowptr), dev(colidx), dev(val)
    Bv, _ = _strided(B, 4, 123.0)
    ws = None
    if schedule != "no_workspace":
        ws = sagnn.spmm_csr_prepare(rp, ci, v, n, f)
        assert ws.info()["mode"] == (1 if schedule.startswith("sweep") else 0), ws.info()
    for acc in (False, True):
        ref, zabs = oracle.spmm(rowptr, colidx, val, B, C=C0 if acc else None, want_abs=True)
        Cv, Cw = _strided(C0, 8, -77.0)
        sagnn.spmm_csr_tallskinny(rp, ci, v, Bv, C=Cv, accumulate=acc, ws=ws)
        torch.cuda.synchronize()
        assert_close(Cv, ref, zabs, RTOL_SPMM, f"strided f={f} {schedule} accumulate={acc}")
        assert torch.all(Cw[:, f:] == -77.0)


@pytest.mark.parametrize("case", ["f128_lane_groups", "f128_one_row_per_load", "f256_one_row_per_load", "f64_quarter_groups",
                                  "f32_perm", "f16_perm", "f128_nonzero_splitting", "f128_no_workspace",
                                  "f100_slabs_and_remainder"])
def test_spmm_operand_larger_than_4gib(case, monkeypatch):
    """Rows of B beyond byte offset 2^32 (k * ldb * 4 > 2^32): the kernels cannot use 32-bit
    buffer offsets and switch to 64-bit addressing; every schedule has such a variant.  B is a
    4.6 GB allocation in which only the referenced rows are filled; the oracle multiplies by
    those rows alone (columns renumbered), which is the same product."""
    f = int(case[1:case.index("_")])
    ld = 256 if f > 128 else 128
    k = (9_000_000 * 128) // ld
    sweep = not ("nonzero" in case or "no_workspace" in case or "slabs" in case)
    monkeypatch.setenv("SAGNN_SWEEP", "1" if sweep else "0")
    if sweep:
        monkeypatch.setenv("SAGNN_SWEEP_MINDEG", "16")
        monkeypatch.setenv("SAGNN_SWEEP_PIECE", "1024")
        monkeypatch.setenv("SAGNN_SWEEP_SLAB_MB", "64")
        monkeypatch.setenv("SAGNN_SWEEP_GROUPS", "1" if "one_row" in case else "2")
    rng = np.random.default_rng(len(case) + f)
    m = 3000
    rowptr, colidx, val = random_csr(m, k, 14, rng, empty_frac=0.05, hubs=[(5, 6000), (70, 1500), (2999, 64)])
    # make sure both sides of the 2^32-byte line and the very last row are referenced
    line = (1 << 32) // (ld * 4)
    colidx[rowptr[5]:rowptr[5] + 6] = np.sort(np.array([0, line - 1, line, line + 1, k - 2, k - 1], np.int32))
    colidx[rowptr[5]:rowptr[6]].sort()
    ucols, inv = np.unique(colidx, return_inverse=True)
    assert ucols[-1] == k - 1 and (ucols.astype(np.int64) * ld * 4 >= (1 << 32)).sum() > 1000
    Bsmall = synth.normal((ucols.size, f), f, synth.STREAM_H)
    buf = torch.empty(9_000_000 * 128, dtype=torch.float32, device="cuda")
    Bfull = buf.view(k, ld)
    Bfull[torch.from_numpy(ucols.astype(np.int64)).cuda(), :f] = dev(Bsmall)
    Bv = Bfull[:, :f]
    rp, ci, v = dev(rowptr), dev(colidx), dev(val)
    ws = None if "no_workspace" in case else sagnn.spmm_csr_prepare(rp, ci, v, k, f)
    if ws is not None:
        assert ws.info()["mode"] == (1 if sweep else 0), ws.info()
    C0 = synth.normal((m, f), 5, synth.STREAM_G)
    for acc in (False, True):
        ref, zabs = oracle.spmm(rowptr, inv.astype(np.int32), val, Bsmall, C=C0 if acc else None, want_abs=True)
        Cv, Cw = _strided(C0, 8, -77.0)
        sagnn.spmm_csr_tallskinny(rp, ci, v, Bv, C=Cv, accumulate=acc, ws=ws)
        torch.cuda.synchronize()
        assert_close(Cv, ref, zabs, RTOL_SPMM, f"{case} accumulate={acc}")
        assert torch.all(Cw[:, f:] == -77.0)
    del buf, Bfull, Bv


def test_spmm_workspace_rejects_a_shorter_operand_and_release_forgets_it(monkeypatch):
    """A schedule prepared for k rows of B holds column ids up to k-1: a call with fewer rows is
    refused on the host (nothing launched).  After spmm_csr_release the address is unknown."""
    import ctypes
    monkeypatch.setenv("SAGNN_SWEEP", "1")
    rng = np.random.default_rng(8)
    m, n, f = 2000, 20_000, 128
    rowptr, colidx, val = random_csr(m, n, 30, rng, hubs=[(1, 4000)])
    rp, ci, v = dev(rowptr), dev(colidx), dev(val)
    B = dev(synth.normal((n, f), 1, synth.STREAM_H))
    for sweep in ("1", "0"):
        monkeypatch.setenv("SAGNN_SWEEP", sweep)
        ws = sagnn.spmm_csr_prepare(rp, ci, v, n, f)
        with pytest.raises(ValueError):
            sagnn.spmm_csr_tallskinny(rp, ci, v, B[: n - 1], ws=ws)
        C = torch.zeros((m, f), device="cuda")
        L = sagnn.lib()
        args = lambda kk: (ctypes.c_void_p(rp.data_ptr()), ctypes.c_void_p(ci.data_ptr()), ctypes.c_void_p(v.data_ptr()),
                           m, kk, ci.numel(), ctypes.c_void_p(B.data_ptr()), f, f, ctypes.c_void_p(C.data_ptr()), f, 0,
                           ctypes.c_void_p(ws.buf.data_ptr()), ws.buf.numel(), None)
        assert L.spmm_csr_tallskinny(*args(n - 1)) == -1
        assert L.spmm_csr_tallskinny(*args(n)) == 0
        torch.cuda.synchronize()
        ptr = ctypes.c_void_p(ws.buf.data_ptr())
        keep = ws.buf
        assert L.spmm_csr_release(ptr) == 0
        assert L.spmm_csr_tallskinny(*args(n)) == -1           # unknown workspace now
        assert L.spmm_csr_release(ptr) == 0                    # releasing twice is harmless
        ws.buf = None
        del keep


@pytest.mark.parametrize("sweep", ["0", "1"])
@pytest.mark.parametrize("f", [16, 32, 64, 128, 256])
def test_spmm_long_rows_of_equal_terms_stay_within_tolerance(f, sweep, monkeypatch):
    """Rows whose products are all the same positive number are the worst case for fp32 rounding:
    every addition of a long serial sum rounds the same way, so the error grows with the length of
    the sum instead of its square root.  The kernels keep every serial run short; the result must
    stay within the SpMM tolerance of the exact value (here known in closed form)."""
    monkeypatch.setenv("SAGNN_SWEEP", sweep)
    rng = np.random.default_rng(f)
    n = 65_536
    # enough entries in long rows for the planner to keep the sweep at every width
    degs = np.concatenate([[60_000] * 8, [33_333] * 4, [4096, 4097, 9000], rng.integers(1, 40, size=3000)])
    rowptr = np.zeros(degs.size + 1, dtype=np.int32)
    rowptr[1:] = np.cumsum(degs)
    colidx = np.concatenate([np.sort(rng.choice(n, size=int(d), replace=False)) for d in degs]).astype(np.int32)
    val = np.concatenate([np.full(int(d), np.float32(1.0 / math.sqrt(d))) for d in degs]).astype(np.float32)
    B = np.full((n, f), np.float32(math.sqrt(3.0)), dtype=np.float32)
    exact = degs.astype(np.float64) * val[rowptr[:-1]].astype(np.float64) * float(B[0, 0])
    got = run_spmm(rowptr, colidx, val, B, True, expect_mode=int(sweep)).cpu().numpy().astype(np.float64)
    rel = np.abs(got - exact[:, None]) / exact[:, None]
    assert rel.max() <= RTOL_SPMM, (rel.max(), int(rel.max(axis=1).argmax()))
    if sweep == "0":                                          # the kernel for calls without a workspace
        got = run_spmm(rowptr, colidx, val, B, False).cpu().numpy().astype(np.float64)
        rel = np.abs(got - exact[:, None]) / exact[:, None]
        assert rel.max() <= RTOL_SPMM, (rel.max(), int(rel.max(axis=1).argmax()))


def test_spmm_prepare_tuned_keeps_a_correct_plan(monkeypatch):
    """The tuned preparation tries several plan variants on the caller's operand; whichever it
    keeps has to give the product, in the buffer it wrote during tuning and in later calls.  A
    matrix too small for the sweep has nothing to vary and behaves like the plain preparation."""
    g = synth.rmat_graph(60_000, 4_000_000, 11)
    H = synth.normal((g.n, 128), 11, synth.STREAM_H)
    ref, zabs = oracle.spmm(g.rowptr, g.colidx, g.val, H, want_abs=True)
    rp, ci, v = dev(g.rowptr), dev(g.colidx), dev(g.val)
    monkeypatch.setenv("SAGNN_SWEEP", "1")
    C = torch.full((g.m, 128), float("nan"), device="cuda")
    ws = sagnn.spmm_csr_prepare_tuned(rp, ci, v, dev(H), C=C)
    torch.cuda.synchronize()
    assert ws.info()["mode"] == 1 and 0 <= ws.choice["variant"] < 5 and ws.choice["best_us"] > 0
    assert_close(C, ref, zabs, RTOL_SPMM, "product left by the tuning runs")
    got = sagnn.spmm_csr_tallskinny(rp, ci, v, dev(H), ws=ws)
    torch.cuda.synchronize()
    assert_close(got, ref, zabs, RTOL_SPMM, f"tuned plan {ws.choice}")
    monkeypatch.setenv("SAGNN_SWEEP", "0")
    ws0 = sagnn.spmm_csr_prepare_tuned(rp, ci, v, dev(H))
    assert ws0.info()["mode"] == 0 and ws0.choice["variant"] == 0
    got0 = sagnn.spmm_csr_tallskinny(rp, ci, v, dev(H), ws=ws0)
    torch.cuda.synchronize()
    assert_close(got0, ref, zabs, RTOL_SPMM, "plain schedule through the tuned entry point")


def test_spmm_rmat_with_and_without_sweep(monkeypatch):
    g = synth.rmat_graph(60_000, 4_000_000, 9)
    H = synth.normal((g.n, 128), 9, synth.STREAM_H)
    ref, zabs = oracle.spmm(g.rowptr, g.colidx, g.val, H, want_abs=True)
    for mode in ("0", "1"):
        monkeypatch.setenv("SAGNN_SWEEP", mode)
        got = run_spmm(g.rowptr, g.colidx, g.val, H, True, expect_mode=int(mode))
        assert_close(got, ref, zabs, RTOL_SPMM, f"rmat sweep={mode}")


@pytest.mark.parametrize("case", ["all_empty", "single_entry", "one_long_row", "exact_chunk", "tail_empty"])
def test_spmm_degenerate(case):
    f, n = 128, 700
    rng = np.random.default_rng(1)
    if case == "all_empty":
        rowptr = np.zeros(11, np.int32); colidx = np.empty(0, np.int32); val = np.empty(0, np.float32)
    elif case == "single_entry":
        rowptr = np.array([0, 0, 1, 1], np.int32); colidx = np.array([699], np.int32); val = np.array([2.5], np.float32)
    elif case == "one_long_row":
        rowptr = np.array([0, 2000], np.int32); colidx = rng.integers(0, n, 2000).astype(np.int32)
        val = rng.standard_normal(2000).astype(np.float32)
    elif case == "exact_chunk":     # rows end exactly on chunk boundaries
        rowptr = np.array([0, 256, 512, 512, 1024], np.int32); colidx = rng.integers(0, n, 1024).astype(np.int32)
        val = rng.standard_normal(1024).astype(np.float32)
    else:
        rowptr = np.array([0, 300, 300, 300], np.int32); colidx = rng.integers(0, n, 300).astype(np.int32)
        val = rng.standard_normal(300).astype(np.float32)
    B = synth.normal((n, f), 9, synth.STREAM_H)
    ref, zabs = oracle.spmm(rowptr, colidx, val, B, want_abs=True)
    for use_ws in (True, False):
        got = torch.full((rowptr.size - 1, f), 7.0, device="cuda")     # stale contents must be overwritten
        rp = dev(rowptr)
        ci = dev(colidx) if colidx.size else torch.empty(0, dtype=torch.int32, device="cuda")
        va = dev(val) if val.size else torch.empty(0, device="cuda")
        ws = sagnn.spmm_csr_prepare(rp, ci, va, n, f) if use_ws else None
        sagnn.spmm_csr_tallskinny(rp, ci, va, dev(B), C=got, ws=ws)
        torch.cuda.synchronize()
        assert_close(got, ref, zabs, RTOL_SPMM, f"{case} ws={use_ws}")


def test_spmm_identity_and_ring_closed_forms():
    n, f = 1000, 128
    H = synth.normal((n, f), 4, synth.STREAM_H)
    rp = np.arange(n + 1, dtype=np.int32); ci = np.arange(n, dtype=np.int32); v = np.ones(n, np.float32)
    got = run_spmm(rp, ci, v, H, True)
    assert got.cpu().numpy().tobytes() == H.tobytes()
    g = synth.ring_graph(4096, 8)
    ones = np.ones((4096, 64), np.float32)
    got = run_spmm(g.rowptr, g.colidx, g.val, ones, True).cpu().numpy()
    assert np.all(got == 8.0)


def test_spmm_cfg1_blocks_through_packed_buffer(cfg1):
    """Configuration 1 end to end: plan -> pack -> SpMM with compact indices, per row block,
    equals the oracle's A_i * H; also the whole matrix as one block."""
    g, H = cfg1
    off = synth.block_offsets(g.n, 4)
    Hd = dev(H)
    for i in range(4):
        blk = g.row_block(int(off[i]), int(off[i + 1]))
        rp, ci, v = csr_dev(blk)
        plan = sagnn.spmm_plan_needed_rows(rp, ci, g.n, off)
        Hn = sagnn.spmm_pack_rows(Hd, plan.needed)
        ws = sagnn.spmm_csr_prepare(rp, plan.colidx_compact, v, plan.N, 16)
        Z = sagnn.spmm_csr_tallskinny(rp, plan.colidx_compact, v, Hn, ws=ws)
        torch.cuda.synchronize()
        ref, zabs = oracle.spmm(blk.rowptr, blk.colidx, blk.val, H, want_abs=True)
        assert_close(Z, ref, zabs, RTOL_SPMM, f"cfg1 block {i}")
        # block-by-block accumulation (Alg. 1 inner loop): Z += A_iq * H[NnzCols(i,q)]
        Zacc = torch.zeros_like(Z)
        comp = plan.colidx_compact.cpu().numpy()
        for q in range(4):
            keep = (blk.colidx >= off[q]) & (blk.colidx < off[q + 1])
            cnt = np.add.reduceat(keep.astype(np.int64), blk.rowptr[:-1]) * (np.diff(blk.rowptr) > 0)
            rpq = np.concatenate([[0], np.cumsum(cnt)]).astype(np.int32)
            ciq = (comp[keep] - plan.blk_off[q]).astype(np.int32)
            Hq = Hn[int(plan.blk_off[q]):int(plan.blk_off[q + 1])].contiguous()
            drp, dci, dva = dev(rpq), dev(ciq), dev(blk.val[keep])
            wsq = sagnn.spmm_csr_prepare(drp, dci, dva, Hq.shape[0], 16)
            sagnn.spmm_csr_tallskinny(drp, dci, dva, Hq, C=Zacc, accumulate=True, ws=wsq)
        torch.cuda.synchronize()
        assert_close(Zacc, ref, zabs, RTOL_SPMM, f"cfg1 block {i} accumulated")
    rp, ci, v = csr_dev(g)
    ws = sagnn.spmm_csr_prepare(rp, ci, v, g.n, 16)
    Z = sagnn.spmm_csr_tallskinny(rp, ci, v, Hd, ws=ws)
    ref, zabs = oracle.spmm(g.rowptr, g.colidx, g.val, H, want_abs=True)
    assert_close(Z, ref, zabs, RTOL_SPMM, "cfg1 whole")


@pytest.mark.parametrize("f", [16, 64, 128, 256])
def test_spmm_small_rmat(f):
    g = synth.rmat_graph(40_000, 2_000_000, 5)
    H = synth.normal((g.n, f), 5, synth.STREAM_H)
    ref, zabs = oracle.spmm(g.rowptr, g.colidx, g.val, H, want_abs=True)
    got = run_spmm(g.rowptr, g.colidx, g.val, H, True)
    assert_close(got, ref, zabs, RTOL_SPMM, f"rmat f={f}")
    # sqrt(d) is an eigenvector of the normalised adjacency matrix (closed form at any size)
    x = np.sqrt(np.diff(g.rowptr).astype(np.float64)).astype(np.float32)
    X = np.repeat(x[:, None], f, axis=1).copy()
    got = run_spmm(g.rowptr, g.colidx, g.val, X, True).cpu().numpy()
    assert np.allclose(got, X, rtol=2e-5, atol=0)


# ------------------------------------------------------------------------------------ GEMM / layer

@pytest.mark.parametrize("m,k,n", [(1, 32, 32), (31, 64, 96), (33, 128, 128), (1000, 160, 256), (4097, 256, 64),
                                   (77, 16, 16), (500, 20, 100), (129, 100, 44), (64, 4, 4)])
@pytest.mark.parametrize("prec", [0, 1, 2])
@pytest.mark.parametrize("transW", [False, True])
def test_dense_gemm(m, k, n, prec, transW):
    X = synth.normal((m, k), m, synth.STREAM_H)
    W = synth.normal((n, k) if transW else (k, n), k, synth.STREAM_W, scale=1 / np.sqrt(k))
    if prec == 1:
        X.reshape(-1)[:4] = [1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(1.0 + 2.0 ** -8), 1.0 + 2.0 ** -8 + 2.0 ** -20][:min(4, X.size)]
    mask = synth.normal((m, n), n, synth.STREAM_G)
    ref, zabs = oracle.gemm(X, W, bf16=(prec == 1), transW=transW, want_abs=True)
    rtol = RTOL_BF16 if prec == 1 else RTOL_GEMM_FP32
    Z, A = sagnn.dense_gemm_act(dev(X), dev(W), transW=transW, prec=prec, act=sagnn.ACT_RELU, want_z=True, want_act=True)
    torch.cuda.synchronize()
    assert_close(Z, ref, zabs, rtol, "gemm Z")
    assert torch.equal(A, torch.clamp_min(Z, 0))
    Zm, _ = sagnn.dense_gemm_act(dev(X), dev(W), transW=transW, prec=prec, mask=dev(mask))
    torch.cuda.synchronize()
    assert_close(Zm, np.where(mask > 0, ref, 0), zabs, rtol, "gemm masked")
    assert torch.equal(Zm == 0, (dev(mask) <= 0) | (Z == 0))


@pytest.mark.parametrize("k,n", [(128, 128), (256, 256), (100, 44)])
def test_bf16x3_gemm_has_the_accuracy_of_the_fp32_gemm(k, n):
    """fp32 operands as three bfloat16 terms, six products: every operand bit takes part, so the
    result must be as close to the fp64 oracle as the fp32 matrix-core product is (both accumulate
    in fp32), and far inside the fp32 tolerance.  Operands with all 24 significant bits set, of both
    signs, very small and very large magnitudes, and zeros: a term lost in the split, a wrong pairing
    of the terms or a rounding that does not sum back to the operand shows at 2^-9 .. 2^-17."""
    m = 777
    X = synth.normal((m, k), 5, synth.STREAM_H)
    W = synth.normal((k, n), 5, synth.STREAM_W, scale=1 / np.sqrt(k))
    X[0, :] = np.float32(1.0) + np.float32(2.0 ** -23) * np.arange(1, 2 * k, 2, dtype=np.float32)   # dense low bits
    X[1, :] = -(np.float32(2.0) - np.float32(2.0 ** -23))                                              # all ones
    X[2, :] = X[2, :] * np.float32(1e-30)
    X[3, :] = X[3, :] * np.float32(1e30)
    X[4, :] = 0
    X[5, ::2] = np.float32(1.0 + 2.0 ** -8 + 2.0 ** -16)      # a tie at the first rounding, low bits behind it
    W[:, 0] = np.float32(1.0) - np.float32(2.0 ** -24)
    W[:, 1] = np.float32(-3.0) * (np.float32(1.0) + np.float32(2.0 ** -23))
    ref, zabs = oracle.gemm(X, W, want_abs=True)
    Z32, _ = sagnn.dense_gemm_act(dev(X), dev(W), prec=0)
    Zs, _ = sagnn.dense_gemm_act(dev(X), dev(W), prec=2)
    torch.cuda.synchronize()
    assert_close(Zs, ref, zabs, RTOL_GEMM_FP32, "bf16x3 gemm")
    scale = np.where(zabs > 0, zabs, 1.0)
    e32 = float(np.max(np.abs(Z32.cpu().numpy().astype(np.float64) - ref) / scale))
    es = float(np.max(np.abs(Zs.cpu().numpy().astype(np.float64) - ref) / scale))
    assert es <= max(2 * e32, 2e-7), (es, e32)
    assert es < 2e-6
    assert bool((Zs[4] == 0).all())


def test_bf16_gemm_is_tight_against_bf16_rounded_oracle():
    """With operands rounded the same way the only difference left is fp32 vs fp64 accumulation,
    so the result must sit far inside the 1e-2 budget; a wrong rounding mode would not."""
    X = synth.normal((512, 256), 1, synth.STREAM_H)
    W = synth.normal((256, 256), 1, synth.STREAM_W, scale=1 / 16)
    ref, zabs = oracle.gemm(X, W, bf16=True, want_abs=True)
    Z, _ = sagnn.dense_gemm_act(dev(X), dev(W), prec=1)
    torch.cuda.synchronize()
    assert_close(Z, ref, zabs, 2e-5, "bf16 gemm vs bf16-rounded oracle")


@pytest.mark.parametrize("prec,fin,fout", [(0, 128, 128), (1, 256, 256), (0, 64, 32), (0, 16, 16), (1, 48, 20),
                                           (2, 128, 128), (2, 256, 256), (2, 48, 20)])
def test_gcn_layer_fwd_bwd_small(prec, fin, fout):
    g = synth.sbm_graph(6000, 16, 40, 2, 3)
    H = synth.normal((g.n, fin), 1, synth.STREAM_H)
    W = synth.normal((fin, fout), 1, synth.STREAM_W, scale=1 / np.sqrt(fin))
    G = synth.normal((g.n, fout), 1, synth.STREAM_G)
    rp, ci, v = csr_dev(g)
    ws_in = sagnn.spmm_csr_prepare(rp, ci, v, g.n, fin)
    ws_out = sagnn.spmm_csr_prepare(rp, ci, v, g.n, fout)
    rtol = RTOL_BF16 if prec == 1 else RTOL_GEMM_FP32
    o = oracle.gcn_layer_fwd(g.rowptr, g.colidx, g.val, H, W, act=1, bf16=(prec == 1))
    T, Z, Ho = sagnn.gcn_layer_fwd(rp, ci, v, dev(H), dev(W), act=sagnn.ACT_RELU, prec=prec, ws=ws_in)
    torch.cuda.synchronize()
    assert_close(T, o["T"], o["Tabs"], RTOL_SPMM, "layer T")
    assert_close(Z, o["Z"], o["Zabs"], rtol, "layer Z")
    assert_close(Ho, o["H"], o["Zabs"], rtol, "layer H")
    # the dense stage by itself, on the very T the library produced: scale |T| |W| (no slack
    # inherited from the sparse product's sum of magnitudes)
    Tg = T.cpu().numpy()
    zt, ztabs = oracle.gemm(Tg, W, bf16=(prec == 1), want_abs=True)
    assert_close(Z, zt, ztabs, rtol, "layer Z vs oracle GEMM of the library's T")
    # backward of this layer with the oracle's own Z / inputs as given data
    Zprev = synth.normal((g.n, fin), 2, synth.STREAM_G)
    ob = oracle.gcn_layer_bwd(g.rowptr, g.colidx, g.val, G, W, Zprev, H, bf16=(prec == 1))
    S, Gp, Y = sagnn.gcn_layer_bwd(rp, ci, v, dev(G), dev(W), dev(Zprev), dev(H), prec=prec, ws=ws_out)
    torch.cuda.synchronize()
    assert_close(S, ob["S"], ob["Sabs"], RTOL_SPMM, "bwd S")
    assert_close(Gp, ob["Gprev"], ob["Gabs"], rtol, "bwd Gprev")
    assert_close(Y, ob["Y"], ob["Yabs"], rtol, "bwd Y")
    Sg = S.cpu().numpy()
    gt, gtabs = oracle.gemm(Sg, W, bf16=(prec == 1), transW=True, want_abs=True)
    assert_close(Gp, np.where(Zprev > 0, gt, 0), gtabs, rtol, "bwd Gprev vs oracle GEMM of the library's S")
    yt, ytabs = oracle.gemm(H, Sg, bf16=(prec == 1), transX=True, want_abs=True)
    assert_close(Y, yt, ytabs, rtol, "bwd Y vs oracle GEMM of the library's S")


@pytest.mark.parametrize("f", [64, 128])
def test_spmm_sweep_interval_barrier_gives_up_and_still_computes(f, force_sweep, monkeypatch):
    """Barrier mode: the workgroups of the sweep wait for each other at interval boundaries, for a
    bounded time.  Here every barrier is then told to expect more arrivals than there are
    workgroups (a host-side test hook), so the first wait runs into its 20-microsecond limit, the
    launch gives all barriers up and free-runs: every kernel still ends and the product is unchanged."""
    rng = np.random.default_rng(9 + f)
    m, n = 6000, 60_000
    rowptr, colidx, val = random_csr(m, n, 25, rng, hubs=[(3, 9000), (7, 3000), (2500, 1024)])
    B = synth.normal((n, f), f, synth.STREAM_H)
    ref, zabs = oracle.spmm(rowptr, colidx, val, B, want_abs=True)
    rp, ci, v = dev(rowptr), dev(colidx), dev(val)

    def run():
        ws = sagnn.spmm_csr_prepare(rp, ci, v, n, f)
        assert ws.info()["mode"] == 1
        out = sagnn.spmm_csr_tallskinny(rp, ci, v, dev(B), ws=ws)
        torch.cuda.synchronize()
        return out, ws

    monkeypatch.setenv("SAGNN_SWEEP_SYNC", "48")             # 384 slabs: 8 intervals
    monkeypatch.setenv("SAGNN_SWEEP_BARRIERS", "1")
    normal, ws = run()
    assert ws.info()["barriers"] == 1 and ws.info()["intervals"] > 1 and not ws.barriers_gave_up()
    assert_close(normal, ref, zabs, RTOL_SPMM, "with interval barriers")
    monkeypatch.setenv("SAGNN_SWEEP_SYNC_TEST_EXTRA", "1000")
    monkeypatch.setenv("SAGNN_SWEEP_SYNC_US", "20")
    gave_up, ws = run()
    assert ws.barriers_gave_up()
    assert torch.equal(gave_up, normal)                       # same summation order either way
    monkeypatch.delenv("SAGNN_SWEEP_SYNC_TEST_EXTRA")
    monkeypatch.delenv("SAGNN_SWEEP_BARRIERS")
    # pacing: every wavefront holds itself to a time schedule (here far slower than it could run,
    # so every boundary really waits); same bits again
    monkeypatch.setenv("SAGNN_SWEEP_PACE_PS", "2000000")
    paced, ws = run()
    assert ws.info()["pace_ps_per_step"] == 2000000 and ws.info()["barriers"] == 0
    assert torch.equal(paced, normal)
    monkeypatch.delenv("SAGNN_SWEEP_PACE_PS")                 # and without intervals at all (the default)
    monkeypatch.delenv("SAGNN_SWEEP_SYNC")
    plain, ws = run()
    assert ws.info()["intervals"] == 1
    assert_close(plain, ref, zabs, RTOL_SPMM, "without intervals")


# ------------------------------------------------------------------------------------ fused layer

@pytest.mark.parametrize("prec,fin,fout", [(0, 128, 128), (1, 256, 256), (0, 64, 32), (1, 128, 100), (0, 128, 256),
                                           (1, 64, 64), (1, 256, 36)])
@pytest.mark.parametrize("graph", ["hubs_and_empty_rows", "sbm", "rmat"])
def test_gcn_layer_fwd_fused(prec, fin, fout, graph, cfg1):
    """The one-kernel layer (T = A H kept on the chip, then the dense transform on the matrix
    cores) against the oracle's layer: without T (gcn_layer_fwd with d_T = NULL) and with T as a
    by-product.  Rows longer than 512 entries take the workgroup-shared path; m is not a
    multiple of the tile height."""
    rng = np.random.default_rng(fin + fout)
    if graph == "hubs_and_empty_rows":
        m, n = 4133, 9000
        rowptr, colidx, val = random_csr(m, n, 20, rng, empty_frac=0.1,
                                         hubs=[(5, 8000), (6, 513), (7, 512), (4132, 5000), (300, 300), (301, 2049)], dup=True)
    elif graph == "sbm":
        g = synth.sbm_graph(6000, 16, 40, 2, 3)
        rowptr, colidx, val, m, n = g.rowptr, g.colidx, g.val, g.m, g.n
    else:
        g = synth.rmat_graph(30_000, 1_500_000, 4)
        rowptr, colidx, val, m, n = g.rowptr, g.colidx, g.val, g.m, g.n
    H = synth.normal((n, fin), 1, synth.STREAM_H)
    W = synth.normal((fin, fout), 1, synth.STREAM_W, scale=1 / np.sqrt(fin))
    rp, ci, v = dev(rowptr), dev(colidx), dev(val)
    rtol = RTOL_BF16 if prec == 1 else RTOL_GEMM_FP32
    o = oracle.gcn_layer_fwd(rowptr, colidx, val, H, W, act=1, bf16=(prec == 1))
    T, Z, Ho = sagnn.gcn_layer_fwd(rp, ci, v, dev(H), dev(W), act=sagnn.ACT_RELU, prec=prec, want_t=False)
    torch.cuda.synchronize()
    assert T is None
    assert_close(Z, o["Z"], o["Zabs"], rtol, "fused Z")
    assert_close(Ho, o["H"], o["Zabs"], rtol, "fused H'")
    assert torch.equal(Ho, torch.clamp_min(Z, 0))
    T, Z2, _ = sagnn.gcn_layer_fwd(rp, ci, v, dev(H), dev(W), act=sagnn.ACT_IDENTITY, prec=prec, fused=True,
                                   want_h=False)
    torch.cuda.synchronize()
    assert_close(T, o["T"], o["Tabs"], RTOL_SPMM, "fused T")
    assert torch.equal(Z2, Z)
    zt, ztabs = oracle.gemm(T.cpu().numpy(), W, bf16=(prec == 1), want_abs=True)
    assert_close(Z, zt, ztabs, rtol, "fused Z vs oracle GEMM of the kernel's own T")


@pytest.mark.parametrize("prec,fin,fout", [(0, 128, 128), (1, 256, 256), (0, 64, 36), (1, 128, 100), (1, 256, 64),
                                           (2, 128, 128), (2, 256, 256), (2, 64, 36), (2, 128, 100)])
@pytest.mark.parametrize("graph", ["regular_all_rows_swept", "with_split_short_and_empty_rows"])
def test_gcn_layer_fwd_sweep_epilogue(prec, fin, fout, graph, monkeypatch):
    """The layer with d_T = NULL on a workspace prepared for the one-row-per-instruction sweep: the
    sweep kernel ends with the dense transform (form 2).  A near-regular graph whose rows are all
    swept, and one with rows cut into pieces, rows outside the sweep and empty rows (the small
    kernel for the rows the sweep does not finish)."""
    monkeypatch.setenv("SAGNN_SWEEP", "1")
    monkeypatch.setenv("SAGNN_SWEEP_GROUPS", "1")
    monkeypatch.setenv("SAGNN_SWEEP_MINDEG", "16")
    monkeypatch.setenv("SAGNN_SWEEP_PIECE", "1024")
    monkeypatch.setenv("SAGNN_SWEEP_SHORT_ROWS", "-1")   # short rows stay outside the sweep: the small kernel takes them
    rng = np.random.default_rng(fin * 3 + fout)
    if graph == "regular_all_rows_swept":
        g = synth.sbm_graph(6000, 16, 40, 2, 5)
        rowptr, colidx, val, m, n = g.rowptr, g.colidx, g.val, g.m, g.n
    else:
        m, n = 5003, 12000
        rowptr, colidx, val = random_csr(m, n, 30, rng, empty_frac=0.05,
                                         hubs=[(7, 5000), (8, 1025), (4000, 3), (4001, 15), (5002, 2100)])
    H = synth.normal((n, fin), 3, synth.STREAM_H)
    W = synth.normal((fin, fout), 3, synth.STREAM_W, scale=1 / np.sqrt(fin))
    rp, ci, v = dev(rowptr), dev(colidx), dev(val)
    ws = sagnn.spmm_csr_prepare(rp, ci, v, n, fin)
    info = ws.info()
    assert info["mode"] == 1 and info["groups"] == 1
    assert sagnn.gcn_layer_fwd_form(ws, fin, fout, prec) == 2
    if graph != "regular_all_rows_swept":
        assert info["split_rows"] >= 3 and info["chunk_rows"] > 0 and info["has_empty_rows"] == 1
    rtol = RTOL_BF16 if prec == 1 else RTOL_GEMM_FP32
    o = oracle.gcn_layer_fwd(rowptr, colidx, val, H, W, act=1, bf16=(prec == 1))
    Z0 = torch.full((m, fout), float("nan"), device="cuda")
    H0 = torch.full((m, fout), float("nan"), device="cuda")
    T, Z, Ho = sagnn.gcn_layer_fwd(rp, ci, v, dev(H), dev(W), act=sagnn.ACT_RELU, prec=prec, ws=ws,
                                   want_t=False, out=(None, Z0, H0))
    torch.cuda.synchronize()
    assert T is None
    assert_close(Z, o["Z"], o["Zabs"], rtol, "sweep epilogue Z")          # every row written (no NaN left)
    assert_close(Ho, o["H"], o["Zabs"], rtol, "sweep epilogue H'")
    assert torch.equal(Ho, torch.clamp_min(Z, 0))
    # only H' wanted, identity activation
    _, Zn, Hi = sagnn.gcn_layer_fwd(rp, ci, v, dev(H), dev(W), act=sagnn.ACT_IDENTITY, prec=prec, ws=ws,
                                    want_t=False, want_z=False)
    torch.cuda.synchronize()
    assert Zn is None and torch.equal(Hi, Z)
    # the schedules with lane groups (two / four rows of H per load) end with the same transform
    monkeypatch.setenv("SAGNN_SWEEP_GROUPS", "2")
    if fin in (64, 128):
        ws2 = sagnn.spmm_csr_prepare(rp, ci, v, n, fin)
        assert ws2.info()["groups"] == (2 if fin == 128 else 4)
        assert sagnn.gcn_layer_fwd_form(ws2, fin, fout, prec) == 2
        Z0.fill_(float("nan"))
        H0.fill_(float("nan"))
        _, Zg, Hg = sagnn.gcn_layer_fwd(rp, ci, v, dev(H), dev(W), act=sagnn.ACT_RELU, prec=prec, ws=ws2,
                                        want_t=False, out=(None, Z0, H0))
        torch.cuda.synchronize()
        assert_close(Zg, o["Z"], o["Zabs"], rtol, "sweep epilogue, lane groups, Z")
        assert_close(Hg, o["H"], o["Zabs"], rtol, "sweep epilogue, lane groups, H'")
    if fin == 64:
        # a workspace prepared for 128 columns (two lane groups) serves a 64-wide layer
        ws3 = sagnn.spmm_csr_prepare(rp, ci, v, n, 128)
        assert ws3.info()["groups"] == 2 and sagnn.gcn_layer_fwd_form(ws3, 64, fout, prec) == 2
        Z0.fill_(float("nan"))
        _, Zw, _ = sagnn.gcn_layer_fwd(rp, ci, v, dev(H), dev(W), act=sagnn.ACT_RELU, prec=prec, ws=ws3,
                                       want_t=False, want_h=False, out=(None, Z0, None))
        torch.cuda.synchronize()
        assert_close(Zw, o["Z"], o["Zabs"], rtol, "sweep epilogue, prepared 128 called 64")
    # a workspace of the 256-wide schedule cannot serve... nothing: every width has a form; an
    # unprepared call (no workspace) takes the row-range kernel
    # (the row-range kernel has no three-term form: such a call is an error, not a silent fp32 product)
    assert sagnn.gcn_layer_fwd_form(None, fin, fout, prec) == (0 if prec == 2 else 1)
    if prec == 2:
        with pytest.raises(sagnn.SagnnError):
            sagnn.gcn_layer_fwd(rp, ci, v, dev(H), dev(W), act=sagnn.ACT_RELU, prec=prec, want_t=False)


def test_gcn_layer_fwd_fused_degenerate_shapes():
    """No entries at all (every row of T is zero, so Z = 0 and H' = 0), a single row, and a
    matrix of one long row that the wavefronts of a workgroup share."""
    f = 128
    W = synth.normal((f, f), 2, synth.STREAM_W, scale=1 / np.sqrt(f))
    H = synth.normal((300, f), 2, synth.STREAM_H)
    empty = torch.zeros(0, dtype=torch.int32, device="cuda")
    rp = dev(np.zeros(8, np.int32))                       # 7 rows, no entries
    T, Z, Ho = sagnn.gcn_layer_fwd(rp, empty, torch.zeros(0, device="cuda"), dev(H), dev(W), want_t=False)
    torch.cuda.synchronize()
    assert T is None and Z.shape == (7, f) and not Z.any().item() and not Ho.any().item()
    for deg in (1, 299):                                  # one row; 299 > none of the thresholds, then a shared row below
        rowptr = np.array([0, deg], np.int32)
        colidx = np.arange(deg, dtype=np.int32)
        val = synth.normal((deg,), deg, synth.STREAM_G).astype(np.float32)
        o = oracle.gcn_layer_fwd(rowptr, colidx, val, H, W, act=1)
        _, Z, Ho = sagnn.gcn_layer_fwd(dev(rowptr), dev(colidx), dev(val), dev(H), dev(W), want_t=False)
        torch.cuda.synchronize()
        assert_close(Z, o["Z"], o["Zabs"], RTOL_GEMM_FP32, f"fused one row of {deg}")
        assert_close(Ho, o["H"], o["Zabs"], RTOL_GEMM_FP32, f"fused one row of {deg} H'")
    rng = np.random.default_rng(4)
    cols = np.sort(rng.integers(0, 300, size=3000)).astype(np.int32)      # one row of 3000 entries (duplicates summed)
    rowptr = np.array([0, 3000], np.int32)
    val = rng.standard_normal(3000).astype(np.float32)
    o = oracle.gcn_layer_fwd(rowptr, cols, val, H, W, act=1)
    _, Z, Ho = sagnn.gcn_layer_fwd(dev(rowptr), dev(cols), dev(val), dev(H), dev(W), want_t=False)
    torch.cuda.synchronize()
    assert_close(Z, o["Z"], o["Zabs"], RTOL_GEMM_FP32, "fused one shared row")


def test_gcn_layer_fwd_fused_strided_h_and_unsupported_shapes():
    rng = np.random.default_rng(2)
    m, n, f = 1000, 2000, 128
    rowptr, colidx, val = random_csr(m, n, 10, rng)
    H = synth.normal((n, f), 1, synth.STREAM_H)
    W = synth.normal((f, f), 1, synth.STREAM_W, scale=1 / np.sqrt(f))
    o = oracle.gcn_layer_fwd(rowptr, colidx, val, H, W, act=1)
    wide = torch.full((n, f + 12), 9.0, device="cuda")
    wide[:, :f] = dev(H)
    _, Z, _ = sagnn.gcn_layer_fwd(dev(rowptr), dev(colidx), dev(val), wide[:, :f], dev(W), want_t=False)
    torch.cuda.synchronize()
    assert_close(Z, o["Z"], o["Zabs"], RTOL_GEMM_FP32, "fused, ldh > f")
    for fin, fout, prec in ((256, 256, 0), (16, 16, 0), (192, 64, 1)):
        Hs = dev(synth.normal((n, fin), 1, synth.STREAM_H))
        Ws = dev(synth.normal((fin, fout), 1, synth.STREAM_W))
        with pytest.raises(sagnn.SagnnError) as ei:
            sagnn.gcn_layer_fwd(dev(rowptr), dev(colidx), dev(val), Hs, Ws, prec=prec, want_t=False)
        assert ei.value.code == -1
