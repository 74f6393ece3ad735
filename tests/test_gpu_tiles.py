"""GPU parity of the dense-tile schedule of the local SpMM (Alg. 1 / 2, `Z <- Z + SpMM(A, H)`): the
tiles of A that are dense enough are multiplied out of LDS, the rest through the other schedules;
the sum is compared element by element with the CPU oracle within 1e-5 * sum|terms|."""
import numpy as np
import pytest
import torch

import oracle
import paper_2504_04673_amd as sagnn
from paper_2504_04673_amd import synth
from tests.test_gpu_parity import RTOL_SPMM, _strided, random_csr
from tests.util import assert_close, dev

pytestmark = pytest.mark.gpu


def _prepare_tiles(rowptr, colidx, val, k, f, monkeypatch, reuse_x10=None, expect=True):
    monkeypatch.setenv("SAGNN_TILES", "1")
    if reuse_x10 is not None:
        monkeypatch.setenv("SAGNN_TILE_REUSE_X10", str(reuse_x10))
    rp, ci, v = dev(rowptr), dev(colidx), dev(val)
    ws = sagnn.spmm_csr_prepare(rp, ci, v, k, f)
    ti = ws.tile_info()
    if expect:
        assert ti["tiles"] == 1 and ti["tile_entries"] > 0, ti
        assert ti["tile_entries"] + ti["rest_entries"] == len(colidx), ti
    return rp, ci, v, ws, ti


@pytest.mark.parametrize("inner", ["nonzero_splitting", "sweep"])
@pytest.mark.parametrize("f", [64, 128, 256])
def test_spmm_dense_tiles_power_law(f, inner, monkeypatch):
    """Power-law graph dense enough that many tiles qualify: hub rows lose most of their entries to
    the tiles (some all of them), the rest goes through either of the other schedules; overwrite,
    accumulate, reproducibility across preparations, strided operands."""
    if inner == "sweep":
        monkeypatch.setenv("SAGNN_SWEEP", "1")
        monkeypatch.setenv("SAGNN_SWEEP_MINDEG", "16")
        monkeypatch.setenv("SAGNN_SWEEP_PIECE", "1024")
        monkeypatch.setenv("SAGNN_SWEEP_SLAB_MB", "0")
    else:
        monkeypatch.setenv("SAGNN_SWEEP", "0")
    g = synth.rmat_graph(6000, 700_000, 5)
    n = g.n
    B = synth.normal((n, f), f, synth.STREAM_H)
    C0 = synth.normal((g.m, f), f + 1, synth.STREAM_G)
    rp, ci, v, ws, ti = _prepare_tiles(g.rowptr, g.colidx, g.val, n, f, monkeypatch)
    assert ws.info()["mode"] == (1 if inner == "sweep" else 0), ws.info()
    assert ti["kept_tiles"] >= 8 and ti["items"] >= 2, ti
    ref, zabs = oracle.spmm(g.rowptr, g.colidx, g.val, B, want_abs=True)
    got = sagnn.spmm_csr_tallskinny(rp, ci, v, dev(B), ws=ws)
    torch.cuda.synchronize()
    assert_close(got, ref, zabs, RTOL_SPMM, f"tiles f={f} {inner}")
    rp2, ci2, v2, ws2, ti2 = _prepare_tiles(g.rowptr, g.colidx, g.val, n, f, monkeypatch)
    assert ti2 == ti
    got_again = sagnn.spmm_csr_tallskinny(rp2, ci2, v2, dev(B), ws=ws2)
    assert torch.equal(got, got_again)
    ref2, zabs2 = oracle.spmm(g.rowptr, g.colidx, g.val, B, C=C0, want_abs=True)
    Bv, _ = _strided(B, 4, 123.0)
    Cv, Cw = _strided(C0, 8, -77.0)
    sagnn.spmm_csr_tallskinny(rp, ci, v, Bv, C=Cv, accumulate=True, ws=ws)
    torch.cuda.synchronize()
    assert_close(Cv, ref2, zabs2, RTOL_SPMM, f"tiles accumulate strided f={f} {inner}")
    assert torch.all(Cw[:, f:] == -77.0)


def test_spmm_dense_tiles_rectangular_unsorted_duplicates(monkeypatch):
    """Rectangular matrix, columns unsorted with repeats, empty rows, a few hubs; a low threshold
    keeps sparse tiles too (the floor of 256 entries per tile still applies)."""
    monkeypatch.setenv("SAGNN_SWEEP", "0")
    rng = np.random.default_rng(77)
    m, n, f = 3001, 2500, 128
    rowptr, colidx, val = random_csr(m, n, 14, rng, empty_frac=0.15, hubs=[(7, 3000), (1500, 777), (3000, 300)],
                                     dup=True)
    B = synth.normal((n, f), 3, synth.STREAM_H)
    rp, ci, v, ws, ti = _prepare_tiles(rowptr, colidx, val, n, f, monkeypatch, reuse_x10=1)
    ref, zabs = oracle.spmm(rowptr, colidx, val, B, want_abs=True)
    got = sagnn.spmm_csr_tallskinny(rp, ci, v, dev(B), ws=ws)
    torch.cuda.synchronize()
    assert_close(got, ref, zabs, RTOL_SPMM, "tiles rectangular")
    # an operand with more rows than the preparation saw is fine, one with fewer is refused
    B_more = np.concatenate([B, synth.normal((5, f), 4, synth.STREAM_H)])
    got = sagnn.spmm_csr_tallskinny(rp, ci, v, dev(B_more), ws=ws)
    torch.cuda.synchronize()
    assert_close(got, ref, zabs, RTOL_SPMM, "tiles rectangular, taller operand")
    with pytest.raises((sagnn.SagnnError, ValueError)):
        sagnn.spmm_csr_tallskinny(rp, ci, v, dev(B[:-1]), ws=ws)
    # the width is part of the tile streams: a narrower call is refused
    with pytest.raises(sagnn.SagnnError):
        sagnn.spmm_csr_tallskinny(rp, ci, v, dev(B[:, :64].copy()), ws=ws)


def test_spmm_dense_tiles_nothing_dense_enough(monkeypatch):
    """No tile reaches the threshold: the preparation is the plain one and says so."""
    rng = np.random.default_rng(5)
    m, n, f = 4000, 50_000, 128
    rowptr, colidx, val = random_csr(m, n, 6, rng)
    rp, ci, v, ws, ti = _prepare_tiles(rowptr, colidx, val, n, f, monkeypatch, expect=False)
    assert ti["tiles"] == 0, ti
    B = synth.normal((n, f), 9, synth.STREAM_H)
    ref, zabs = oracle.spmm(rowptr, colidx, val, B, want_abs=True)
    got = sagnn.spmm_csr_tallskinny(rp, ci, v, dev(B), ws=ws)
    torch.cuda.synchronize()
    assert_close(got, ref, zabs, RTOL_SPMM, "no tiles")


@pytest.mark.parametrize("f", [64, 128, 256])
def test_spmm_dense_tiles_rows_of_equal_terms(f, monkeypatch):
    """Worst case for fp32 summation: every product of a row is the same positive number, so each
    addition of a serial run rounds the same way.  A fully dense block (every entry in a kept tile,
    the rest CSR empty) with 2048 entries per row must stay within 1e-5."""
    monkeypatch.setenv("SAGNN_SWEEP", "0")
    m, n = 700, 2048
    rowptr = (np.arange(m + 1, dtype=np.int64) * n).astype(np.int32)
    colidx = np.tile(np.arange(n, dtype=np.int32), m)
    val = np.full(m * n, 0.37, np.float32)
    B = np.tile(np.linspace(0.5, 1.5, f, dtype=np.float32), (n, 1))
    rp, ci, v, ws, ti = _prepare_tiles(rowptr, colidx, val, n, f, monkeypatch)
    assert ti["rest_entries"] == 0, ti
    ref, zabs = oracle.spmm(rowptr, colidx, val, B, want_abs=True)
    got = sagnn.spmm_csr_tallskinny(rp, ci, v, dev(B), ws=ws)
    torch.cuda.synchronize()
    assert_close(got, ref, zabs, RTOL_SPMM, f"tiles equal terms f={f}")


def test_spmm_dense_tiles_layer_falls_back_to_split_or_row_range_form(monkeypatch):
    """gcn_layer_fwd on a workspace with dense tiles: with T wanted it is product + dense transform,
    without T the row-range kernel; both against the oracle's layer."""
    monkeypatch.setenv("SAGNN_SWEEP", "1")
    monkeypatch.setenv("SAGNN_SWEEP_MINDEG", "16")
    g = synth.rmat_graph(5000, 500_000, 11)
    f = 128
    H = synth.normal((g.n, f), 1, synth.STREAM_H)
    W = synth.normal((f, f), 2, synth.STREAM_W, scale=1 / np.sqrt(f))
    rp, ci, v, ws, ti = _prepare_tiles(g.rowptr, g.colidx, g.val, g.n, f, monkeypatch)
    assert sagnn.gcn_layer_fwd_form(ws, f, f) != 2
    ref = oracle.gcn_layer_fwd(g.rowptr, g.colidx, g.val, H, W)
    T, Z, Ho = sagnn.gcn_layer_fwd(rp, ci, v, dev(H), dev(W), ws=ws)
    torch.cuda.synchronize()
    assert_close(T, ref["T"], ref["Tabs"], RTOL_SPMM, "layer T with tiles")
    assert_close(Z, ref["Z"], ref["Zabs"], 2e-5, "layer Z with tiles")
    _, Z2, _ = sagnn.gcn_layer_fwd(rp, ci, v, dev(H), dev(W), ws=ws, want_t=False)
    torch.cuda.synchronize()
    assert_close(Z2, ref["Z"], ref["Zabs"], 2e-5, "layer Z with tiles, T not stored")


def test_spmm_dense_tiles_full_size_cfg2(monkeypatch):
    """The configuration the dense tiles were built for, at full size: the whole product against the
    oracle, and the eigenvector closed form A sqrt(d) = sqrt(d) (all terms positive, per-column
    scales), on the launch configuration that profiles/ holds the counters of."""
    from paper_2504_04673_amd import workloads
    from tests.test_gpu_fullsize import check_eigenvector, check_spmm_full
    wl = workloads.cfg2()
    g, f = wl.g, 128
    rp, ci, v, ws, ti = _prepare_tiles(g.rowptr, g.colidx, g.val, g.n, f, monkeypatch)
    assert ti["tile_entries"] > 0.8 * g.nnz and ws.info()["mode"] == 1, (ti, ws.info())
    Z = sagnn.spmm_csr_tallskinny(rp, ci, v, dev(wl.H), ws=ws)
    torch.cuda.synchronize()
    check_spmm_full(g, Z, wl.H, "cfg2 with dense tiles")
    check_eigenvector(g, f, ws, rp, ci, v)


@pytest.mark.parametrize("m,k", [(40, 50), (513, 129), (1, 300), (600, 1)])
def test_spmm_dense_tiles_ragged_small_shapes(m, k, monkeypatch):
    """Fully dense small matrices whose last row group and last column chunk are partial (one row,
    one column): every entry lands in a kept tile or, below 256 entries per tile, in the rest."""
    monkeypatch.setenv("SAGNN_SWEEP", "0")
    f = 128
    rng = np.random.default_rng(m * 1000 + k)
    rowptr = (np.arange(m + 1, dtype=np.int64) * k).astype(np.int32)
    colidx = np.tile(np.arange(k, dtype=np.int32), m)
    val = rng.standard_normal(m * k).astype(np.float32)
    B = synth.normal((k, f), 21, synth.STREAM_H)
    rp, ci, v, ws, ti = _prepare_tiles(rowptr, colidx, val, k, f, monkeypatch, expect=False)
    # a tile (512 rows x 128 columns here) is kept from 320 entries on
    fullest = min(m, 512) * min(k, 128)
    assert ti["tiles"] == (1 if fullest >= 320 else 0), ti
    ref, zabs = oracle.spmm(rowptr, colidx, val, B, want_abs=True)
    C0 = synth.normal((m, f), 22, synth.STREAM_G)
    got = sagnn.spmm_csr_tallskinny(rp, ci, v, dev(B), ws=ws)
    torch.cuda.synchronize()
    assert_close(got, ref, zabs, RTOL_SPMM, f"dense {m}x{k}")
    ref2, zabs2 = oracle.spmm(rowptr, colidx, val, B, C=C0, want_abs=True)
    got2 = sagnn.spmm_csr_tallskinny(rp, ci, v, dev(B), C=dev(C0), accumulate=True, ws=ws)
    torch.cuda.synchronize()
    assert_close(got2, ref2, zabs2, RTOL_SPMM, f"dense {m}x{k} accumulate")
