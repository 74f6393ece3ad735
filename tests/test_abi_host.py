"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and argument validation rejects bad calls before any HIP call is made."""
import ctypes
import os
import re

import pytest

import paper_2504_04673_amd as sagnn
from paper_2504_04673_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "sagnn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(?:int|const char\*)\s+([a-z_0-9]+)\s*\(", text)))


def test_header_symbols_are_exported():
    L = sagnn.lib()
    names = declared_functions()
    assert len(names) >= 12
    for n in names:
        assert hasattr(L, n), n
    assert sorted(binding.EXPORTS) == names


def test_binding_constants_match_the_header():
    """The binding repeats the header's flag and mode values; a change on one side only would
    silently select another path."""
    text = open(os.path.join(ROOT, "include", "sagnn.h")).read()
    defs = {k: int(v.rstrip("u"), 0) for k, v in re.findall(r"#define\s+(SAGNN_[A-Z0-9_]+)\s+(-?\d+u?)\b", text)}
    pairs = {"SAGNN_PLAN_VALIDATE": binding.PLAN_VALIDATE, "SAGNN_PLAN_OBLIVIOUS": binding.PLAN_OBLIVIOUS,
             "SAGNN_PLAN_MULTIPASS": binding.PLAN_MULTIPASS, "SAGNN_GEMM_FP32": binding.GEMM_FP32,
             "SAGNN_GEMM_BF16": binding.GEMM_BF16, "SAGNN_GEMM_FP32_BF16X3": binding.GEMM_FP32_BF16X3,
             "SAGNN_ACT_IDENTITY": binding.ACT_IDENTITY, "SAGNN_ACT_RELU": binding.ACT_RELU}
    for name, value in pairs.items():
        assert defs[name] == value, name
    assert len({binding.PLAN_VALIDATE, binding.PLAN_OBLIVIOUS, binding.PLAN_MULTIPASS}) == 3
    assert binding.PLAN_VALIDATE & binding.PLAN_OBLIVIOUS == 0 and binding.PLAN_MULTIPASS & 3 == 0


def test_version_and_strerror():
    L = sagnn.lib()
    assert L.sagnn_version() >= 100
    for code in (0, -1, -2, -3, -4, -99):
        assert len(L.sagnn_strerror(code)) > 0


def test_workspace_queries():
    L = sagnn.lib()
    b = ctypes.c_size_t(0)
    assert L.spmm_plan_workspace_bytes(10, 1000, 50, 4, ctypes.byref(b)) == 0 and b.value >= 1000 // 8
    assert L.spmm_plan_workspace_bytes(10, 1000, 50, 0, ctypes.byref(b)) == -1
    assert L.spmm_plan_workspace_bytes(10, 1 << 33, 50, 1, ctypes.byref(b)) == -1
    assert L.spmm_csr_workspace_bytes(10, 1000, 128, ctypes.byref(b)) == 0
    assert b.value >= 4 * 128 * 4
    assert L.spmm_csr_workspace_bytes(10, 1000, 6, ctypes.byref(b)) == -1
    plain = b.value
    assert L.spmm_csr_workspace_bytes_opt(10, 20, 1000, 128, None, ctypes.byref(b)) == 0 and b.value == plain
    tiles = sagnn.SpmmOptions()
    tiles.dense_tiles = 1
    # the tile region holds the rest CSR (8 bytes per entry) and the tile streams (8 bytes per entry)
    assert L.spmm_csr_workspace_bytes_opt(10, 20, 1000, 128, ctypes.byref(tiles), ctypes.byref(b)) == 0
    assert b.value >= plain + 16 * 1000
    assert L.spmm_csr_workspace_bytes_opt(10, 20, 1000, 100, ctypes.byref(tiles), ctypes.byref(b)) == 0  # no tile kernel at this width
    assert L.spmm_csr_workspace_bytes_opt(10, -1, 1000, 128, None, ctypes.byref(b)) == -1
    assert L.spmm_csr_workspace_bytes_opt(10, 20, 1000, 128, None, None) == -1
    assert L.gcn_bwd_workspace_bytes(1000, 256, 256, ctypes.byref(b)) == 0 and b.value >= 256 * 256 * 4
    assert L.gcn_bwd_workspace_bytes(1000, 102, 256, ctypes.byref(b)) == -1
    assert L.gcn_bwd_workspace_bytes(1000, 16, 260, ctypes.byref(b)) == -1


def test_argument_validation_before_launch():
    L = sagnn.lib()
    # pack: bad f, null pointers, bad leading dimension
    assert L.spmm_pack_rows(None, 10, 16, 16, None, 5, None, 16, None) == -1
    assert L.spmm_pack_rows(None, 10, 16, 6, None, 0, None, 16, None) == -1
    assert L.spmm_pack_rows(None, 10, 8, 16, None, 0, None, 16, None) == -1
    assert L.spmm_pack_rows(None, 10, 16, 16, None, 0, None, 16, None) == 0     # N = 0: nothing to do
    # SpMM: null pointers with work to do, bad f
    assert L.spmm_csr_tallskinny(None, None, None, 4, 4, 4, None, 16, 16, None, 16, 0, None, 0, None) == -1
    assert L.spmm_csr_tallskinny(None, None, None, 0, 4, 0, None, 16, 16, None, 16, 0, None, 0, None) == 0
    assert L.spmm_csr_tallskinny(None, None, None, 4, 4, 4, None, 16, 18, None, 16, 0, None, 0, None) == -1
    assert L.spmm_csr_prepare(None, None, None, 4, 4, 4, 16, None, 0, None) == -1
    assert L.spmm_csr_prepare_tuned(None, None, None, 4, 4, 4, 16, None, 0, None, 16, None, 16, None, None, None) == -1
    assert L.spmm_csr_prepare_opt(None, None, None, 4, 4, 4, 16, None, 0, None, None) == -1
    bad = sagnn.SpmmOptions()
    bad.short_rows = 2                                    # not one of -1, 0, 1
    import ctypes as _c
    assert L.spmm_csr_prepare_opt(None, None, None, 4, 4, 4, 16, None, 0, _c.byref(bad), None) == -1
    bad = sagnn.SpmmOptions()
    bad.dense_tiles = 2                                   # not one of -1, 0, 1
    assert L.spmm_csr_prepare_opt(None, None, None, 4, 4, 4, 16, None, 0, _c.byref(bad), None) == -1
    assert L.spmm_csr_release(None) == -1
    assert L.spmm_csr_tile_info(None, None) == -1
    import numpy as _np
    info = _np.zeros(6, dtype=_np.int64)
    never_prepared = _c.c_void_p(0x1000)
    assert L.spmm_csr_tile_info(never_prepared, info.ctypes.data_as(_c.c_void_p)) == -1
    # plan: missing host arrays
    assert L.spmm_plan_needed_rows(None, None, 4, 4, 0, None, 1, None, 0, None, None, None, 0, 0, None) == -1
    # GEMM: unsupported sizes
    assert L.dense_gemm_act(None, 128, None, 128, 0, 10, 102, 128, 0, 0, None, 0, None, 0, None, 0, None) == -1
    assert L.dense_gemm_act(None, 128, None, 128, 0, 10, 128, 512, 0, 0, None, 0, None, 0, None, 0, None) == -1
    # split / stage loop: bad block count, missing arrays, too many blocks
    b = ctypes.c_size_t(0)
    assert L.spmm_split_workspace_bytes(100, 4, ctypes.byref(b)) == 0 and b.value > 0
    assert L.spmm_split_workspace_bytes(100, 257, ctypes.byref(b)) == -1
    assert L.spmm_split_colblocks(None, None, None, 4, 0, None, 2, None, None, None, None, None, 0, None) == -1
    assert L.spmm_stage_loop(None, 1, 4, None, 4, 16, 16, None, None, 4, None, 16, 0, None, None) == -1


def test_options_from_env_translation(monkeypatch):
    """The library reads no environment; the binding turns the experiment variables into the
    options struct (host only)."""
    for k in list(os.environ):
        if k.startswith("SAGNN_SWEEP") or k.startswith("SAGNN_TILE"):
            monkeypatch.delenv(k)
    o = sagnn.options_from_env()
    assert all(getattr(o, n) == 0 for n, _ in sagnn.SpmmOptions._fields_)
    monkeypatch.setenv("SAGNN_SWEEP", "1")
    monkeypatch.setenv("SAGNN_SWEEP_SLAB_MB", "0")
    monkeypatch.setenv("SAGNN_SWEEP_LPT", "0")
    monkeypatch.setenv("SAGNN_SWEEP_SYNC", "0")
    monkeypatch.setenv("SAGNN_SWEEP_PIECE", "1024")
    o = sagnn.options_from_env()
    assert (o.schedule, o.slab_kb, o.snake, o.sync_slabs, o.piece) == (2, -1, 1, -1, 1024)
    monkeypatch.setenv("SAGNN_SWEEP", "0")
    monkeypatch.setenv("SAGNN_SWEEP_SLAB_MB", "2")
    monkeypatch.setenv("SAGNN_SWEEP_SYNC", "8")
    o = sagnn.options_from_env()
    assert (o.schedule, o.slab_kb, o.sync_slabs) == (1, 2048, 8)
    monkeypatch.setenv("SAGNN_TILES", "1")
    monkeypatch.setenv("SAGNN_TILE_REUSE_X10", "40")
    o = sagnn.options_from_env()
    assert (o.dense_tiles, o.tile_reuse_x10) == (1, 40)
    src = open(os.path.join(ROOT, "paper_2504_04673_amd", "csrc", "spmm_sweep.hip")).read()
    assert "getenv" not in open(os.path.join(ROOT, "paper_2504_04673_amd", "csrc", "tiles.hip")).read()
    assert "getenv" not in src and "getenv" not in open(os.path.join(ROOT, "paper_2504_04673_amd", "csrc", "spmm.hip")).read()


def test_volume_stats_host_only():
    """spmm_volume_stats is host arithmetic: it runs without a GPU.  Hand-counted 3 x 3 case."""
    st = sagnn.spmm_volume_stats([[9, 1, 2], [4, 9, 0], [5, 6, 9]], 2, 4)
    assert st["total_bytes"] == 144 and st["avg_bytes"] == 48 and st["max_recv_bytes"] == 88
    assert st["max_send_bytes"] == 72 and st["cut_rows"] == 6 and st["cut_bytes"] == 48
    assert st["send_imbalance_pct"] == pytest.approx(50.0)
    assert sagnn.lib().spmm_volume_stats(None, 3, 2, 4, None) == -1


def test_binding_refuses_cpu_tensors():
    import torch
    with pytest.raises(ValueError):
        sagnn.spmm_pack_rows(torch.zeros(4, 4), torch.zeros(2, dtype=torch.int32))


def test_bench_refuses_more_than_one_gpu():
    """The benchmark measures one GPU's share: --gpus N > 1 exits with a message (no GPU needed)."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr or "one GPU" in r.stderr.lower()
    assert r.stdout.strip() == ""
