"""ctypes binding of libsagnn.so: same names as the C ABI, argument marshalling only."""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import numpy as np
import torch

from . import build as _build

ACT_IDENTITY, ACT_RELU = 0, 1
GEMM_FP32, GEMM_BF16, GEMM_FP32_BF16X3 = 0, 1, 2
PLAN_VALIDATE, PLAN_OBLIVIOUS, PLAN_MULTIPASS = 1, 2, 4

EXPORTS = [
    "sagnn_strerror", "sagnn_last_hip_error", "sagnn_version",
    "spmm_plan_workspace_bytes", "spmm_plan_needed_rows", "spmm_plan_needed_rows_noalloc", "spmm_pack_rows",
    "spmm_csr_workspace_bytes", "spmm_csr_workspace_bytes_opt", "spmm_csr_tile_info", "spmm_csr_prepare", "spmm_csr_prepare_opt", "spmm_csr_prepare_tuned", "spmm_csr_schedule_info",
    "spmm_csr_release", "spmm_csr_tallskinny",
    "dense_gemm_act", "gcn_layer_fwd", "gcn_layer_fwd_fused", "gcn_layer_fwd_form", "gcn_bwd_workspace_bytes", "gcn_layer_bwd",
    "spmm_split_workspace_bytes", "spmm_split_colblocks", "spmm_stage_loop", "spmm_volume_stats",
    "spmm_transpose_workspace_bytes", "spmm_csr_transpose",
    "spmm_permute_workspace_bytes", "spmm_perm_from_labels", "spmm_csr_permute_symmetric",
]


class _Stage(ctypes.Structure):
    """struct sagnn_stage of the C header."""
    _fields_ = [("d_rowptr", ctypes.c_void_p), ("d_colidx", ctypes.c_void_p),
                ("d_val", ctypes.c_void_p), ("nnz", ctypes.c_int64), ("d_rows", ctypes.c_void_p),
                ("N", ctypes.c_int64), ("d_ws", ctypes.c_void_p), ("ws_bytes", ctypes.c_size_t)]


class SpmmOptions(ctypes.Structure):
    """struct sagnn_spmm_options of the C header (zero = let the library decide)."""
    _fields_ = [(n, ctypes.c_int32) for n in
                ("schedule", "min_long", "piece", "slab_kb", "min_waves", "window_pct", "snake", "groups",
                 "sync_slabs", "pace_ps_per_step", "barriers", "sync_timeout_us", "sync_test_extra",
                 "narrow_slots", "slab_width", "short_rows", "dense_tiles", "tile_reuse_x10")]


# The library itself reads no environment variables.  For experiments and for tests that force a
# code path on small inputs, the binding translates these variables into the options struct:
#   SAGNN_SWEEP=0|1 (never / whenever possible), SAGNN_SWEEP_MINDEG, SAGNN_SWEEP_PIECE,
#   SAGNN_SWEEP_SLAB_MB (0 = as many slabs as possible), SAGNN_SWEEP_MIN_WAVES,
#   SAGNN_SWEEP_WINDOW_PCT (0 = one window), SAGNN_SWEEP_LPT=0 (snake dealing),
#   SAGNN_SWEEP_GROUPS=1|2, SAGNN_SWEEP_SYNC (slabs per interval, 0 = one interval),
#   SAGNN_SWEEP_PACE_PS (picoseconds per stream step, -1 = never pace), SAGNN_SWEEP_BARRIERS=1,
#   SAGNN_SWEEP_SYNC_US, SAGNN_SWEEP_SYNC_TEST_EXTRA, SAGNN_SWEEP_NARROW_SLOTS=1, SAGNN_SWEEP_SLAB_WIDTH=128,
#   SAGNN_SWEEP_SHORT_ROWS=1 (short rows swept as whole rows),
#   SAGNN_TILES=1|-1 (dense tiles out of LDS: always / never), SAGNN_TILE_REUSE_X10
def options_from_env() -> SpmmOptions:
    o = SpmmOptions()
    env = os.environ.get

    def num(name):
        v = env(name)
        return None if v is None or v == "" else int(v)

    v = num("SAGNN_SWEEP")
    if v is not None:
        o.schedule = 1 if v == 0 else (2 if v == 1 else 0)
    for name, field in (("SAGNN_SWEEP_MINDEG", "min_long"), ("SAGNN_SWEEP_PIECE", "piece"),
                        ("SAGNN_SWEEP_MIN_WAVES", "min_waves"), ("SAGNN_SWEEP_GROUPS", "groups"),
                        ("SAGNN_SWEEP_SYNC_US", "sync_timeout_us"), ("SAGNN_SWEEP_PACE_PS", "pace_ps_per_step"),
                        ("SAGNN_SWEEP_BARRIERS", "barriers"), ("SAGNN_SWEEP_NARROW_SLOTS", "narrow_slots"),
                        ("SAGNN_SWEEP_SYNC_TEST_EXTRA", "sync_test_extra"), ("SAGNN_SWEEP_SLAB_WIDTH", "slab_width"),
                        ("SAGNN_SWEEP_SHORT_ROWS", "short_rows"), ("SAGNN_TILES", "dense_tiles"),
                        ("SAGNN_TILE_REUSE_X10", "tile_reuse_x10")):
        v = num(name)
        if v is not None:
            setattr(o, field, v)
    v = num("SAGNN_SWEEP_SLAB_MB")
    if v is not None:
        o.slab_kb = -1 if v <= 0 else v * 1024
    v = num("SAGNN_SWEEP_WINDOW_PCT")
    if v is not None:
        o.window_pct = -1 if v <= 0 else v
    v = num("SAGNN_SWEEP_LPT")
    if v is not None:
        o.snake = 1 if v == 0 else 0
    v = num("SAGNN_SWEEP_SYNC")
    if v is not None:
        o.sync_slabs = -1 if v <= 0 else v
    return o


class SagnnError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = lib().sagnn_strerror(code).decode()
        extra = f" (hipError {lib().sagnn_last_hip_error()})" if code == -4 else ""
        super().__init__(f"{where}: {msg}{extra} [{code}]")


_lib = None


def lib_path() -> str:
    return _build.LIB


def lib():
    """Load libsagnn.so (building it first only if it does not exist)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_build.LIB):
            _build.build_hip()
        L = ctypes.CDLL(_build.LIB)
        i64, i32, u32, vp, sz = (ctypes.c_int64, ctypes.c_int32, ctypes.c_uint32, ctypes.c_void_p,
                                 ctypes.c_size_t)
        psz = ctypes.POINTER(ctypes.c_size_t)
        L.sagnn_strerror.restype = ctypes.c_char_p
        L.sagnn_strerror.argtypes = [ctypes.c_int]
        L.sagnn_last_hip_error.restype = ctypes.c_int
        L.sagnn_version.restype = ctypes.c_int
        L.spmm_plan_workspace_bytes.argtypes = [i64, i64, i64, i32, psz]
        L.spmm_plan_needed_rows.argtypes = [vp, vp, i64, i64, i64, vp, i32, vp, i64, vp, vp, vp, sz,
                                            u32, vp]
        L.spmm_plan_needed_rows_noalloc.argtypes = [vp, vp, i64, i64, i64, vp, i32, vp, i64, vp, vp, u32, vp]
        L.spmm_pack_rows.argtypes = [vp, i64, i64, i32, vp, i64, vp, i64, vp]
        L.spmm_csr_workspace_bytes.argtypes = [i64, i64, i32, psz]
        L.spmm_csr_workspace_bytes_opt.argtypes = [i64, i64, i64, i32, vp, psz]
        L.spmm_csr_tile_info.argtypes = [vp, vp]
        L.spmm_csr_prepare.argtypes = [vp, vp, vp, i64, i64, i64, i32, vp, sz, vp]
        L.spmm_csr_prepare_opt.argtypes = [vp, vp, vp, i64, i64, i64, i32, vp, sz, vp, vp]
        L.spmm_csr_prepare_tuned.argtypes = [vp, vp, vp, i64, i64, i64, i32, vp, sz, vp, i64, vp, i64, vp, vp, vp]
        L.spmm_csr_schedule_info.argtypes = [vp, vp]
        L.spmm_csr_release.argtypes = [vp]
        L.spmm_csr_tallskinny.argtypes = [vp, vp, vp, i64, i64, i64, vp, i64, i32, vp, i64, i32, vp,
                                          sz, vp]
        L.dense_gemm_act.argtypes = [vp, i64, vp, i64, i32, i64, i32, i32, i32, i32, vp, i64, vp, i64,
                                     vp, i64, vp]
        L.gcn_layer_fwd.argtypes = [vp, vp, vp, i64, i64, i64, vp, i64, i32, vp, i32, i32, i32, vp,
                                    vp, vp, vp, sz, vp]
        L.gcn_layer_fwd_fused.argtypes = [vp, vp, vp, i64, i64, i64, vp, i64, i32, vp, i32, i32, i32, vp,
                                          vp, vp, vp]
        L.gcn_layer_fwd_form.argtypes = [vp, i32, i32, i32, ctypes.POINTER(ctypes.c_int32)]
        L.gcn_bwd_workspace_bytes.argtypes = [i64, i32, i32, psz]
        L.gcn_layer_bwd.argtypes = [vp, vp, vp, i64, i64, vp, i32, vp, i32, vp, vp, i32, vp, vp, vp,
                                    vp, sz, vp, sz, vp]
        L.spmm_split_workspace_bytes.argtypes = [i64, i32, psz]
        L.spmm_split_colblocks.argtypes = [vp, vp, vp, i64, i64, vp, i32, vp, vp, vp, vp, vp, sz, vp]
        L.spmm_stage_loop.argtypes = [vp, i32, i64, vp, i64, i64, i32, vp, vp, i64, vp, i64, i32, vp,
                                      vp]
        L.spmm_volume_stats.argtypes = [vp, i32, i32, i32, vp]
        L.spmm_transpose_workspace_bytes.argtypes = [i64, psz]
        L.spmm_csr_transpose.argtypes = [vp, vp, vp, i64, i64, i64, vp, vp, vp, vp, sz, vp]
        L.spmm_permute_workspace_bytes.argtypes = [i64, i64, psz]
        L.spmm_perm_from_labels.argtypes = [vp, i64, i32, vp, vp, vp, vp, sz, vp]
        L.spmm_csr_permute_symmetric.argtypes = [vp, vp, vp, i64, i64, vp, vp, vp, vp, vp, sz, vp]
        for name in EXPORTS[3:]:
            getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def _check(rc: int, where: str):
    if rc != 0:
        raise SagnnError(rc, where)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t: torch.Tensor, dtype, name: str):
    if not t.is_cuda:
        raise ValueError(f"{name} must be a CUDA/HIP tensor (there is no CPU path)")
    if t.dtype != dtype or not t.is_contiguous():
        raise ValueError(f"{name}: expected contiguous {dtype}")
    return t


def _mat(t: torch.Tensor, name: str):
    """A row-major fp32 matrix, possibly a column slice of a wider one: unit stride along a row,
    the row stride is passed to the library as the leading dimension."""
    if not t.is_cuda:
        raise ValueError(f"{name} must be a CUDA/HIP tensor (there is no CPU path)")
    if t.dtype != torch.float32 or t.dim() != 2:
        raise ValueError(f"{name}: expected a 2-D float32 tensor")
    if t.shape[0] > 1 and t.shape[1] > 0 and (t.stride(1) != 1 or t.stride(0) < t.shape[1]):
        raise ValueError(f"{name}: rows must be contiguous (unit stride inside a row)")
    return t


def _ld(t: torch.Tensor) -> int:
    return int(t.stride(0)) if t.shape[0] > 1 else max(int(t.stride(0)), int(t.shape[1]))


def _ws(nbytes: int, device) -> torch.Tensor:
    # torch's caching allocator returns 512-byte aligned blocks
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


@dataclass
class Plan:
    needed: torch.Tensor          # int32 [N], ascending global column ids
    blk_off: np.ndarray           # int64 [nb+1] (host)
    colidx_compact: torch.Tensor  # int32 [nnz] or None

    @property
    def N(self) -> int:
        return int(self.blk_off[-1])


def _plan_flags(validate, oblivious, multipass):
    if multipass is None:
        multipass = os.environ.get("SAGNN_PLAN_MULTIPASS", "0") not in ("", "0")
    return ((PLAN_VALIDATE if validate else 0) | (PLAN_OBLIVIOUS if oblivious else 0) |
            (PLAN_MULTIPASS if multipass else 0))


def spmm_plan_needed_rows(rowptr, colidx, n: int, colblk, want_compact=True, validate=False,
                          needed_cap=None, bufs=None, oblivious=False, multipass=None) -> Plan:
    """NnzCols of every column block (Sec. 4.1).  Outputs are torch tensors; `needed` is sized
    min(n, nnz) unless needed_cap is given.  `bufs` = (ws, needed, compact) reuses buffers of an
    earlier call (see plan_buffers) so that a repeated call allocates nothing.  `multipass=True`
    (default: the environment variable SAGNN_PLAN_MULTIPASS) keeps small blocks off the one-launch
    path."""
    rowptr = _dev(rowptr, torch.int32, "rowptr")
    colidx = _dev(colidx, torch.int32, "colidx")
    m, nnz = rowptr.numel() - 1, colidx.numel()
    colblk = np.ascontiguousarray(colblk, dtype=np.int64)
    nb = colblk.size - 1
    L = lib()
    cap = int((n if oblivious else min(n, nnz)) if needed_cap is None else needed_cap)
    if bufs is None:
        bufs = plan_buffers(m, n, nnz, nb, rowptr.device, cap, want_compact)
    ws, needed, compact = bufs
    blk_off = np.zeros(nb + 1, dtype=np.int64)
    rc = L.spmm_plan_needed_rows(_ptr(rowptr), _ptr(colidx), m, n, nnz,
                                 colblk.ctypes.data_as(ctypes.c_void_p), nb, _ptr(needed), cap,
                                 blk_off.ctypes.data_as(ctypes.c_void_p), _ptr(compact), _ptr(ws),
                                 ws.numel(), _plan_flags(validate, oblivious, multipass), _stream())
    _check(rc, "spmm_plan_needed_rows")
    N = int(blk_off[-1])
    return Plan(needed[:N], blk_off, compact[:nnz] if compact is not None else None)


def spmm_plan_needed_rows_noalloc(rowptr, colidx, n: int, colblk, needed, compact=None, validate=False,
                                  oblivious=False, multipass=None) -> Plan:
    """spmm_plan_needed_rows without a workspace: the library's fixed per-GPU scratch array is
    used and nothing is allocated, here or in the library.  `needed` (int32, capacity = its
    length) and `compact` (int32, nnz entries, or None) are the caller's output buffers."""
    rowptr = _dev(rowptr, torch.int32, "rowptr")
    colidx = _dev(colidx, torch.int32, "colidx")
    needed = _dev(needed, torch.int32, "needed")
    if compact is not None:
        compact = _dev(compact, torch.int32, "compact")
    m, nnz = rowptr.numel() - 1, colidx.numel()
    colblk = np.ascontiguousarray(colblk, dtype=np.int64)
    nb = colblk.size - 1
    blk_off = np.zeros(nb + 1, dtype=np.int64)
    rc = lib().spmm_plan_needed_rows_noalloc(
        _ptr(rowptr), _ptr(colidx), m, n, nnz, colblk.ctypes.data_as(ctypes.c_void_p), nb, _ptr(needed),
        needed.numel(), blk_off.ctypes.data_as(ctypes.c_void_p), _ptr(compact),
        _plan_flags(validate, oblivious, multipass), _stream())
    _check(rc, "spmm_plan_needed_rows_noalloc")
    N = int(blk_off[-1])
    return Plan(needed[:N], blk_off, compact[:nnz] if compact is not None else None)


def plan_buffers(m, n, nnz, nb, device, cap=None, want_compact=True):
    """Workspace and output buffers of spmm_plan_needed_rows."""
    wsb = ctypes.c_size_t(0)
    _check(lib().spmm_plan_workspace_bytes(m, n, nnz, nb, ctypes.byref(wsb)), "spmm_plan_workspace_bytes")
    cap = int(min(n, nnz) if cap is None else cap)
    ws = _ws(wsb.value, device)
    needed = torch.empty(max(cap, 1), dtype=torch.int32, device=device)
    compact = torch.empty(max(nnz, 1), dtype=torch.int32, device=device) if want_compact else None
    return ws, needed, compact


def spmm_pack_rows(H, rows, out=None):
    """out[r,:] = H[rows[r],:] (Alg. 1, packed buffer)."""
    H = _mat(H, "H")
    rows = _dev(rows, torch.int32, "rows")
    n, f = H.shape
    N = rows.numel()
    if out is None:
        out = torch.empty((N, f), dtype=torch.float32, device=H.device)
    _mat(out, "out")
    _check(lib().spmm_pack_rows(_ptr(H), n, _ld(H), f, _ptr(rows), N, _ptr(out), _ld(out),
                                _stream()), "spmm_pack_rows")
    return out


@dataclass
class SpmmWorkspace:
    buf: torch.Tensor
    m: int
    nnz: int
    f: int
    choice: dict = None           # filled in by spmm_csr_prepare_tuned
    k: int = 0                    # rows of B the schedule was prepared for

    def release(self):
        """Drop the library's host descriptor of this workspace (spmm_csr_release)."""
        if self.buf is not None:
            lib().spmm_csr_release(_ptr(self.buf))
            self.buf = None

    def __del__(self):
        try:
            self.release()
        except Exception:
            pass

    def info(self) -> dict:
        """Schedule chosen by spmm_csr_prepare (see spmm_csr_schedule_info)."""
        a = np.zeros(16, dtype=np.int64)
        _check(lib().spmm_csr_schedule_info(_ptr(self.buf), a.ctypes.data_as(ctypes.c_void_p)),
               "spmm_csr_schedule_info")
        keys = ("mode", "sweep_waves", "sweep_entries", "chunk_rows", "chunk_entries", "chunks",
                "split_rows", "has_empty_rows", "intervals", "sync_slabs", "gave_up_offset", "groups",
                "pace_ps_per_step", "barriers", "slots", "longest_stream_steps")
        return dict(zip(keys, (int(x) for x in a)))

    def tile_info(self) -> dict:
        """What a preparation with dense tiles decided (see spmm_csr_tile_info)."""
        a = np.zeros(6, dtype=np.int64)
        _check(lib().spmm_csr_tile_info(_ptr(self.buf), a.ctypes.data_as(ctypes.c_void_p)), "spmm_csr_tile_info")
        keys = ("tiles", "tile_entries", "kept_tiles", "items", "ranked_rows", "rest_entries")
        return dict(zip(keys, (int(x) for x in a)))

    def barriers_gave_up(self) -> bool:
        """True if a barrier wait of the most recent product hit its time limit (synchronises)."""
        off = self.info()["gave_up_offset"]
        return bool(self.buf[off:off + 4].view(torch.int32).item() != 0)


def spmm_csr_prepare(rowptr, colidx, val, k: int, f: int, options: SpmmOptions = None) -> SpmmWorkspace:
    """One-time schedule for C = A*B with A = (rowptr, colidx, val), B of k rows and width f.
    `options` defaults to options_from_env() (all zero unless SAGNN_SWEEP* variables are set)."""
    rowptr = _dev(rowptr, torch.int32, "rowptr")
    colidx = _dev(colidx, torch.int32, "colidx")
    val = _dev(val, torch.float32, "val")
    m, nnz = rowptr.numel() - 1, colidx.numel()
    L = lib()
    wsb = ctypes.c_size_t(0)
    opt = options if options is not None else options_from_env()
    _check(L.spmm_csr_workspace_bytes_opt(m, k, nnz, f, ctypes.byref(opt), ctypes.byref(wsb)),
           "spmm_csr_workspace_bytes_opt")
    buf = _ws(wsb.value, rowptr.device)
    _check(L.spmm_csr_prepare_opt(_ptr(rowptr), _ptr(colidx), _ptr(val), m, k, nnz, f, _ptr(buf),
                                  buf.numel(), ctypes.byref(opt), _stream()), "spmm_csr_prepare_opt")
    return SpmmWorkspace(buf, m, nnz, f, None, int(k))


def spmm_csr_prepare_tuned(rowptr, colidx, val, B, C=None, options: SpmmOptions = None) -> SpmmWorkspace:
    """spmm_csr_prepare with a measured choice between a few plan variants, timed on B (k x f).
    C (m x f) is overwritten with the product; allocated here when not given."""
    rowptr = _dev(rowptr, torch.int32, "rowptr")
    colidx = _dev(colidx, torch.int32, "colidx")
    val = _dev(val, torch.float32, "val")
    B = _dev(B, torch.float32, "B")
    m, nnz = rowptr.numel() - 1, colidx.numel()
    k, f = B.shape
    if C is None:
        C = torch.empty((m, f), dtype=torch.float32, device=B.device)
    _dev(C, torch.float32, "C")
    L = lib()
    wsb = ctypes.c_size_t(0)
    opt = options if options is not None else options_from_env()
    _check(L.spmm_csr_workspace_bytes_opt(m, k, nnz, f, ctypes.byref(opt), ctypes.byref(wsb)),
           "spmm_csr_workspace_bytes_opt")
    buf = _ws(wsb.value, rowptr.device)
    choice = np.zeros(4, dtype=np.int32)
    _check(L.spmm_csr_prepare_tuned(_ptr(rowptr), _ptr(colidx), _ptr(val), m, k, nnz, f, _ptr(buf),
                                    buf.numel(), _ptr(B), B.stride(0), _ptr(C), C.stride(0),
                                    choice.ctypes.data_as(ctypes.c_void_p), ctypes.byref(opt), _stream()),
           "spmm_csr_prepare_tuned")
    return SpmmWorkspace(buf, m, nnz, f, {"piece": int(choice[0]), "min_long": int(choice[1]),
                                         "best_us": int(choice[2]), "variant": int(choice[3])}, int(k))


def spmm_csr_tallskinny(rowptr, colidx, val, B, C=None, accumulate=False, ws: SpmmWorkspace = None):
    """C (+)= A * B (Alg. 1/2 local SpMM)."""
    rowptr = _dev(rowptr, torch.int32, "rowptr")
    colidx = _dev(colidx, torch.int32, "colidx")
    val = _dev(val, torch.float32, "val")
    B = _mat(B, "B")
    m, nnz = rowptr.numel() - 1, colidx.numel()
    k, f = B.shape
    if C is None:
        if accumulate:
            raise ValueError("accumulate needs C")
        C = torch.empty((m, f), dtype=torch.float32, device=B.device)
    _mat(C, "C")
    if ws is not None and (ws.m != m or ws.nnz != nnz or ws.f < f or k < ws.k):
        raise ValueError("workspace was prepared for another matrix or a taller operand")
    rc = lib().spmm_csr_tallskinny(_ptr(rowptr), _ptr(colidx), _ptr(val), m, k, nnz, _ptr(B),
                                   _ld(B), f, _ptr(C), _ld(C), int(accumulate),
                                   _ptr(ws.buf) if ws else None, ws.buf.numel() if ws else 0,
                                   _stream())
    _check(rc, "spmm_csr_tallskinny")
    return C


def dense_gemm_act(X, W, transW=False, prec=GEMM_FP32, act=ACT_IDENTITY, mask=None, want_z=True,
                   want_act=False, out=None):
    X = _mat(X, "X")
    W = _mat(W, "W")
    m, kdim = X.shape
    nout = W.shape[0] if transW else W.shape[1]
    if out is not None:
        Z, A = out
    else:
        Z = torch.empty((m, nout), dtype=torch.float32, device=X.device) if want_z else None
        A = torch.empty((m, nout), dtype=torch.float32, device=X.device) if want_act else None
    rc = lib().dense_gemm_act(_ptr(X), _ld(X), _ptr(W), _ld(W), int(transW), m, kdim, nout,
                              prec, act, _ptr(mask), _ld(mask) if mask is not None else 0,
                              _ptr(Z), nout, _ptr(A), nout, _stream())
    _check(rc, "dense_gemm_act")
    return Z, A


def gcn_layer_fwd(rowptr, colidx, val, H, W, act=ACT_RELU, prec=GEMM_FP32, ws: SpmmWorkspace = None,
                  want_z=True, want_h=True, out=None, want_t=True, fused=False):
    """T = A H, Z = T W, Hout = sigma(Z).  Returns (T, Z, Hout).  want_t=False: T is not stored
    (returned as None) and the layer runs as one fused kernel; fused=True calls that kernel
    directly and still returns T."""
    rowptr = _dev(rowptr, torch.int32, "rowptr")
    colidx = _dev(colidx, torch.int32, "colidx")
    val = _dev(val, torch.float32, "val")
    H = _mat(H, "H")
    W = _dev(W, torch.float32, "W")
    m, nnz = rowptr.numel() - 1, colidx.numel()
    k, f_in = H.shape
    f_out = W.shape[1]
    if out is None:
        T = torch.empty((m, f_in), dtype=torch.float32, device=H.device) if want_t else None
        Z = torch.empty((m, f_out), dtype=torch.float32, device=H.device) if want_z else None
        Ho = torch.empty((m, f_out), dtype=torch.float32, device=H.device) if want_h else None
    else:
        T, Z, Ho = out
    if fused:
        rc = lib().gcn_layer_fwd_fused(_ptr(rowptr), _ptr(colidx), _ptr(val), m, k, nnz, _ptr(H), _ld(H),
                                       f_in, _ptr(W), f_out, act, prec, _ptr(T), _ptr(Z), _ptr(Ho), _stream())
        _check(rc, "gcn_layer_fwd_fused")
        return T, Z, Ho
    rc = lib().gcn_layer_fwd(_ptr(rowptr), _ptr(colidx), _ptr(val), m, k, nnz, _ptr(H), _ld(H),
                             f_in, _ptr(W), f_out, act, prec, _ptr(T), _ptr(Z), _ptr(Ho),
                             _ptr(ws.buf) if ws else None, ws.buf.numel() if ws else 0, _stream())
    _check(rc, "gcn_layer_fwd")
    return T, Z, Ho


def gcn_layer_fwd_form(ws: SpmmWorkspace, f_in: int, f_out: int, prec=GEMM_FP32) -> int:
    """Which form gcn_layer_fwd(want_t=False) takes: 2 sweep with the dense transform as epilogue,
    1 row-range kernel, 0 unsupported shape."""
    form = ctypes.c_int32(0)
    _check(lib().gcn_layer_fwd_form(_ptr(ws.buf) if ws else None, f_in, f_out, prec, ctypes.byref(form)),
           "gcn_layer_fwd_form")
    return form.value


def gcn_layer_bwd(rowptr, colidx, val, G, W, Zprev, Hprev, prec=GEMM_FP32, ws: SpmmWorkspace = None,
                  want_gprev=True, want_y=True):
    """S = A G, Gprev = (S W^T) .* [Zprev > 0], Y = Hprev^T S.  Returns (S, Gprev, Y)."""
    rowptr = _dev(rowptr, torch.int32, "rowptr")
    colidx = _dev(colidx, torch.int32, "colidx")
    val = _dev(val, torch.float32, "val")
    G = _dev(G, torch.float32, "G")
    W = _dev(W, torch.float32, "W")
    m, nnz = rowptr.numel() - 1, colidx.numel()
    f_in, f_out = W.shape
    dev = G.device
    S = torch.empty((m, f_out), dtype=torch.float32, device=dev)
    Gp = torch.empty((m, f_in), dtype=torch.float32, device=dev) if want_gprev else None
    Y = torch.empty((f_in, f_out), dtype=torch.float32, device=dev) if want_y else None
    yws = None
    if want_y:
        b = ctypes.c_size_t(0)
        _check(lib().gcn_bwd_workspace_bytes(m, f_in, f_out, ctypes.byref(b)), "gcn_bwd_workspace_bytes")
        yws = _ws(b.value, dev)
    rc = lib().gcn_layer_bwd(_ptr(rowptr), _ptr(colidx), _ptr(val), m, nnz, _ptr(G), f_out, _ptr(W),
                             f_in, _ptr(Zprev), _ptr(Hprev), prec, _ptr(S), _ptr(Gp), _ptr(Y),
                             _ptr(ws.buf) if ws else None, ws.buf.numel() if ws else 0,
                             _ptr(yws), yws.numel() if yws is not None else 0, _stream())
    _check(rc, "gcn_layer_bwd")
    return S, Gp, Y


@dataclass
class ColBlocks:
    """Result of spmm_split_colblocks: nb CSR matrices sharing three buffers."""
    rowptr_blk: torch.Tensor      # int32 [nb, m+1]
    colidx_blk: torch.Tensor      # int32 [nnz]
    val_blk: torch.Tensor         # float32 [nnz]
    nnz_off: np.ndarray           # int64 [nb+1] (host)

    def block(self, q: int):
        a, b = int(self.nnz_off[q]), int(self.nnz_off[q + 1])
        return self.rowptr_blk[q], self.colidx_blk[a:b], self.val_blk[a:b]


def spmm_split_colblocks(rowptr, colidx, val, bounds) -> ColBlocks:
    """Split a CSR row block into one CSR per column range (Sec. 4.2; the A_iq of Alg. 2)."""
    rowptr = _dev(rowptr, torch.int32, "rowptr")
    colidx = _dev(colidx, torch.int32, "colidx")
    val = _dev(val, torch.float32, "val")
    m, nnz = rowptr.numel() - 1, colidx.numel()
    bounds = np.ascontiguousarray(bounds, dtype=np.int64)
    nb = bounds.size - 1
    dev = rowptr.device
    L = lib()
    wsb = ctypes.c_size_t(0)
    _check(L.spmm_split_workspace_bytes(m, nb, ctypes.byref(wsb)), "spmm_split_workspace_bytes")
    ws = _ws(wsb.value, dev)
    rp = torch.empty((nb, m + 1), dtype=torch.int32, device=dev)
    ci = torch.empty(max(nnz, 1), dtype=torch.int32, device=dev)
    va = torch.empty(max(nnz, 1), dtype=torch.float32, device=dev)
    off = np.zeros(nb + 1, dtype=np.int64)
    rc = L.spmm_split_colblocks(_ptr(rowptr), _ptr(colidx), _ptr(val), m, nnz,
                                bounds.ctypes.data_as(ctypes.c_void_p), nb, _ptr(rp), _ptr(ci), _ptr(va),
                                off.ctypes.data_as(ctypes.c_void_p), _ptr(ws), ws.numel(), _stream())
    _check(rc, "spmm_split_colblocks")
    return ColBlocks(rp, ci[:nnz], va[:nnz], off)


def spmm_stage_loop(stages, m: int, H, T0, T1, Z, accumulate_first=False, pack_stream=None):
    """Stage loop of Alg. 2 on one rank.  `stages` is a list of dicts with keys rowptr, colidx,
    val, rows and optionally ws (SpmmWorkspace).  Products run on the current stream, packs on
    `pack_stream` (a torch.cuda.Stream; None = the current stream)."""
    H = _dev(H, torch.float32, "H")
    Z = _dev(Z, torch.float32, "Z")
    T0 = _dev(T0, torch.float32, "T0")
    T1 = _dev(T1, torch.float32, "T1")
    n, f = H.shape
    arr = (_Stage * max(len(stages), 1))()
    for k, st in enumerate(stages):
        rp = _dev(st["rowptr"], torch.int32, "stage rowptr")
        ci = _dev(st["colidx"], torch.int32, "stage colidx")
        va = _dev(st["val"], torch.float32, "stage val")
        rows = _dev(st["rows"], torch.int32, "stage rows")
        if rp.numel() != m + 1:
            raise ValueError("stage rowptr must have m+1 entries")
        ws = st.get("ws")
        arr[k] = _Stage(rp.data_ptr(), ci.data_ptr() if ci.numel() else None,
                        va.data_ptr() if va.numel() else None, ci.numel(),
                        rows.data_ptr() if rows.numel() else None, rows.numel(),
                        ws.buf.data_ptr() if ws else None, ws.buf.numel() if ws else 0)
    cap = min(T0.shape[0], T1.shape[0])
    if T0.shape[1] != f or T1.shape[1] != f:
        raise ValueError("packed buffers must have H's width")
    ps = _stream() if pack_stream is None else ctypes.c_void_p(pack_stream.cuda_stream)
    rc = lib().spmm_stage_loop(ctypes.cast(arr, ctypes.c_void_p), len(stages), m, _ptr(H), n,
                               H.stride(0), f, _ptr(T0), _ptr(T1), cap, _ptr(Z), Z.stride(0),
                               int(accumulate_first), _stream(), ps)
    _check(rc, "spmm_stage_loop")
    return Z


def spmm_volume_stats(counts, f: int, elem_bytes: int = 4) -> dict:
    """Volume statistics of one SpMM from the P x P matrix of |NnzCols(i,q)| (host arithmetic)."""
    c = np.ascontiguousarray(counts, dtype=np.int64)
    if c.ndim != 2 or c.shape[0] != c.shape[1]:
        raise ValueError("counts must be P x P")
    out = np.zeros(8, dtype=np.float64)
    _check(lib().spmm_volume_stats(c.ctypes.data_as(ctypes.c_void_p), c.shape[0], f, elem_bytes,
                                   out.ctypes.data_as(ctypes.c_void_p)), "spmm_volume_stats")
    keys = ("total_bytes", "avg_bytes", "max_recv_bytes", "recv_imbalance_pct", "max_send_bytes",
            "send_imbalance_pct", "cut_rows", "cut_bytes")
    return dict(zip(keys, (float(x) for x in out)))


def spmm_csr_transpose(rowptr, colidx, val, n: int):
    """CSR of A^T for A = (rowptr, colidx, val) with n columns.  Returns (rowptr_t, colidx_t, val_t)."""
    rowptr = _dev(rowptr, torch.int32, "rowptr")
    colidx = _dev(colidx, torch.int32, "colidx")
    val = _dev(val, torch.float32, "val")
    m, nnz = rowptr.numel() - 1, colidx.numel()
    dev = rowptr.device
    L = lib()
    wsb = ctypes.c_size_t(0)
    _check(L.spmm_transpose_workspace_bytes(nnz, ctypes.byref(wsb)), "spmm_transpose_workspace_bytes")
    ws = _ws(wsb.value, dev)
    rpt = torch.empty(n + 1, dtype=torch.int32, device=dev)
    cit = torch.empty(max(nnz, 1), dtype=torch.int32, device=dev)
    vat = torch.empty(max(nnz, 1), dtype=torch.float32, device=dev)
    _check(L.spmm_csr_transpose(_ptr(rowptr), _ptr(colidx), _ptr(val), m, n, nnz, _ptr(rpt), _ptr(cit),
                                _ptr(vat), _ptr(ws), ws.numel(), _stream()), "spmm_csr_transpose")
    return rpt, cit[:nnz], vat[:nnz]


def _permute_ws(n: int, nnz: int, device):
    wsb = ctypes.c_size_t(0)
    _check(lib().spmm_permute_workspace_bytes(n, nnz, ctypes.byref(wsb)), "spmm_permute_workspace_bytes")
    return _ws(wsb.value, device)


def spmm_perm_from_labels(labels, n_parts: int):
    """Vertex order by part label (Sec. 5 / 6.1 renumbering).  Returns (perm, inv, part_off): perm[i] =
    old id of new vertex i, inv[v] = new id of old vertex v, part_off (host, n_parts+1)."""
    labels = _dev(labels, torch.int32, "labels")
    n = labels.numel()
    dev = labels.device
    ws = _permute_ws(n, n, dev)
    perm = torch.empty(max(n, 1), dtype=torch.int32, device=dev)
    inv = torch.empty(max(n, 1), dtype=torch.int32, device=dev)
    off = np.zeros(n_parts + 1, dtype=np.int64)
    _check(lib().spmm_perm_from_labels(_ptr(labels), n, n_parts, _ptr(perm), _ptr(inv),
                                       off.ctypes.data_as(ctypes.c_void_p), _ptr(ws), ws.numel(), _stream()),
           "spmm_perm_from_labels")
    return perm[:n], inv[:n], off


def spmm_csr_permute_symmetric(rowptr, colidx, val, inv):
    """B = P A P^T with B[inv[r], inv[c]] = A[r, c].  Returns (rowptr_p, colidx_p, val_p)."""
    rowptr = _dev(rowptr, torch.int32, "rowptr")
    colidx = _dev(colidx, torch.int32, "colidx")
    val = _dev(val, torch.float32, "val")
    inv = _dev(inv, torch.int32, "inv")
    n, nnz = rowptr.numel() - 1, colidx.numel()
    if inv.numel() != n:
        raise ValueError("inv must have one entry per row")
    dev = rowptr.device
    ws = _permute_ws(n, nnz, dev)
    rpp = torch.empty(n + 1, dtype=torch.int32, device=dev)
    cip = torch.empty(max(nnz, 1), dtype=torch.int32, device=dev)
    vap = torch.empty(max(nnz, 1), dtype=torch.float32, device=dev)
    _check(lib().spmm_csr_permute_symmetric(_ptr(rowptr), _ptr(colidx), _ptr(val), n, nnz, _ptr(inv), _ptr(rpp),
                                            _ptr(cip), _ptr(vap), _ptr(ws), ws.numel(), _stream()),
           "spmm_csr_permute_symmetric")
    return rpp, cip[:nnz], vap[:nnz]
