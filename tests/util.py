"""Shared helpers of the GPU parity tests."""
import numpy as np
import torch


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def csr_dev(g):
    return dev(g.rowptr), dev(g.colidx), dev(g.val)


def assert_close(got, ref, scale, rtol, what=""):
    """|got - ref| <= rtol * scale + 1e-30 element-wise, where `scale` is the sum of the absolute
    values of the terms of each output (forward-error form of the tolerance)."""
    got = got.detach().cpu().numpy() if isinstance(got, torch.Tensor) else np.asarray(got)
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    bound = rtol * scale + 1e-30
    bad = err > bound
    if bad.any():
        i = np.unravel_index(np.argmax(err / bound), err.shape)
        raise AssertionError(f"{what}: {bad.sum()} of {bad.size} elements out of tolerance; worst at {i}: "
                             f"got {got[i]!r} ref {ref[i]!r} err {err[i]:.3e} bound {bound[i]:.3e}")
    return float((err / np.maximum(bound, 1e-300)).max())


def sample_rows_csr(g, rows):
    """Sub-CSR holding only `rows` of g (same column space)."""
    rows = np.asarray(rows, dtype=np.int64)
    cnt = (g.rowptr[rows + 1] - g.rowptr[rows]).astype(np.int64)
    rp = np.concatenate([[0], np.cumsum(cnt)]).astype(np.int32)
    idx = np.concatenate([np.arange(g.rowptr[r], g.rowptr[r + 1], dtype=np.int64) for r in rows]) \
        if rows.size else np.empty(0, np.int64)
    return rp, g.colidx[idx], g.val[idx]
