"""The planning entry point that allocates nothing (fixed per-GPU scratch array inside the
library) against the entry point with a caller workspace: same outputs bit for bit, on two
calls in a row, the second on a smaller input (stale scratch contents must not leak)."""
import numpy as np
import pytest
import torch

import paper_2504_04673_amd as sagnn

pytestmark = pytest.mark.gpu


def _random_block(m, n, avg, nb, seed):
    rng = np.random.default_rng(seed)
    deg = rng.poisson(avg, size=m)
    rowptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)
    colidx = (rng.random(int(rowptr[-1])) ** 2 * n).astype(np.int32)     # skewed, unsorted, repeated
    cuts = np.sort(rng.integers(0, n + 1, size=nb - 1))
    return rowptr, colidx, np.array([0, *cuts, n], dtype=np.int64)


def _both(rowptr, colidx, n, colblk, validate, multipass=None):
    rp = torch.from_numpy(rowptr).cuda()
    ci = torch.from_numpy(colidx).cuda()
    ref = sagnn.spmm_plan_needed_rows(rp, ci, n, colblk, validate=validate, multipass=multipass)
    torch.cuda.synchronize()
    needed = torch.full((max(min(n, colidx.size), 1),), -7, dtype=torch.int32, device="cuda")
    compact = torch.full((max(colidx.size, 1),), -7, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    got = sagnn.spmm_plan_needed_rows_noalloc(rp, ci, n, colblk, needed, compact, validate=validate,
                                              multipass=multipass)
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before      # torch's allocator untouched
    assert np.array_equal(got.blk_off, ref.blk_off)
    assert torch.equal(got.needed, ref.needed)
    assert torch.equal(got.colidx_compact, ref.colidx_compact)
    return got


def test_noalloc_plan_matches_workspace_plan_twice_in_a_row():
    # first call: 3 M columns (most of the fixed array); second: a much smaller problem
    big = _random_block(20_000, 3_000_001, 40, 9, 1)
    small = _random_block(700, 4_097, 3, 4, 2)
    g1 = _both(*big[:2], 3_000_001, big[2], validate=True)
    # (the small one through the general path, which reuses the scratch arrays the big call filled, and
    # through the one-launch path small blocks take by default)
    g2 = _both(*small[:2], 4_097, small[2], validate=False, multipass=True)
    g3 = _both(*small[:2], 4_097, small[2], validate=False)
    assert g1.N > g2.N > 0 and g3.N == g2.N
    # and the big one again: the scratch left by the small call must not matter either
    _both(*big[:2], 3_000_001, big[2], validate=False)


def test_noalloc_plan_rejects_sizes_beyond_the_fixed_scratch():
    rp = torch.zeros(2, dtype=torch.int32, device="cuda")
    ci = torch.zeros(0, dtype=torch.int32, device="cuda")
    needed = torch.zeros(1, dtype=torch.int32, device="cuda")
    n = 5_000_001
    with pytest.raises(sagnn.SagnnError) as ei:
        sagnn.spmm_plan_needed_rows_noalloc(rp, ci, n, np.array([0, n]), needed)
    assert ei.value.code == -2
    with pytest.raises(sagnn.SagnnError) as ei:
        sagnn.spmm_plan_needed_rows_noalloc(rp, ci, 2000, np.concatenate([[0], np.full(1025, 2000)]), needed)
    assert ei.value.code == -2
    # the limit itself is accepted (empty matrix: N = 0)
    n = 5_000_000
    p = sagnn.spmm_plan_needed_rows_noalloc(rp, ci, n, np.array([0, n]), needed)
    assert p.N == 0
