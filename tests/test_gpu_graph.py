"""The per-step entry points only enqueue kernels (no host synchronisation, no memset, no
allocation), so a caller can record them into a HIP graph.  Each case captures a sequence once,
replays it several times with new inputs and eager work in between, and compares every replay
bit for bit with the eager result of the same calls."""
import numpy as np
import pytest
import torch

import paper_2504_04673_amd as sagnn
from paper_2504_04673_amd import synth
from tests.test_gpu_parity import random_csr
from tests.util import dev

pytestmark = pytest.mark.gpu


def capture(fn):
    """Warm up on a side stream, then record fn into a graph (torch supplies the capture calls)."""
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        fn()
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=s):
            fn()
    torch.cuda.synchronize()
    return g


def replay_and_compare(g, fn, refresh, outputs, reps=3):
    for rep in range(reps):
        refresh(rep)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = [o.clone() for o in outputs]
        for o in outputs:
            o.fill_(float("nan"))                    # eager work between the replays
        fn()
        torch.cuda.synchronize()
        for a, b in zip(got, outputs):
            assert torch.equal(a, b), f"replay {rep} differs from the eager run"


def problem(seed, m=6000, n=50_000):
    rng = np.random.default_rng(seed)
    rowptr, colidx, val = random_csr(m, n, 25, rng, empty_frac=0.05, hubs=[(0, 9000), (77, 3000)])
    return m, n, dev(rowptr), dev(colidx), dev(val)


@pytest.mark.parametrize("sweep", ["0", "1"])
def test_graph_of_pack_spmm_gemm(sweep, monkeypatch):
    monkeypatch.setenv("SAGNN_SWEEP", sweep)
    m, n, rp, ci, v = problem(3)
    f, fo = 128, 64
    plan = sagnn.spmm_plan_needed_rows(rp, ci, n, np.array([0, n // 3, n]))
    ws = sagnn.spmm_csr_prepare(rp, plan.colidx_compact, v, plan.N, f)
    assert ws.info()["mode"] == int(sweep)
    H = torch.empty((n, f), device="cuda")
    W = dev(synth.normal((f, fo), 5, synth.STREAM_W))
    T = torch.empty((plan.N, f), device="cuda")
    Z = torch.empty((m, f), device="cuda")
    Zo, Ho = torch.empty((m, fo), device="cuda"), torch.empty((m, fo), device="cuda")

    def step():
        sagnn.spmm_pack_rows(H, plan.needed, out=T)
        sagnn.spmm_csr_tallskinny(rp, plan.colidx_compact, v, T, C=Z, ws=ws)
        sagnn.dense_gemm_act(Z, W, act=sagnn.ACT_RELU, want_z=True, want_act=True, out=(Zo, Ho))

    def refresh(rep):
        H.copy_(dev(synth.normal((n, f), 20 + rep, synth.STREAM_H)))

    refresh(-1)
    g = capture(step)
    replay_and_compare(g, step, refresh, [T, Z, Zo, Ho])


def test_graph_of_layer_forward_and_backward():
    m, n, rp, ci, v = problem(4, m=5000, n=5000)
    f = 64
    ws = sagnn.spmm_csr_prepare(rp, ci, v, n, f)
    H = torch.empty((n, f), device="cuda")
    G = torch.empty((m, f), device="cuda")
    W = dev(synth.normal((f, f), 6, synth.STREAM_W))
    out = {}

    def step():
        T, Z, Ho = sagnn.gcn_layer_fwd(rp, ci, v, H, W, act=sagnn.ACT_RELU, ws=ws)
        S, Gp, Y = sagnn.gcn_layer_bwd(rp, ci, v, G, W, Z, H, ws=ws)
        out["t"] = (T, Z, Ho, S, Gp, Y)

    def refresh(rep):
        H.copy_(dev(synth.normal((n, f), 30 + rep, synth.STREAM_H)))
        G.copy_(dev(synth.normal((m, f), 40 + rep, synth.STREAM_G)))

    refresh(-1)
    g = capture(step)                                # the binding's outputs live in the graph's pool
    captured = out["t"]
    for rep in range(3):
        refresh(rep)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = [o.clone() for o in captured]
        step()
        torch.cuda.synchronize()
        for a, b in zip(got, out["t"]):
            assert torch.equal(a, b), f"replay {rep} differs from the eager run"


@pytest.mark.parametrize("two_streams", [False, True])
def test_graph_of_stage_loop(two_streams):
    m, n, rp, ci, v = problem(5, m=4000, n=40_000)
    f = 128
    bounds = np.array([0, 9000, 9000, 25_000, n])
    cb = sagnn.spmm_split_colblocks(rp, ci, v, bounds)
    stages, cap = [], 0
    for q in range(bounds.size - 1):
        rq, cq, vq = cb.block(q)
        plan = sagnn.spmm_plan_needed_rows(rq, cq, n, np.array([0, n]))
        wsq = sagnn.spmm_csr_prepare(rq, plan.colidx_compact, vq, plan.N, f) if cq.numel() else None
        stages.append({"rowptr": rq, "colidx": plan.colidx_compact, "val": vq, "rows": plan.needed, "ws": wsq})
        cap = max(cap, plan.N)
    H = torch.empty((n, f), device="cuda")
    T0, T1 = torch.empty((cap, f), device="cuda"), torch.empty((cap, f), device="cuda")
    Z = torch.empty((m, f), device="cuda")
    side = torch.cuda.Stream() if two_streams else None

    def step():
        sagnn.spmm_stage_loop(stages, m, H, T0, T1, Z, pack_stream=side)

    def refresh(rep):
        H.copy_(dev(synth.normal((n, f), 50 + rep, synth.STREAM_H)))

    refresh(-1)
    g = capture(step)
    replay_and_compare(g, step, refresh, [Z])
