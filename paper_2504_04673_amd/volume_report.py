"""Sparsity-aware versus sparsity-oblivious data volume and single-GPU cost on one harness.

For a whole (symmetric) graph cut into P row blocks (Sec. 4.1, 1D block-row distribution) this
plans every row block on the GPU, forms the P x P matrix of |NnzCols(i,q)|, and prints the
statistics of Table 2 (average and maximum data per process, load imbalance) and cut_P(G) for
both algorithms; it then times, for row block 0, what one GPU does per SpMM in each algorithm
(pack the rows it needs / all rows, local product).  Every step runs through the C ABI.

    python -m paper_2504_04673_amd.volume_report --workload cfg5 --order random --P 16

Inputs are the seeded synthetic graphs of `workloads.py`; no dataset of the paper is used.
"""
from __future__ import annotations

import argparse
import json

import numpy as np
import torch

from . import binding as B
from . import synth, workloads


def _time_ms(fn, reps=5):
    fn()
    torch.cuda.synchronize()
    best = 1e30
    for _ in range(reps):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        torch.cuda.synchronize()
        best = min(best, a.elapsed_time(b))
    return best


def report(g, H, P, f, label):
    dev = torch.device("cuda:0")
    off = synth.block_offsets(g.n, P)
    counts = np.zeros((P, P), dtype=np.int64)
    rowptr = torch.from_numpy(g.rowptr).to(dev)
    colidx = torch.from_numpy(g.colidx).to(dev)
    for i in range(P):
        r0, r1 = int(off[i]), int(off[i + 1])
        a, b = int(g.rowptr[r0]), int(g.rowptr[r1])
        rp = (rowptr[r0:r1 + 1] - a).contiguous()
        plan = B.spmm_plan_needed_rows(rp, colidx[a:b].contiguous(), g.n, off, want_compact=False)
        counts[i] = np.diff(plan.blk_off)
    obl = np.tile(np.diff(off), (P, 1))
    st_a, st_o = B.spmm_volume_stats(counts, f), B.spmm_volume_stats(obl, f)

    # one GPU's work per SpMM for row block 0, both algorithms
    r1 = int(off[1])
    b = int(g.rowptr[r1])
    rp = rowptr[:r1 + 1].contiguous()
    ci = colidx[:b].contiguous()
    va = torch.from_numpy(g.val[:b]).to(dev)
    Hd = torch.from_numpy(H).to(dev)
    out = {"label": label, "P": P, "n": int(g.n), "nnz": int(g.nnz), "f": f,
           "aware": st_a, "oblivious": st_o, "block0": {}}
    for name, oblivious in (("aware", False), ("oblivious", True)):
        plan = B.spmm_plan_needed_rows(rp, ci, g.n, off, oblivious=oblivious)
        T = torch.empty((plan.N, f), dtype=torch.float32, device=dev)
        ws = B.spmm_csr_prepare(rp, plan.colidx_compact, va, plan.N, f)
        Z = torch.empty((r1, f), dtype=torch.float32, device=dev)
        t_pack = _time_ms(lambda: B.spmm_pack_rows(Hd, plan.needed, out=T))
        t_spmm = _time_ms(lambda: B.spmm_csr_tallskinny(rp, plan.colidx_compact, va, T, C=Z, ws=ws))
        out["block0"][name] = {"rows_packed": plan.N, "pack_ms": round(t_pack, 4),
                               "spmm_ms": round(t_spmm, 4),
                               "offdiag_rows": int(plan.N - (plan.blk_off[1] - plan.blk_off[0]))}
        del T, ws, Z
    return out


def to_markdown(r):
    mb = 1e6
    lines = [f"### {r['label']}: n={r['n']:,} nnz={r['nnz']:,} P={r['P']} f={r['f']} (fp32)", "",
             "| algorithm | average MB | max MB (recv) | load imbalance % | max MB (send) | cut_P rows | total MB |",
             "|---|---|---|---|---|---|---|"]
    for name in ("aware", "oblivious"):
        s = r[name]
        lines.append(f"| sparsity-{name} | {s['avg_bytes'] / mb:.1f} | {s['max_recv_bytes'] / mb:.1f} | "
                     f"{s['recv_imbalance_pct']:.1f} | {s['max_send_bytes'] / mb:.1f} | {int(s['cut_rows']):,} | "
                     f"{s['total_bytes'] / mb:.1f} |")
    lines += ["", "| row block 0 on one MI355X | rows packed | off-diagonal rows | pack ms | SpMM ms |", "|---|---|---|---|---|"]
    for name in ("aware", "oblivious"):
        b = r["block0"][name]
        lines.append(f"| sparsity-{name} | {b['rows_packed']:,} | {b['offdiag_rows']:,} | {b['pack_ms']:.3f} | {b['spmm_ms']:.3f} |")
    return "\n".join(lines)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="cfg5", choices=["cfg1", "cfg2", "cfg3", "cfg5"])
    ap.add_argument("--order", default="community", choices=["community", "random"], help="cfg5 only")
    ap.add_argument("--P", type=int, default=0, help="row blocks (default: the configuration's)")
    ap.add_argument("--f", type=int, default=0)
    ap.add_argument("--scale", type=float, default=1.0)
    ap.add_argument("--json", action="store_true")
    a = ap.parse_args()
    if a.workload == "cfg1":
        wl = workloads.cfg1()
    elif a.workload == "cfg5":
        wl = workloads.cfg5(scale=a.scale, order=a.order, **({"f": a.f} if a.f else {}))
    else:
        wl = getattr(workloads, a.workload)(scale=a.scale, **({"f": a.f} if a.f else {}))
    P = a.P or int(wl.extra.get("P", 16))
    label = wl.name + (f" ({a.order} order)" if a.workload == "cfg5" else "")
    r = report(wl.g, wl.H, P, wl.f, label)
    print(json.dumps(r) if a.json else to_markdown(r), flush=True)


if __name__ == "__main__":
    main()
