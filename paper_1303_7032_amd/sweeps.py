"""Erasure and reinforcement sweeps on the GPU (Section VII-A, VII-B and VII-D of the paper).

For a network of C clusters x L neurons holding M uniformly random messages, and for each number of
erased clusters e, K probes are drawn from the stored messages, e of their symbols are erased, and
every (rule, gamma) of the sweep retrieves them through gbnn_retrieve_symbols.  Reported per cell:
  retrieval_rate   fraction of probes whose every cluster ends with exactly the source symbol
                   (the strict reading of "successfully retrieved": an ambiguous cluster is a miss)
  mean_passes      mean number of passes, capped probes counted at the cap
  capped           fraction of probes that reached max_iters without reproducing their input
  period2          (sum-of-sum only) fraction of probes that reached the cap while alternating
                   between two vectors (Section V-A): the results at caps T, T+1, T+2 satisfy
                   out(T) = out(T+2) != out(T+1)

Storing, retrieval and decoding run in the HIP kernels; this module only draws the inputs, compares
the returned symbols with the source messages and counts.  Scenario 1 is C=8, L=128, M=5000 with 3000
probes, Scenario 2 is C=16, L=512, M=50000 with 30000 probes.

    python -m paper_1303_7032_amd.sweeps --scenario 1
"""
from __future__ import annotations

import argparse
import json

import numpy as np
import torch

from . import binding as gb
from . import inputs

SCENARIOS = {
    1: dict(C=8, L=128, M=5000, K=3000, erasures=(1, 2, 3, 4, 5, 6, 7)),
    2: dict(C=16, L=512, M=50000, K=30000, erasures=(2, 4, 6, 8, 10, 12, 13, 14, 15)),
}
DEFAULT_CELLS = (("sum_of_sum", 0), ("sum_of_sum", 1), ("sum_of_sum", 2), ("sum_of_sum", 5), ("sum_of_max", 1), ("hybrid", 1))


def draw_probes(C: int, L: int, M: int, K: int, e: int, seed: int, msgs: np.ndarray):
    """K probes with e erased clusters each (-1), and the messages they were made from."""
    q, er = inputs.make_probe_plan(C, M, K, e, seed + 1 + e)
    probes = msgs[q].copy()
    probes[er] = -1
    return probes, msgs[q]


def erasure_sweep(C: int, L: int, M: int, K: int, erasures, cells=DEFAULT_CELLS, max_iters: int = 20,
                  seed: int = 0x13037032 + 11, detect_period2: bool = True):
    """Runs the sweep on the current CUDA device; returns a list of dicts, one per (e, rule, gamma)."""
    msgs = inputs.make_messages(C, L, M, seed)
    W = gb.new_network(C, L)
    gb.gbnn_store(W, C, L, torch.from_numpy(msgs).cuda())
    ws = gb.gbnn_prepare(W, C, L)
    rows = []
    for e in erasures:
        probes, truth = draw_probes(C, L, M, K, e, seed, msgs)
        pd = torch.from_numpy(probes).cuda()
        td = torch.from_numpy(truth).cuda()
        for rule, gamma in cells:
            bits, sym, it = gb.gbnn_retrieve_symbols(W, C, L, pd, rule, gamma, max_iters, workspace=ws)
            ok = (sym == td).all(dim=1)
            capped = it < 0
            row = {"C": C, "L": L, "M": M, "K": K, "erased": int(e), "rule": rule, "gamma": int(gamma),
                   "max_iters": int(max_iters), "retrieval_rate": float(ok.float().mean()),
                   "mean_passes": float(it.abs().float().mean()), "capped": float(capped.float().mean())}
            if rule == "sum_of_sum" and detect_period2:
                b1, _, _ = gb.gbnn_retrieve_symbols(W, C, L, pd, rule, gamma, max_iters + 1, workspace=ws,
                                                    want_symbols=False, want_iters=False)
                b2, _, _ = gb.gbnn_retrieve_symbols(W, C, L, pd, rule, gamma, max_iters + 2, workspace=ws,
                                                    want_symbols=False, want_iters=False)
                p2 = capped & (bits == b2).all(dim=1) & (bits != b1).any(dim=1)
                row["period2"] = float(p2.float().mean())
            rows.append(row)
    return rows


def format_table(rows) -> str:
    cells = []
    for r in rows:
        key = (r["rule"], r["gamma"])
        if key not in cells:
            cells.append(key)
    es = sorted({r["erased"] for r in rows})
    by = {(r["erased"], r["rule"], r["gamma"]): r for r in rows}
    head = "erased | " + " | ".join(f"{rule} g={g}" for rule, g in cells)
    lines = [head, "-" * len(head)]
    for e in es:
        lines.append(f"{e:6d} | " + " | ".join(
            f"{by[(e, rule, g)]['retrieval_rate']:.3f} ({by[(e, rule, g)]['mean_passes']:.1f}p)".ljust(len(f"{rule} g={g}"))
            for rule, g in cells))
    return "\n".join(lines)


def main() -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--scenario", type=int, choices=sorted(SCENARIOS), default=1)
    ap.add_argument("--probes", type=int, default=0, help="probes per cell (default: the scenario's)")
    ap.add_argument("--max-iters", type=int, default=20)
    ap.add_argument("--json", action="store_true", help="print one JSON object per cell instead of the table")
    args = ap.parse_args()
    sc = dict(SCENARIOS[args.scenario])
    if args.probes:
        sc["K"] = args.probes
    rows = erasure_sweep(sc["C"], sc["L"], sc["M"], sc["K"], sc["erasures"], max_iters=args.max_iters)
    if args.json:
        for r in rows:
            print(json.dumps(r))
    else:
        print(f"retrieval rate (mean passes), C={sc['C']} L={sc['L']} M={sc['M']} probes={sc['K']} cap={args.max_iters}")
        print(format_table(rows))
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
