"""Sparse W' against the packed W (Section IV-B, "Sparsification"): sizes and sum-of-max retrieval time.

For each network (C, L, M) and K probes with e erased clusters, messages at the boundary, cap 20:
  density        measured edge density of W between clusters
  packed_MiB     bytes of W plus its prepared table (what gbnn_retrieve_symbols reads)
  sparse_MiB     bytes of W'
  packed_us      gbnn_retrieve_symbols(sum_of_max), microseconds per call, and the kernel family it ran
  sparse_us      gbnn_retrieve_sparse, microseconds per call
and the two results are checked to be identical.

    python -m paper_1303_7032_amd.sparsity
"""
from __future__ import annotations

import argparse
import json

import torch

from . import binding as gb
from . import inputs

GRID = (
    # C, L, M, K, e
    (8, 256, 20000, 65536, 4),
    (8, 256, 1500, 65536, 4),
    (16, 512, 100000, 32768, 8),
    (16, 512, 15000, 32768, 8),
    (16, 512, 4000, 32768, 8),
    (8, 2048, 400000, 4096, 4),
    (8, 2048, 40000, 4096, 4),
    (4, 4096, 160000, 4096, 2),
)


def _events_us(fn, reps: int) -> float:
    fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) * 1e3 / reps


def compare(C: int, L: int, M: int, K: int, e: int, seed: int = 0x13037032 + 31, reps: int = 5):
    msgs = inputs.make_messages(C, L, M, seed)
    W = gb.new_network(C, L)
    gb.gbnn_store(W, C, L, torch.from_numpy(msgs).cuda())
    ws = gb.gbnn_prepare(W, C, L)
    nnz = gb.gbnn_sparse_count(W, C, L)
    Wp = gb.gbnn_sparsify(W, C, L)
    q, er = inputs.make_probe_plan(C, M, K, e, seed + 1)
    probes = msgs[q].copy()
    probes[er] = -1
    pd = torch.from_numpy(probes).cuda()
    nw = gb.gbnn_w_row_words(C, L)
    outs = [(torch.empty((K, nw), dtype=torch.int32, device="cuda"), torch.empty((K, C), dtype=torch.int32, device="cuda"),
             torch.empty(K, dtype=torch.int32, device="cuda")) for _ in range(2)]

    def packed():
        gb.gbnn_retrieve_symbols(W, C, L, pd, "sum_of_max", 1, 20, bits_out=outs[0][0], symbols_out=outs[0][1],
                                 iters_out=outs[0][2], workspace=ws)

    def sparse():
        gb.gbnn_retrieve_sparse(Wp, C, L, pd, 20, bits_out=outs[1][0], symbols_out=outs[1][1], iters_out=outs[1][2])

    packed_us = _events_us(packed, reps)
    sparse_us = _events_us(sparse, reps)
    same = all(torch.equal(x, y) for x, y in zip(outs[0], outs[1]))
    n = C * L
    return {"C": C, "L": L, "M": M, "K": K, "erased": e, "density": nnz / (n * (n - L)),
            "packed_MiB": (W.numel() * 4 + ws.numel()) / 2**20, "sparse_MiB": Wp.numel() / 2**20,
            "packed_us": packed_us, "packed_kernel": gb.gbnn_retrieve_path(C, L, "sum_of_max", None, None),
            "sparse_us": sparse_us, "mean_passes": float(outs[0][2].abs().float().mean()), "identical": same}


def main() -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--json", action="store_true")
    args = ap.parse_args()
    print("C x L, M | density | packed MiB | W' MiB | packed us (kernel) | W' us | passes | identical")
    for cfg in GRID:
        r = compare(*cfg)
        if args.json:
            print(json.dumps(r), flush=True)
        else:
            print(f"{r['C']}x{r['L']}, M={r['M']}, K={r['K']}, e={r['erased']} | {r['density']:.4f} | {r['packed_MiB']:.1f} | "
                  f"{r['sparse_MiB']:.1f} | {r['packed_us']:.0f} ({r['packed_kernel']}) | {r['sparse_us']:.0f} | "
                  f"{r['mean_passes']:.2f} | {r['identical']}", flush=True)
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
