"""One-after-another ("serial", Section VII-C) decoding on the GPU, timed beside batch decoding.

For a network of C x L holding M random messages and probes with e erased clusters, through
gbnn_retrieve_symbols, per rule:
  call_us        one probe per call, calls issued back to back on one stream (device time per call)
  call_sync_us   one probe per call, the host waiting for each result (wall time per call)
  graph_us       the same calls captured 64 to a HIP graph, per call of a replay
  turn_us        store one message (gbnn_store_update) then retrieve one probe, captured 32 turns to a
                 graph, per turn of a replay
  batch_us       per probe of one call with K = 65536 probes
All of it runs in the library's kernels; this module only draws inputs and reads the clocks.

    python -m paper_1303_7032_amd.serial --C 8 --L 256 --M 20000 --erased 4
"""
from __future__ import annotations

import argparse
import json
import time

import torch

from . import binding as gb
from . import inputs

RULES = ("sum_of_max", "hybrid", "sum_of_sum")


def _events_us(fn, reps: int) -> float:
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) * 1e3 / reps


def measure(C: int, L: int, M: int, e: int, max_iters: int = 20, seed: int = 0x13037032 + 29, per_graph: int = 64,
            batch: int = 65536):
    """Returns one dict per rule with the figures of the module docstring (microseconds)."""
    nw = gb.gbnn_w_row_words(C, L)
    msgs = inputs.make_messages(C, L, M + 4096, seed)
    W = gb.new_network(C, L)
    gb.gbnn_store(W, C, L, torch.from_numpy(msgs[:M].copy()).cuda())
    ws = gb.gbnn_prepare(W, C, L)
    q, er = inputs.make_probe_plan(C, M, batch, e, seed + 1)
    probes = msgs[q].copy()
    probes[er] = -1
    pd = torch.from_numpy(probes).cuda()
    extra = torch.from_numpy(msgs[M:].copy()).cuda()
    bits = torch.empty((batch, nw), dtype=torch.int32, device="cuda")
    sym = torch.empty((batch, C), dtype=torch.int32, device="cuda")
    it = torch.empty(batch, dtype=torch.int32, device="cuda")
    side = torch.cuda.Stream()
    rows = []
    for rule in RULES:
        def one(k, rule=rule):
            gb.gbnn_retrieve_symbols(W, C, L, pd[k:k + 1], rule, 1, max_iters, bits_out=bits[k:k + 1],
                                     symbols_out=sym[k:k + 1], iters_out=it[k:k + 1], workspace=ws)

        for k in range(8):
            one(k)
        torch.cuda.synchronize()
        counter = iter(range(1 << 30))
        call_us = _events_us(lambda: one(next(counter) % 4096), 512)
        t0 = time.perf_counter()
        for k in range(256):
            one(k)
            torch.cuda.synchronize()
        call_sync_us = (time.perf_counter() - t0) / 256 * 1e6

        with torch.cuda.stream(side):
            one(0)
        side.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            for k in range(per_graph):
                one(k)
        g.replay()
        torch.cuda.synchronize()
        graph_us = _events_us(g.replay, 20) / per_graph

        # store one message, retrieve one probe, in turn (a copy of the network: the turns change it)
        W2 = W.clone()
        ws2 = gb.gbnn_prepare(W2, C, L)

        def turn(k, rule=rule):
            gb.gbnn_store_update(W2, C, L, extra[k:k + 1], ws2)
            gb.gbnn_retrieve_symbols(W2, C, L, pd[k:k + 1], rule, 1, max_iters, bits_out=bits[k:k + 1],
                                     symbols_out=sym[k:k + 1], iters_out=it[k:k + 1], workspace=ws2)

        with torch.cuda.stream(side):
            turn(0)
        side.synchronize()
        g2 = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g2, stream=side):
            for k in range(per_graph // 2):
                turn(k)
        g2.replay()
        torch.cuda.synchronize()
        turn_us = _events_us(g2.replay, 20) / (per_graph // 2)

        def whole(rule=rule):
            gb.gbnn_retrieve_symbols(W, C, L, pd, rule, 1, max_iters, bits_out=bits, symbols_out=sym, iters_out=it,
                                     workspace=ws)

        whole()
        torch.cuda.synchronize()
        batch_us = _events_us(whole, 10) / batch
        rows.append({"C": C, "L": L, "M": M, "erased": e, "rule": rule, "call_us": call_us,
                     "call_sync_us": call_sync_us, "graph_us": graph_us, "turn_us": turn_us, "batch_us": batch_us,
                     "batch": batch})
    return rows


def main() -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--C", type=int, default=8)
    ap.add_argument("--L", type=int, default=256)
    ap.add_argument("--M", type=int, default=20000)
    ap.add_argument("--erased", type=int, default=4)
    ap.add_argument("--json", action="store_true")
    args = ap.parse_args()
    rows = measure(args.C, args.L, args.M, args.erased)
    if args.json:
        for r in rows:
            print(json.dumps(r))
        return 0
    print(f"C={args.C} L={args.L} M={args.M} erased={args.erased}: microseconds per probe")
    print("rule        | call   | call+sync | in a graph | store+retrieve turn (graph) | batch of 65536")
    for r in rows:
        print(f"{r['rule']:11s} | {r['call_us']:6.2f} | {r['call_sync_us']:9.2f} | {r['graph_us']:10.2f} | "
              f"{r['turn_us']:27.2f} | {r['batch_us']:.5f}")
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
