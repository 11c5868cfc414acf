#!/usr/bin/env python3
"""Benchmark: retrieved queries per second at c=8, l=256 (sum-of-max and hybrid), one MI355X.

A step is one sweep of the retrieval hot path over one batch of K device-resident probes:
one gbnn_retrieve call with the sum-of-max rule and one with the hybrid rule (probe load and
rule initialisation, scoring, per-cluster selection, iteration to the fixed point or the cap,
result store).  value = 2*K*steps / elapsed.  Storing the messages (the feeder) is timed
separately and is not part of value; neither are host<->device copies: probes and results stay
in HBM.  Inputs are seeded synthetic uniform-random messages, the paper's own workload.

The same JSON line carries
  roofline      the dominant kernel of the headline workload: algorithmic bytes per launch over its
                launch duration, the median of SAMPLES groups of GROUP launches, each group between two
                HIP events on the launch stream (an event pair around a single launch adds 3-5 us to a
                40 us kernel), in a loop of its own after the timed region (so that the events do not
                stretch that region), the rules taking turns;
  per_config    the same measurement for every other configuration that has a throughput (cfg2,
                cfg4 at three M, cfg5), each with copies of its probe tensor timed beside it (the
                framework's, and the library's reference copy kernel with plain and with non-temporal
                accesses) and a sample of its results compared with the CPU oracle;
  cpu_baseline  the CPU oracle timed on the host cores;
  parity_ok     every sampled result of every workload equals the oracle's.  The exit status is 1
                when it is false.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
SAMPLES = 32           # event-bracketed groups of launches per rule behind every median
GROUP = 4              # launches per group
ORACLE_SAMPLE = 4096   # probes per workload and rule compared with the oracle in per_config
OTHER_WORKLOADS = ("cfg2", "cfg4_m10k", "cfg4_m30k", "cfg4_m50k", "cfg5")


def algorithmic_bytes_per_probe(n: int, K: int, with_iters: bool) -> float:
    """Read the probe once, write the result once, read W once per batch (+ the pass count)."""
    return 2.0 * n + (n * n / 8.0) / K + (4.0 if with_iters else 0.0)


class Loaded:
    """One workload resident in HBM: network stored and prepared, probes, result buffers."""

    def __init__(self, name, torch, gb, inputs):
        import numpy as np
        self.w = w = inputs.WORKLOADS[name]
        self.rules = [r for r in ("sum_of_max", "hybrid", "sum_of_sum") if r in w.rules]
        self.msgs = w.messages()
        self.q, self.er = w.probe_plan()
        self.msgs_d = torch.from_numpy(self.msgs).cuda()
        # probes: the one-hot byte image, built on the device from the same plan (input plumbing)
        idx = torch.from_numpy(inputs.active_neurons(self.msgs[self.q], w.L)).cuda()
        keep = torch.from_numpy((~self.er).astype(np.uint8)).cuda()
        self.V0d = torch.zeros((w.K, w.n), dtype=torch.uint8, device="cuda")
        self.V0d.scatter_(1, idx, keep)
        self.target_idx = idx
        self.W = gb.new_network(w.C, w.L)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        gb.gbnn_store(self.W, w.C, w.L, self.msgs_d)
        torch.cuda.synchronize()
        self.store_s = time.perf_counter() - t0
        self.outs = {r: torch.empty_like(self.V0d) for r in self.rules}
        self.iters = {r: torch.empty(w.K, dtype=torch.int32, device="cuda") for r in self.rules}
        self.ws = torch.empty(gb.gbnn_workspace_bytes(w.C, w.L, w.K, self.rules[0]), dtype=torch.uint8, device="cuda")
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        gb.gbnn_prepare(self.W, w.C, w.L, self.ws)  # once per network, like the store: derived tables of W
        torch.cuda.synchronize()
        self.prepare_s = time.perf_counter() - t0
        self.gb, self.torch = gb, torch

    def call(self, rule):
        w = self.w
        self.gb.gbnn_retrieve(self.W, w.C, w.L, self.V0d, rule, w.gamma, w.max_iters, V_out=self.outs[rule],
                              iters_out=self.iters[rule], workspace=self.ws)

    def host_probes(self, K):
        """First K probes on the host, from the plan (what the oracle reads)."""
        from paper_1303_7032_amd import inputs
        return inputs.one_hot(self.msgs[self.q[:K]], self.w.L, self.er[:K])


def event_samples(torch, fn, count, warm=3):
    """Milliseconds of `count` single launches of fn, each between two events on the current stream."""
    import numpy as np
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(count)]
    for _ in range(warm):
        fn()
    for a, b in evs:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    return np.array([a.elapsed_time(b) for a, b in evs])


def measure_rules(ld, torch):
    """Per rule: median / min / mean launch duration over SAMPLES groups of GROUP launches, each group between
    two HIP events, and what they mean in bytes.  The rules take turns group by group."""
    import numpy as np
    w = ld.w
    abytes = algorithmic_bytes_per_probe(w.n, w.K, True) * w.K
    evs = {r: [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(SAMPLES)]
           for r in ld.rules}
    for _ in range(3):
        for r in ld.rules:
            ld.call(r)
    for i in range(SAMPLES):
        for r in ld.rules:
            a, b = evs[r][i]
            a.record()
            for _ in range(GROUP):
                ld.call(r)
            b.record()
    torch.cuda.synchronize()
    per_rule = {}
    for r in ld.rules:
        ms = np.array([a.elapsed_time(b) for a, b in evs[r]]) / GROUP
        med = float(np.median(ms))
        per_rule[r] = {"us_median": med * 1e3, "us_min": float(ms.min()) * 1e3, "us_mean": float(ms.mean()) * 1e3,
                       "samples": SAMPLES, "launches_per_sample": GROUP, "qps": w.K / (med * 1e-3),
                       "hbm_GBs": abytes / (med * 1e-3) / 1e9, "frac_of_8TBs": abytes / (med * 1e-3) / 1e9 / HBM_PEAK_GBS}
    return per_rule, abytes


def device_copy(ld, torch):
    """A plain device copy of the probe tensor (read K*n bytes, write K*n): median of 10, GB/s."""
    import numpy as np
    scratch = torch.empty_like(ld.V0d)
    ms = event_samples(torch, lambda: scratch.view(torch.int64).copy_(ld.V0d.view(torch.int64)), 10)
    del scratch
    med = float(np.median(ms))
    return med * 1e3, 2.0 * ld.w.K * ld.w.n / (med * 1e-3) / 1e9


def reference_copies(ld, torch):
    """The library's own copy kernel on the probe tensor (one wavefront per 2 KiB, as the retrieval kernels move
    activity), with plain and with non-temporal accesses: what the memory system delivers for one read and one
    write stream of the batch's size.  Microseconds (median of 10 groups of GROUP launches) and GB/s."""
    import numpy as np
    scratch = torch.empty_like(ld.V0d)
    out = {}
    for name, streaming in (("plain", False), ("streaming", True)):
        def go():
            for _ in range(GROUP):
                ld.gb.gbnn_reference_copy(scratch, ld.V0d, streaming)
        med = float(np.median(event_samples(torch, go, 10))) / GROUP
        out[name] = {"us": med * 1e3, "GBs": 2.0 * ld.w.K * ld.w.n / (med * 1e-3) / 1e9}
    assert torch.equal(scratch, ld.V0d)
    del scratch
    return out


def outcome(ld, torch):
    """Error rate (exact one-hot match with the source message), mean passes, capped probes, per rule."""
    w = ld.w
    stats = {}
    for r in ld.rules:
        o = ld.outs[r].view(w.K, w.n)
        ok = (o.sum(dim=1, dtype=torch.int32) == w.C) & (o.gather(1, ld.target_idx).sum(dim=1, dtype=torch.int32) == w.C)
        it = ld.iters[r]
        stats[r] = {"error_rate": 1.0 - float(ok.float().mean()), "mean_passes": float(it.abs().float().mean()),
                    "capped": int((it < 0).sum())}
    return stats


def oracle_check(ld, Ks, nthreads=0):
    """The oracle on the first Ks probes, every rule; returns (all results equal, seconds, threads used)."""
    from oracle import gbnn_oracle as orc
    w = ld.w
    Wo, _ = orc.store(w.C, w.L, ld.msgs)
    V0 = ld.host_probes(Ks)
    same, used = {}, 1
    t0 = time.perf_counter()
    refs = {}
    for r in ld.rules:
        refs[r] = orc.retrieve(Wo, w.C, w.L, V0, r, w.gamma, w.max_iters, nthreads=nthreads)
        used = refs[r][2]
    secs = time.perf_counter() - t0
    for r in ld.rules:  # untimed: the GPU results against the oracle's
        ref, itref, _ = refs[r]
        same[r] = bool((ld.outs[r][:Ks].cpu().numpy() == ref).all() and (ld.iters[r][:Ks].cpu().numpy() == itref).all())
    return same, secs, used, Wo, V0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg3", help="cfg3 (default), cfg4_m10k, cfg4_m30k, cfg4_m50k, cfg5, cfg2")
    ap.add_argument("--only", action="store_true", help="the named workload alone: no per_config section")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle (no cpu_baseline, no parity check)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the message-boundary and dense-product reference points (for profiler runs)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run 3 plain device copies of the probe tensor (K*n bytes read, K*n written) after the "
                         "timed region: the known-size reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (probes are independent, so more GPUs would just "
              "shard the batch with no exchange); run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_1303_7032_amd import binding as gb
    from paper_1303_7032_amd import inputs

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    gb.lib()

    # ---- inputs, resident in HBM before anything is timed
    ld = Loaded(args.workload, torch, gb, inputs)
    w, rules = ld.w, ld.rules
    C, L, n, K = w.C, w.L, w.n, w.K

    # the same store into a zeroed scratch network, bracketed by events (device time, first call excluded)
    W2 = gb.new_network(C, L)
    store_us = []
    for _ in range(5):
        W2.zero_()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        gb.gbnn_store(W2, C, L, ld.msgs_d)
        ev1.record()
        torch.cuda.synchronize()
        store_us.append(ev0.elapsed_time(ev1) * 1e3)
    assert torch.equal(ld.W, W2)
    del W2
    store_event_us = sorted(store_us)[len(store_us) // 2]

    for _ in range(args.warmup):
        for r in rules:
            ld.call(r)
    torch.cuda.synchronize()

    # ---- timed region: exactly `steps` steps of plain launches
    t0 = time.perf_counter()
    for _ in range(args.steps):
        for r in rules:
            ld.call(r)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    queries_per_step = K * len(rules)
    value = queries_per_step * args.steps / elapsed

    # ---- per launch, after the timed region: SAMPLES launches of each rule between HIP events
    per_rule, abytes = measure_rules(ld, torch)
    dominant = max(rules, key=lambda r: per_rule[r]["us_median"])
    achieved = per_rule[dominant]["hbm_GBs"]
    # HBM-side bytes per launch of the dominant kernel, from rocprofv3 counter runs kept under profiles/
    traffic = traffic_detail = None
    tfile = ROOT / "profiles" / "hbm_traffic.json"
    if tfile.exists():
        traffic_detail = json.loads(tfile.read_text()).get(f"{args.workload}:{dominant}")
        if traffic_detail:
            traffic = traffic_detail["total_bytes"]

    copy_us, copy_GBs = device_copy(ld, torch)
    ref_copies = reference_copies(ld, torch)

    # ---- reference point: the same retrieval with messages at the boundary (gbnn_retrieve_symbols: symbols in,
    # packed bits + symbols + pass counts out)
    message_boundary = {}
    dense_product = None
    if not args.no_extras:
        probes_h = ld.msgs[ld.q].copy()
        probes_h[ld.er] = -1
        probes_d = torch.from_numpy(probes_h).cuda()
        nw = gb.gbnn_w_row_words(C, L)
        mb_bits = torch.empty((K, nw), dtype=torch.int32, device="cuda")
        mb_sym = torch.empty((K, C), dtype=torch.int32, device="cuda")
        mb_it = torch.empty(K, dtype=torch.int32, device="cuda")
        mb_bytes = (4.0 * C + 4.0 * nw + 4.0 * C + 4.0) * K + n * n / 8.0
        for r in rules:
            ms = event_samples(torch, lambda: gb.gbnn_retrieve_symbols(
                ld.W, C, L, probes_d, r, w.gamma, w.max_iters, bits_out=mb_bits, symbols_out=mb_sym, iters_out=mb_it,
                workspace=ld.ws), SAMPLES)
            med = float(np.median(ms))
            message_boundary[r] = {"us_median": med * 1e3, "qps": K / (med * 1e-3), "hbm_bytes_per_launch": mb_bytes,
                                   "hbm_GBs": mb_bytes / (med * 1e-3) / 1e9,
                                   "same_pass_counts_as_activity_boundary": bool((mb_it == ld.iters[r]).all())}
        del probes_d, mb_bits, mb_sym, mb_it

        # ---- sum-of-sum only: what one pass of the dense formulation S = W V (Eq. 8) costs as a library int8
        # GEMM on the same batch (a reference point for the choice of the sparse bit-sliced form; not used by
        # the path, and its output S would still need Eq. (4)-(5))
        if "sum_of_sum" in rules:
            try:
                shifts = torch.arange(32, device="cuda", dtype=torch.int32)
                W8 = ((ld.W.view(n, nw, 1) >> shifts) & 1).reshape(n, nw * 32)[:, :n].to(torch.int8).contiguous()
                V8 = ld.V0d.t().contiguous().view(torch.int8)
                S = None

                def gemm():
                    nonlocal S
                    S = torch._int_mm(W8, V8)
                us = float(np.median(event_samples(torch, gemm, 5, warm=2))) * 1e3
                dense_product = {"what": "torch._int_mm(W int8[n][n], V int8[n][K]) -> int32[n][K], one pass, library GEMM",
                                 "us_per_pass": us, "int8_TOPs": 2.0 * n * n * K / (us * 1e-6) / 1e12}
                del S, W8, V8
            except Exception as exc:  # the library may lack the routine for this shape
                dense_product = {"error": repr(exc)[:200]}

    if args.calibrate_copy:
        for _ in range(3):
            ld.outs[rules[0]].view(torch.int64).copy_(ld.V0d.view(torch.int64))  # 8-byte elements: full-width stores
        torch.cuda.synchronize()
        ld.call(rules[0])  # restore the result the copy overwrote
        torch.cuda.synchronize()

    # ---- outcome of the retrieval (outside the timed region)
    for r, st in outcome(ld, torch).items():
        per_rule[r].update(st)

    # ---- CPU oracle on the host cores (a reported baseline, not the target)
    cpu = None
    parity = {}
    if not args.no_cpu_baseline:
        from oracle import gbnn_oracle as orc
        Ks = min(K, 65536)
        same, cpu_s, used, Wo, V0 = oracle_check(ld, Ks)
        for r in rules:
            per_rule[r]["matches_oracle_on_sample"] = same[r]
            parity[f"{args.workload}:{r}"] = same[r]
        K1 = min(K, 4096)
        t0 = time.perf_counter()
        for r in rules:
            orc.retrieve(Wo, C, L, V0[:K1], r, w.gamma, w.max_iters, nthreads=1)
        one_s = time.perf_counter() - t0
        cpu = {"value": Ks * len(rules) / cpu_s, "unit": "queries/s", "cores": used, "kind": "oracle",
               "sample": f"first {Ks} probes of the batch, rules {'+'.join(rules)}, {cpu_s:.2f} s wall on {used} threads",
               "single_thread_value": K1 * len(rules) / one_s, "single_thread_sample": f"first {K1} probes, {one_s:.2f} s"}
        del Wo, V0

    headline = {"store_s": ld.store_s, "prepare_s": ld.prepare_s, "seed": w.seed, "density": w.density(), "M": w.M,
                "kernel_path": gb.gbnn_retrieve_path(C, L, rules[0], ld.V0d, ld.outs[rules[0]])}
    del ld
    gc.collect()
    torch.cuda.empty_cache()

    # ---- every other configuration with a throughput: the same per-launch measurement
    per_config = {}
    if not args.only and args.workload == "cfg3":
        for name in OTHER_WORKLOADS:
            o = Loaded(name, torch, gb, inputs)
            rules_o, abytes_o = measure_rules(o, torch)
            cus, cgbs = device_copy(o, torch)
            refc = reference_copies(o, torch)
            for r, st in outcome(o, torch).items():
                rules_o[r].update(st)
                rules_o[r]["frac_of_device_copy"] = rules_o[r]["hbm_GBs"] / cgbs
            if not args.no_cpu_baseline:
                same, _, _, _, _ = oracle_check(o, min(o.w.K, ORACLE_SAMPLE))
                for r in o.rules:
                    rules_o[r]["matches_oracle_on_sample"] = same[r]
                    parity[f"{name}:{r}"] = same[r]
            per_config[name] = {"workload": f"C={o.w.C} L={o.w.L} n={o.w.n} M={o.w.M} K={o.w.K} erased={o.w.e} "
                                            f"cap={o.w.max_iters} gamma={o.w.gamma}",
                                "kernel_path": gb.gbnn_retrieve_path(o.w.C, o.w.L, o.rules[0], o.V0d, o.outs[o.rules[0]]),
                                "algorithmic_bytes_per_launch": abytes_o, "device_copy_us": cus, "device_copy_GBs": cgbs,
                                "reference_copy": refc,
                                "oracle_sample": 0 if args.no_cpu_baseline else min(o.w.K, ORACLE_SAMPLE), "rules": rules_o}
            del o
            gc.collect()
            torch.cuda.empty_cache()

    parity_ok = all(parity.values()) if parity else None
    line = {
        "metric": "retrieved queries/sec at c=8,l=256 (sum-of-max, hybrid)" if (C, L) == (8, 256)
                  else f"retrieved queries/sec at c={C},l={L} ({', '.join(rules)})",
        "value": value, "unit": "queries/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32",  # bitwise / integer arithmetic on 32-bit words of packed bits (activity crosses the boundary as u8)
        "data": "synthetic",
        "config": {"workload": f"{w.name}: C={C} L={L} n={n} M={headline['M']} K={K} erased={w.e} cap={w.max_iters} "
                               f"rules={'+'.join(rules)} (one step = one gbnn_retrieve per rule over the batch)",
                   "queries_per_step": queries_per_step, "seed": headline["seed"], "density": headline["density"],
                   "kernel_path": headline["kernel_path"]},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_detail": traffic_detail,
                     "kernel": f"gbnn_retrieve[{dominant}]", "us_median": per_rule[dominant]["us_median"],
                     "event_samples": SAMPLES, "launches_per_sample": GROUP, "algorithmic_bytes_per_launch": abytes,
                     "device_copy_us_same_run": copy_us, "device_copy_GBs_same_run": copy_GBs,
                     "frac_of_device_copy": achieved / copy_GBs, "reference_copy": ref_copies},
        "cpu_baseline": cpu,
        "parity_ok": parity_ok,
        "per_rule": per_rule,
        "per_config": per_config,
        "message_boundary": message_boundary,
        "dense_product_reference": dense_product,
        "store": {"messages": headline["M"], "seconds_incl_launch_and_sync": headline["store_s"], "event_us": store_event_us,
                  "messages_per_second": headline["M"] / (store_event_us * 1e-6),
                  "prepare_seconds_incl_launch_and_sync": headline["prepare_s"]},
    }
    print(json.dumps(line))
    if parity_ok is False:
        print("bench.py: a sampled result differs from the oracle: " +
              ", ".join(k for k, v in parity.items() if not v), file=sys.stderr)
        return 1
    return 0


if __name__ == "__main__":
    sys.exit(main())
