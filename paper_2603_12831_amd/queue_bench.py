"""Timing of the output-queue leg of the piggybacking data path on the GPU.

    python -m paper_2603_12831_amd.queue_bench [--requests 400] [--reps 50]

For `requests` best-effort requests (32 query heads, head_dim 128) whose attention comes back as one fp32
partial row each: push the rows into the device-resident output queues (O rows and LSE rows, tagged with
the request number), pop them, build their CSR offsets from the tags, and merge them with one GPU-side
partial row per request.  The paper's context figure (System Implementation, overhead analysis) is at most
75 us for queue read / write plus residual save at 400 concurrent requests on its hardware, and about 0.5 ms
for the non-contiguous residual load.  Prints one JSON line with the median time of each operation, of the
whole leg, and of a residual save and load of 16 KiB rows.
"""
from __future__ import annotations

import argparse
import json
import sys

import numpy as np


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--requests", type=int, default=400)
    ap.add_argument("--reps", type=int, default=50)
    args = ap.parse_args()
    import torch
    from . import binding

    if not torch.cuda.is_available():
        print("needs a GPU", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    n, hq, d = args.requests, 32, 128
    cap = 2 * n
    # (a queue struct holds addresses only: the tensors stay alive in `mem`)
    mem = [(torch.zeros((cap, row_bytes), dtype=torch.uint8, device=dev), torch.zeros(cap, dtype=torch.int32, device=dev),
            torch.zeros(4, dtype=torch.int32, device=dev)) for row_bytes in (hq * d * 4, hq * 4)]
    qo, ql = binding.make_queue(*mem[0]), binding.make_queue(*mem[1])
    o = torch.randn(n, hq, d, device=dev)
    lse = torch.randn(n, hq, device=dev)
    tags = torch.arange(n, dtype=torch.int32, device=dev)
    got_o, got_l, got_t = torch.empty_like(o), torch.empty_like(lse), torch.empty_like(tags)
    n_pop = torch.zeros(1, dtype=torch.int32, device=dev)
    offsets = torch.zeros(n + 1, dtype=torch.int32, device=dev)
    tail_o = torch.randn(n, 1, hq, d, device=dev)
    tail_l = torch.randn(n, 1, hq, device=dev)
    out_o = torch.empty(n, hq, d, dtype=torch.bfloat16, device=dev)
    out_l = torch.empty(n, hq, device=dev)
    o8, l8 = o.view(torch.uint8).reshape(n, -1), lse.view(torch.uint8).reshape(n, -1)
    g8, gl8 = got_o.view(torch.uint8).reshape(n, -1), got_l.view(torch.uint8).reshape(n, -1)
    ops = {
        "push": lambda: (binding.omni_queue_push(qo, o8, tags), binding.omni_queue_push(ql, l8, tags)),
        "pop": lambda: (binding.omni_queue_pop(qo, g8, got_t, n_pop), binding.omni_queue_pop(ql, gl8, None, None)),
        "csr_from_tags": lambda: binding.omni_csr_from_tags(got_t, n_pop, n, offsets),
        "merge": lambda: binding.omni_merge_partials(n, hq, d, [(got_o, got_l, offsets, 0), (tail_o, tail_l, None, 1)],
                                                     out_o, out_l),
    }
    # Device-side times: a ~150 us streaming read goes first, so that the host has issued every call of the leg
    # before the GPU gets to the first one (otherwise these short launches are timed at the rate the host
    # issues them).  Host-side time of the whole leg: from the first call to the end of a synchronisation.
    import time
    busy = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    sink = torch.zeros(16, dtype=torch.uint8, device=dev)
    times = {k: [] for k in list(ops) + ["whole_leg", "whole_leg_host_driven"]}
    for rep in range(args.reps + 3):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(len(ops) + 1)]
        binding.omni_debug_stream_read(busy, sink)
        ev[0].record()
        for i, fn in enumerate(ops.values()):
            fn()
            ev[i + 1].record()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for fn in ops.values():
            fn()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        if rep >= 3:
            for i, k in enumerate(ops):
                times[k].append(ev[i].elapsed_time(ev[i + 1]) * 1e3)
            times["whole_leg"].append(ev[0].elapsed_time(ev[-1]) * 1e3)
            times["whole_leg_host_driven"].append((t1 - t0) * 1e6)
    assert torch.equal(got_o, o) and torch.equal(got_l, lse) and int(n_pop.item()) == n
    # the residual store beside it: 16 KiB rows (a hidden state of 8192 bf16 values) saved to and loaded from
    # scattered slots of a store four times the number of requests
    store = torch.zeros((4 * n, 16384), dtype=torch.uint8, device=dev)
    slots = torch.randperm(4 * n, device=dev)[:n].to(torch.int32)
    resid = torch.randint(0, 255, (n, 16384), dtype=torch.uint8, device=dev)
    back = torch.empty_like(resid)
    rops = {"residual_save": lambda: binding.omni_residual_save(store, slots, resid),
            "residual_load": lambda: binding.omni_residual_load(store, slots, back)}
    for k in rops:
        times[k] = []
    for rep in range(args.reps + 3):
        for k, fn in rops.items():
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            binding.omni_debug_stream_read(busy, sink)
            a.record()
            fn()
            b.record()
            torch.cuda.synchronize()
            if rep >= 3:
                times[k].append(a.elapsed_time(b) * 1e3)
    assert torch.equal(back, resid)
    res = {"requests": n, "row_bytes": hq * d * 4 + hq * 4, "residual_row_bytes": 16384,
           "unit": "us (median of %d)" % args.reps}
    res.update({k: float(np.median(v)) for k, v in times.items()})
    print(json.dumps(res))
    return 0


if __name__ == "__main__":
    sys.exit(main())
