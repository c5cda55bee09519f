"""Timing of the output-queue leg of the piggybacking data path on the GPU.

    python -m paper_2603_12831_amd.queue_bench [--requests 400] [--reps 50]

For `requests` best-effort requests (32 query heads, head_dim 128) whose attention comes back as one fp32
partial row each: push the rows into the device-resident output queues (O rows and LSE rows, tagged with
the request number), pop them, build their CSR offsets from the tags, and merge them with one GPU-side
partial row per request.  The paper's context figure (System Implementation, overhead analysis) is at most
75 us for queue read / write plus residual save at 400 concurrent requests on its hardware.  Prints one JSON line
with the median time of each operation and of the whole leg.
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
    times = {k: [] for k in list(ops) + ["whole_leg"]}
    for rep in range(args.reps + 3):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(len(ops) + 1)]
        ev[0].record()
        for i, fn in enumerate(ops.values()):
            fn()
            ev[i + 1].record()
        torch.cuda.synchronize()
        if rep >= 3:
            for i, k in enumerate(ops):
                times[k].append(ev[i].elapsed_time(ev[i + 1]) * 1e3)
            times["whole_leg"].append(ev[0].elapsed_time(ev[-1]) * 1e3)
    assert torch.equal(got_o, o) and torch.equal(got_l, lse) and int(n_pop.item()) == n
    res = {"requests": n, "row_bytes": hq * d * 4 + hq * 4, "unit": "us (median of %d)" % args.reps}
    res.update({k: float(np.median(v)) for k, v in times.items()})
    print(json.dumps(res))
    return 0


if __name__ == "__main__":
    sys.exit(main())
