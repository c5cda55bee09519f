#!/usr/bin/env python3
"""Benchmark of the paged decode-attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3]

A step is one pass of the whole hot path over one batch of synthetic input
resident in HBM: every decode-attention call of the workload, then the merge
of the partials.  The default workload is the GQA batch-256 decode step
(32 q / 8 kv heads, head_dim 128, bf16, lognormal contexts, split-KV chunks of
1024 tokens, merge).  One JSON line is printed.

  value      KV bytes the step must read / step time  (GB/s), whole job
  roofline   the decode-attention kernel alone: algorithmic bytes per launch /
             its mean duration measured with events on the launch stream,
             against the 8 TB/s HBM peak
  stream_read_GBps   a plain streaming read of the K pool on the same GPU; pct_of_stream_read: value against it
  list_reused   the same step when one work list serves many calls (the layers of a decoding iteration)
  cpu_baseline  the CPU fp64 oracle timed on this host on the same workload
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0

# HBM bytes per decode-attention launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (see
# profiles/), scaled by the factor the same counters show for the plain copy kernel; None = not measured.
MEASURED_TRAFFIC_BYTES = {"cfg3-gqa-b256": 1996.7e6,      # profiles/decode_mfma_persistent_cfg3_pmc.md
                          "cfg2-mha-b64": 2327.6e6,       # profiles/decode_mfma_persistent_cfg2_cfg4_cfg5_pmc.md
                          "cfg4-hybrid-32ls-224be": 322.0e6, "cfg5-long-b32-L32768": 4337.0e6}


def algorithmic_bytes(w) -> int:
    """Bytes one pass of the decode-attention calls must move: the KV of every attended token,
    its share of the block table (4 bytes per 16-token page), q, and the partial rows written."""
    total = w.kv_bytes()
    for c in w.calls:
        tok = np.maximum(c.ctx_end.astype(np.int64) - c.ctx_begin, 0)
        total += int(((tok + w.block_size - 1) // w.block_size).sum()) * 4
        total += w.batch * w.num_q_heads * w.head_dim * w.elem_bytes
        if c.chunk_tokens:
            n_part = int(((tok + c.chunk_tokens - 1) // c.chunk_tokens).sum())
        else:
            n_part = int((tok > 0).sum())
        total += n_part * w.num_q_heads * (w.head_dim + 1) * 4
    return total


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg3", choices=["cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--pools", type=int, default=2, help="physical KV pool copies rotated between steps")
    ap.add_argument("--kernel", type=int, default=0, help="0 auto, 1 vector, 2 matrix-core")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run the plain 1 GiB copy kernel a few times (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (--gpus must be 1)",
              file=sys.stderr)
        return 2

    import torch
    from paper_2603_12831_amd import binding, workloads as wl
    from paper_2603_12831_amd.runner import DeviceWorkload

    if not torch.cuda.is_available():
        print("no GPU visible; the benchmark has no CPU path", file=sys.stderr)
        return 2
    binding.load_library()
    cores = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "16")))

    w = wl.MAKERS[args.workload](workers=cores)
    ext = {}
    host_producer = None
    if w.ext_ranges is not None:
        # hybrid batch: the partial rows over the context that is not GPU-resident come from the host-side
        # producer (KV in host memory, host cores), once, before the timed region
        off = wl.ext_row_offsets(w)
        row_seq = np.array([i for i, rs in enumerate(w.ext_ranges) for _ in rs], dtype=np.int32)
        row_begin = np.array([b for rs in w.ext_ranges for (b, _) in rs], dtype=np.int32)
        row_end = np.array([e for rs in w.ext_ranges for (_, e) in rs], dtype=np.int32)
        h0 = time.perf_counter()
        ext_o, ext_lse = binding.omni_host_partial_attn(w.q, w.k_pool, w.v_pool, w.block_table, row_seq, row_begin,
                                                        row_end, w.sm_scale, w.dtype, n_threads=cores)
        h1 = time.perf_counter()
        host_kv = int((row_end - row_begin).sum()) * 2 * w.num_kv_heads * w.head_dim * w.elem_bytes
        host_producer = {"value": host_kv / (h1 - h0) / 1e9, "unit": "GB/s", "threads": cores,
                         "rows": int(len(row_seq)), "kv_bytes": host_kv, "seconds": h1 - h0}
        ext = dict(ext_o=ext_o, ext_lse=ext_lse, ext_offsets=off)
    dw = DeviceWorkload(w, n_pool_copies=max(1, args.pools), **ext)
    kv_bytes = w.kv_bytes()
    alg_bytes = algorithmic_bytes(w)

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            binding.omni_debug_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst

    # One step = work list + decode attention (the dominant kernel, bracketed by events on its own
    # stream) + merge.  The list is rebuilt every step, as a caller without plan reuse would.
    def step(i, e0=None, e1=None):
        dw.plan()
        if e0 is not None:
            e0.record()
        dw.run_attention(kernel=args.kernel, pool=i % args.pools, planned=True)
        if e1 is not None:
            e1.record()
        dw.run_merge()

    for i in range(args.warmup):
        step(i)
    # events bracket the dominant kernel on every 4th timed step (each record costs a few microseconds of
    # stream time, which would otherwise be charged to every step)
    ev = {i: (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for i in range(0, args.steps, 4)}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i, *ev.get(i, (None, None)))
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    step_ms = (t1 - t0) * 1e3 / args.steps
    attn_ms = float(np.mean([a.elapsed_time(b) for a, b in ev.values()])) / len(w.calls)
    attn_ms_min = float(np.min([a.elapsed_time(b) for a, b in ev.values()])) / len(w.calls)

    achieved = alg_bytes / len(w.calls) / (attn_ms * 1e-3) / 1e9
    out = {
        "metric": "decode-attention KV GB/s (paged decode attention + partial merge, whole step)",
        "value": kv_bytes / (step_ms * 1e-3) / 1e9,
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": step_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == "bf16" else "f32", "accumulate_dtype": "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "q_heads": w.num_q_heads, "kv_heads": w.num_kv_heads,
                   "head_dim": w.head_dim, "page_tokens": w.block_size,
                   "context_tokens_total": int(w.ctx_len.astype(np.int64).sum()),
                   "chunk_tokens": w.calls[0].chunk_tokens, "kv_bytes_per_step": kv_bytes,
                   "pool_copies_rotated": args.pools},
        "pct_hbm_peak": 100.0 * kv_bytes / (step_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "merged_tokens_per_s": w.batch / (step_ms * 1e-3),
        "attention_kernel_ms": attn_ms, "attention_kernel_ms_min": attn_ms_min,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": MEASURED_TRAFFIC_BYTES.get(w.name),
                     "kernel": "decode_mfma_persistent_kernel" if dw.calls[0]["workspace"] is not None and
                     w.dtype == "bf16" and w.head_dim == 128 and args.kernel != 1 else "decode attention",
                     "algorithmic_bytes_per_launch": alg_bytes // len(w.calls)},
    }

    # After the timed loop: the read rate of a plain streaming kernel over the same K pool (what this GPU's
    # HBM gives a pure read).
    def timed(fn, n=50):                # n launches back to back between one pair of events
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        fn()
        a.record()
        for _ in range(n):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n
    # The same step with the work list built once and reused (omni_decode_plan + workspace_planned), as the
    # layers of one decoding iteration would share it: extra information, never `value`.
    def step_planned(i):
        dw.run_attention(kernel=args.kernel, pool=i % args.pools, planned=True)
        dw.run_merge()
    dw.plan()
    for i in range(min(args.warmup, 5)):
        step_planned(i)
    torch.cuda.synchronize()
    p0 = time.perf_counter()
    for i in range(args.steps):
        step_planned(i)
    torch.cuda.synchronize()
    planned_ms = (time.perf_counter() - p0) * 1e3 / args.steps
    out["list_reused"] = {"ms_per_step": planned_ms, "value": kv_bytes / (planned_ms * 1e-3) / 1e9, "unit": "GB/s",
                          "pct_hbm_peak": 100.0 * kv_bytes / (planned_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS}
    pool0 = dw.k_pools[0]
    sink = torch.zeros(16, dtype=torch.uint8, device="cuda")
    nbytes = min(pool0.numel() * pool0.element_size(), 2 << 30)
    stream_ms = timed(lambda: binding.omni_debug_stream_read(pool0, sink, nbytes), n=10)
    out["stream_read_GBps"] = nbytes / (stream_ms * 1e-3) / 1e9
    out["pct_of_stream_read"] = 100.0 * out["value"] / out["stream_read_GBps"]

    if host_producer is not None:
        out["host_partial_producer"] = host_producer

    if not args.no_cpu_baseline:
        from oracle import oracle
        # bounded sample: as many whole sequences (every head, full context) as fit ~2 GB of KV
        per_seq = w.ctx_len.astype(np.int64) * 2 * w.num_kv_heads * w.head_dim * w.elem_bytes
        n_seq = int(min(w.batch, max(1, np.searchsorted(np.cumsum(per_seq), 2.2e9) + 1)))
        seqs = np.arange(n_seq)
        reps = 0
        c0 = time.perf_counter()
        while reps < 20 and (reps == 0 or time.perf_counter() - c0 < 1.5):      # ~20-30 core-seconds of work
            oracle.paged_attn(w.q, w.k_pool, w.v_pool, w.block_table, None, w.ctx_len, w.sm_scale, w.dtype,
                              seqs=seqs, n_threads=cores)
            reps += 1
        c1 = time.perf_counter()
        sample_bytes = int(per_seq[:n_seq].sum()) * reps
        out["cpu_baseline"] = {"value": sample_bytes / (c1 - c0) / 1e9, "unit": "GB/s", "cores": cores,
                               "kind": "oracle",
                               "sample": "fp64 oracle, attention of the first %d of %d sequences (all heads, "
                                         "full contexts), %d passes, %.2f GB of KV in all, %.2f s wall" %
                                         (n_seq, w.batch, reps, sample_bytes / 1e9, c1 - c0)}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
