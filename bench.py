#!/usr/bin/env python3
"""Benchmark of the paged decode-attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3] [--only]

A step is one pass of the whole hot path over one batch of synthetic input resident in HBM: the work list,
every decode-attention call of the workload, then the merge of the partial rows of the sequences the
attention call could not finish itself.  The headline workload is the GQA batch-256 decode step (32 q / 8 kv
heads, head_dim 128, bf16, lognormal contexts, split-KV chunks of 1024 tokens, merge); unless --only is
given, the other bandwidth workloads (MHA batch 64, hybrid piggyback batch, long-context batch 32) are
measured after it with the same protocol and reported under "workloads".  One JSON line is printed.

  value         KV bytes the step must read / step time (GB/s), whole job, wall clock over the K timed steps
  step_ms_median / step_ms_min   the same step bracketed by events, once per step, in a second pass of K steps
  roofline      the decode-attention kernel alone: algorithmic bytes per launch / its mean duration measured
                with events on the launch stream inside the timed loop, against the 8 TB/s HBM peak;
                traffic = HBM bytes per launch from counter runs (profiles/hbm_traffic.json), null if the
                kernel sources have changed since they were taken
  stream_read_GBps   a plain streaming read of the K pool on the same GPU; pct_of_stream_read: value against it
  list_reused   the same step when one work list serves many calls (the layers of a decoding iteration)
  unsplit       (chunked workloads; not with --only) context only: the same batch as one range per sequence,
                i.e. without the split-KV the configuration prescribes (no partial rows, no merge launch)
  fused_form    (hybrid batch) the step when the attention launch folds the host-produced rows in and finishes
                every sequence itself: no merge launch
  host_partial_producer   (hybrid batch) the host-side producer of the rows computed elsewhere, against a
                streaming read of the same host memory by the same threads
  cpu_baseline  the CPU fp64 oracle timed on this host on a bounded sample of the headline workload
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")
KERNEL_SOURCES = ("paper_2603_12831_amd/csrc/decode_mfma.hip", "paper_2603_12831_amd/csrc/omni_internal.hpp")
OTHER_WORKLOADS = ("cfg2", "cfg4", "cfg5")


def kernel_source_hash() -> str:
    h = hashlib.sha256()
    for rel in KERNEL_SOURCES:
        with open(os.path.join(ROOT, rel), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic(workload_name: str):
    """HBM bytes per decode-attention launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (see profiles/),
    valid only for the kernel sources they were taken with."""
    try:
        with open(TRAFFIC_FILE) as f:
            t = json.load(f)
    except (OSError, ValueError):
        return None
    if t.get("kernel_source_hash") != kernel_source_hash():
        return None
    return t.get("bytes_per_launch", {}).get(workload_name)


def algorithmic_bytes(w, final_rows: bool) -> int:
    """Bytes one pass of the decode-attention calls must move: the KV of every attended token, its share of
    the block table (4 bytes per 16-token page), q, and one output row per non-empty chunk: an fp32 partial
    row with its LSE, or, where the call writes final rows, the row in the output type with its LSE for a
    sequence that has a single non-empty chunk and no rows from elsewhere."""
    total = w.kv_bytes()
    out_bytes = 2 if w.out_dtype == "bf16" else 4
    has_ext = np.zeros(w.batch, dtype=bool)            # sequences with rows computed elsewhere are never final
    if w.ext_ranges is not None:
        has_ext = np.array([len(rs) > 0 for rs in w.ext_ranges])
    for c in w.calls:
        tok = np.maximum(c.ctx_end.astype(np.int64) - c.ctx_begin, 0)
        total += int(((tok + w.block_size - 1) // w.block_size).sum()) * 4
        total += w.batch * w.num_q_heads * w.head_dim * w.elem_bytes
        n_chunks = (tok + c.chunk_tokens - 1) // c.chunk_tokens if c.chunk_tokens else (tok > 0).astype(np.int64)
        n_final = int(((n_chunks == 1) & ~has_ext).sum()) if final_rows else 0
        total += (int(n_chunks.sum()) - n_final) * w.num_q_heads * (w.head_dim + 1) * 4
        total += n_final * w.num_q_heads * (w.head_dim * out_bytes + 4)
    return total


def make_device_workload(name, cores, pools):
    """Synthetic inputs of one workload, uploaded; for the hybrid batch the rows of the context that is not
    GPU-resident come from the host-side producer (KV in host memory, host cores), once, before any timing."""
    from paper_2603_12831_amd import binding, workloads as wl
    from paper_2603_12831_amd.runner import DeviceWorkload

    w = wl.MAKERS[name](workers=cores)
    ext, host_producer = {}, None
    if w.ext_ranges is not None:
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
        host_producer.update(host_stream_reference(w, cores, host_kv, h1 - h0))
        ext = dict(ext_o=ext_o, ext_lse=ext_lse, ext_offsets=off)
    # "final": the attention call writes the final rows of the sequences it can finish (one non-empty chunk),
    # the masked merge does the rest; a single one-chunk call with nothing to merge writes all rows itself
    mode = "final" if len(w.calls) == 1 else "merge"
    dw = DeviceWorkload(w, n_pool_copies=max(1, pools), mode=mode, **ext)
    dw.host_rows = ext                                  # (kept for the fused-form measurement of the hybrid batch)
    return w, dw, host_producer


def host_stream_reference(w, cores, host_kv, producer_seconds):
    """What this host's memory gives `cores` threads that only read the same K and V pools (contiguous slabs,
    one per thread): the streaming reference the host-side producer is set against."""
    from paper_2603_12831_amd import binding
    pools = (w.k_pool, w.v_pool)
    for p in pools:
        binding.omni_debug_host_stream_read(p, cores)          # page the data in
    t0 = time.perf_counter()
    for p in pools:
        binding.omni_debug_host_stream_read(p, cores)
    t1 = time.perf_counter()
    rate = sum(p.nbytes for p in pools) / (t1 - t0) / 1e9
    return {"host_stream_read_GBps": rate, "frac_of_host_stream_read": (host_kv / producer_seconds / 1e9) / rate}


def run_workload(name, steps, warmup, pools, kernel, cores, min_seconds=0.0, unsplit=True):
    """Times one workload; returns (its report, the workload, the device buffers).  `min_seconds`: take more
    than `steps` steps (and warm-up steps) if that many would fill less than this much time - a timed region
    of a few milliseconds mostly measures its own two ends."""
    import torch
    from paper_2603_12831_amd import binding

    w, dw, host_producer = make_device_workload(name, cores, pools)
    kv_bytes = w.kv_bytes()
    alg_bytes = algorithmic_bytes(w, dw.mode == "final")
    n_calls = len(w.calls)

    # One step = work list + decode attention (the dominant kernel, bracketed by events on its own stream) +
    # merge.  The list is rebuilt every step, as a caller without plan reuse would.
    def step(i, e0=None, e1=None):
        dw.plan()
        if e0 is not None:
            e0.record()
        dw.run_attention(kernel=kernel, pool=i % pools, planned=True)
        if e1 is not None:
            e1.record()
        dw.run_merge()

    # bring the GPU to its operating clocks before the warm-up steps (not steps: plain streaming reads of the
    # K pool for about 50 ms; a fresh process that goes straight into a few short steps is otherwise timed
    # while the clocks still ramp up)
    sink = torch.zeros(16, dtype=torch.uint8, device="cuda")
    spin_bytes = min(dw.k_pools[0].numel() * dw.k_pools[0].element_size(), 1 << 30)
    for _ in range(int(0.05 / (spin_bytes / 6e12)) + 1):
        binding.omni_debug_stream_read(dw.k_pools[0], sink, spin_bytes)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    if min_seconds > 0.0 and warmup > 0:
        est = (time.perf_counter() - t0) / warmup
        steps = max(steps, int(min_seconds / est))
        for i in range(int(0.4 * min_seconds / est)):
            step(i)
    # events bracket the dominant kernel on every 4th timed step (each record costs a few microseconds of
    # stream time, which would otherwise be charged to every step)
    ev = {i: (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for i in range(0, steps, 4)}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i, *ev.get(i, (None, None)))
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    step_ms = (t1 - t0) * 1e3 / steps
    attn = [a.elapsed_time(b) / n_calls for a, b in ev.values()]
    attn_ms, attn_ms_min = float(np.mean(attn)), float(np.min(attn))

    # second pass: every step bracketed by its own pair of events (median and minimum of the step)
    sev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for i, (a, b) in enumerate(sev):
        a.record()
        step(i)
        b.record()
    torch.cuda.synchronize()
    per_step = sorted(a.elapsed_time(b) for a, b in sev)

    args0 = dw.decode_args(dw.calls[0], kernel, 0, True)
    achieved = alg_bytes / n_calls / (attn_ms * 1e-3) / 1e9
    rep = {
        "ms_per_step": step_ms, "value": kv_bytes / (step_ms * 1e-3) / 1e9, "unit": "GB/s",
        "pct_hbm_peak": 100.0 * kv_bytes / (step_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "step_ms_median": per_step[len(per_step) // 2], "step_ms_min": per_step[0],
        "merged_tokens_per_s": w.batch / (step_ms * 1e-3),
        "attention_kernel_ms": attn_ms, "attention_kernel_ms_min": attn_ms_min,
        "kv_bytes_per_step": kv_bytes, "pool_copies_rotated": pools, "final_rows": dw.mode, "steps": steps,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": measured_traffic(w.name),
                     "kernel": binding.omni_decode_kernel_name(args0),
                     "algorithmic_bytes_per_launch": alg_bytes // n_calls},
    }
    # The same step with the work list built once and reused (omni_decode_plan + workspace_planned), as the
    # layers of one decoding iteration would share it: extra information, never `value`.
    def rate(ms):
        return {"ms_per_step": ms, "value": kv_bytes / (ms * 1e-3) / 1e9, "unit": "GB/s",
                "pct_hbm_peak": 100.0 * kv_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS}

    def time_steps(fn, n_warm):
        for i in range(n_warm):
            fn(i)
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        for i in range(steps):
            fn(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - c0) * 1e3 / steps

    def step_planned(i):
        dw.run_attention(kernel=kernel, pool=i % pools, planned=True)
        dw.run_merge()

    dw.plan()
    rep["list_reused"] = rate(time_steps(step_planned, 5))
    if unsplit and len(w.calls) == 1 and w.calls[0].chunk_tokens > 0 and w.ext_ranges is None:
        # Context, never `value`: the same batch handed over as one range per sequence (no split-KV, hence no
        # partial rows and no merge launch; the kernel's tickets balance the load by themselves), list rebuilt.
        import copy
        from paper_2603_12831_amd.runner import DeviceWorkload
        from paper_2603_12831_amd.workloads import DecodeCall
        w1 = copy.copy(w)
        w1.calls = [DecodeCall(w.calls[0].ctx_begin, w.calls[0].ctx_end, 0, 1)]
        udw = DeviceWorkload(w1, mode="final", pools_from=dw)

        def unsplit_step(i):
            udw.plan()
            udw.run_attention(kernel=kernel, pool=i % pools, planned=True)

        rep["unsplit"] = rate(time_steps(unsplit_step, max(warmup, 10)))
        del udw
    if host_producer is not None:
        rep["host_partial_producer"] = host_producer
        # the hybrid batch also in the fused form: the attention launch folds the host-produced rows in and
        # finishes every sequence itself, no merge launch (same inputs, list rebuilt every step)
        from paper_2603_12831_amd.runner import DeviceWorkload
        fdw = DeviceWorkload(w, n_pool_copies=max(1, pools), mode="fused", **dw.host_rows)

        def fused_step(i):
            fdw.plan()
            fdw.run_attention(kernel=kernel, pool=i % pools, planned=True)

        rep["fused_form"] = rate(time_steps(fused_step, max(warmup, 10)))
        rep["fused_form"]["list_reused"] = rate(time_steps(lambda i: fdw.run_attention(kernel=kernel, pool=i % pools, planned=True), 5))
        del fdw
    return rep, w, dw


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg3", choices=["cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--only", action="store_true", help="measure the named workload only")
    ap.add_argument("--pools", type=int, default=0,
                    help="physical KV pool copies rotated between steps (0: 2, and 4 for the hybrid batch)")
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
    from paper_2603_12831_amd import binding

    if not torch.cuda.is_available():
        print("no GPU visible; the benchmark has no CPU path", file=sys.stderr)
        return 2
    binding.load_library()
    cores = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "16")))

    def pools_for(name):
        # the hybrid batch's 0.3 GB would stay in the 256 MB Infinity Cache: four copies of its pools
        return args.pools if args.pools > 0 else (4 if name == "cfg4" else 2)

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            binding.omni_debug_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst

    # (--only is what the profiles run: every launch of the attention kernel is then one of the workload as configured)
    head, w, dw = run_workload(args.workload, args.steps, args.warmup, pools_for(args.workload), args.kernel, cores,
                               unsplit=not args.only)
    pools = pools_for(args.workload)
    kv_bytes = w.kv_bytes()
    out = {
        "metric": "decode-attention KV GB/s (paged decode attention + partial merge, whole step)",
        "value": head["value"], "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == "bf16" else "f32", "accumulate_dtype": "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "q_heads": w.num_q_heads, "kv_heads": w.num_kv_heads,
                   "head_dim": w.head_dim, "page_tokens": w.block_size,
                   "context_tokens_total": int(w.ctx_len.astype(np.int64).sum()),
                   "chunk_tokens": w.calls[0].chunk_tokens, "kv_bytes_per_step": kv_bytes,
                   "pool_copies_rotated": pools, "final_rows": head["final_rows"]},
    }
    for k in ("pct_hbm_peak", "step_ms_median", "step_ms_min", "merged_tokens_per_s", "attention_kernel_ms",
              "attention_kernel_ms_min", "roofline", "host_partial_producer", "fused_form"):
        if k in head:
            out[k] = head[k]

    def timed(fn, n=50):                # n launches back to back between one pair of events
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        fn()
        a.record()
        for _ in range(n):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n

    out["list_reused"] = head["list_reused"]
    if "unsplit" in head:
        out["unsplit"] = head["unsplit"]
    # the read rate of a plain streaming kernel over the same K pool (what this GPU's HBM gives a pure read)
    pool0 = dw.k_pools[0]
    sink = torch.zeros(16, dtype=torch.uint8, device="cuda")
    nbytes = min(pool0.numel() * pool0.element_size(), 2 << 30)
    stream_ms = timed(lambda: binding.omni_debug_stream_read(pool0, sink, nbytes), n=10)
    out["stream_read_GBps"] = nbytes / (stream_ms * 1e-3) / 1e9
    out["pct_of_stream_read"] = 100.0 * out["value"] / out["stream_read_GBps"]

    if not args.no_cpu_baseline:
        from oracle import oracle
        per_seq = w.ctx_len.astype(np.int64) * 2 * w.num_kv_heads * w.head_dim * w.elem_bytes

        def time_oracle(budget_bytes, n_threads, max_reps, min_seconds):
            n_seq = int(min(w.batch, max(1, np.searchsorted(np.cumsum(per_seq), budget_bytes) + 1)))
            seqs = np.arange(n_seq)
            reps, c0 = 0, time.perf_counter()
            while reps < max_reps and (reps == 0 or time.perf_counter() - c0 < min_seconds):
                oracle.paged_attn(w.q, w.k_pool, w.v_pool, w.block_table, None, w.ctx_len, w.sm_scale, w.dtype,
                                  seqs=seqs, n_threads=n_threads)
                reps += 1
            secs = time.perf_counter() - c0
            return int(per_seq[:n_seq].sum()) * reps / secs / 1e9, n_seq, reps, secs

        # bounded samples: whole sequences (every head, full context), ~20-30 core-seconds on all cores and a
        # few seconds on one
        rate, n_seq, reps, secs = time_oracle(2.2e9, cores, 20, 1.5)
        out["cpu_baseline"] = {"value": rate, "unit": "GB/s", "cores": cores, "kind": "oracle",
                               "sample": "fp64 oracle, attention of the first %d of %d sequences (all heads, full "
                                         "contexts), %d passes, %.2f s wall" % (n_seq, w.batch, reps, secs)}
        rate1, n1, reps1, secs1 = time_oracle(1.0e9, 1, 1, 0.0)
        out["cpu_baseline"]["single_thread"] = {
            "value": rate1, "unit": "GB/s", "cores": 1,
            "sample": "the first %d sequences, one pass, %.2f s wall" % (n1, secs1)}

    if not args.only:
        del dw
        torch.cuda.empty_cache()
        out["workloads"] = {w.name: {k: head[k] for k in head}}
        n_other = max(10, min(args.steps, 60))
        for name in OTHER_WORKLOADS:
            if name == args.workload:
                continue
            rep, wo, dwo = run_workload(name, n_other, max(3, min(args.warmup, 10)), pools_for(name), args.kernel, cores,
                                        min_seconds=0.05)
            out["workloads"][wo.name] = rep
            del dwo, wo
            torch.cuda.empty_cache()
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
