"""Where the time of a persistent decode launch goes, workgroup by workgroup.

    python3 -m paper_2603_12831_amd.timeline --workload cfg4 [--launches 20]

Runs the workload's decode call through the library's time-stamping kernel instance
(omni_debug_decode_timeline: the plain persistent kernel plus clock stamps, a few per ticket) and prints,
over the launches after a warm-up: when the workgroups start, get their first data and finish (relative to
the earliest start of the launch), how long the launch runs with some workgroups already idle, and how the
time of a ticket compares with the bytes it stands for.  The stamping instance is a little slower than the
plain one (a clock read and a store per ticket); its launch time is printed beside the plain kernel's.
"""
import argparse
import sys

import numpy as np


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="cfg3", choices=["cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--launches", type=int, default=20)
    ap.add_argument("--fused", action="store_true", help="the fused form (the launch finishes every sequence)")
    args = ap.parse_args()
    import torch
    from paper_2603_12831_amd import binding, workloads as wl
    from paper_2603_12831_amd.runner import DeviceWorkload

    if not torch.cuda.is_available():
        print("no GPU visible", file=sys.stderr)
        return 2
    binding.load_library()
    w = wl.MAKERS[args.workload](workers=16)
    ext = {}
    if w.ext_ranges is not None:                       # only the row counts matter here
        off = wl.ext_row_offsets(w)
        n = int(off[-1])
        ext = dict(ext_o=np.zeros((n, w.num_q_heads, w.head_dim), np.float32),
                   ext_lse=np.zeros((n, w.num_q_heads), np.float32), ext_offsets=off)
    pools = 4 if args.workload == "cfg4" else 2
    dw = DeviceWorkload(w, n_pool_copies=pools, mode="fused" if args.fused else ("final" if len(w.calls) == 1 else "merge"),
                        **ext)
    n_wg, words = binding.omni_debug_decode_timeline_shape()
    stamps = torch.zeros(n_wg * words, dtype=torch.int64, device="cuda")
    dw.plan()
    recs, t_timed, t_plain = [], [], []
    for i in range(args.launches + 5):
        a = dw.decode_args(dw.calls[0], binding.OMNI_KERNEL_AUTO, i % pools, True)
        stamps.zero_()
        e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        e0.record()
        binding.omni_debug_decode_timeline(a, stamps)
        e1.record()
        binding.omni_paged_decode_attn_raw(a)
        e2.record()
        torch.cuda.synchronize()
        if i >= 5:
            recs.append(stamps.cpu().numpy().reshape(n_wg, words).astype(np.float64) * 0.01)      # -> microseconds
            t_timed.append(e0.elapsed_time(e1) * 1e3)
            t_plain.append(e1.elapsed_time(e2) * 1e3)
    r = np.stack(recs)                                 # [launch, workgroup, word] in us (counts scaled too)
    active = r[:, :, 2] > 0
    t0 = np.where(r[:, :, 0] > 0, r[:, :, 0], np.inf).min(axis=1)[:, None]
    start, first, stream_end, writer_end = (np.where(active, r[:, :, k] - t0, np.nan) for k in range(4))
    tickets, steps = r[:, :, 4] * 100, r[:, :, 5] * 100
    end = np.nanmax(writer_end, axis=1)

    def q(x, qs=(0, 10, 50, 90, 100)):
        return " ".join("%7.2f" % v for v in np.nanpercentile(x, qs))

    print("%s%s: %d launches, %d workgroups (%d with work); events: stamping instance %.2f us, plain kernel %.2f us"
          % (w.name, " (fused form)" if args.fused else "", len(recs), n_wg, int(active[0].sum()), float(np.median(t_timed)), float(np.median(t_plain))))
    print("  times in us after the launch's earliest workgroup start; percentiles over workgroups and launches")
    print("                                 min     p10     p50     p90     max")
    print("  workgroup start            %s" % q(start))
    print("  first query rows in LDS    %s" % q(first))
    print("  streaming waves done       %s" % q(stream_end))
    print("  last store done            %s" % q(writer_end))
    print("  launch end (last workgroup done), median over launches: %.2f us" % float(np.median(end)))
    idle = (end[:, None] - writer_end)
    print("  idle before the launch's end, per workgroup: mean %.2f us, p50 %.2f, p90 %.2f, max %.2f  "
          "(mean idle / launch = %.1f %%)" % (float(np.nanmean(idle)), float(np.nanpercentile(idle, 50)),
                                             float(np.nanpercentile(idle, 90)), float(np.nanmax(idle)),
                                             100.0 * float(np.nanmean(idle)) / float(np.median(end))))
    for frac in (0.5, 0.25, 0.1):
        t = np.array([np.sort(writer_end[i][active[i]])[::-1][max(int(frac * active[i].sum()) - 1, 0)] for i in range(len(recs))])
        print("  %3.0f %% of the workgroups are still at work until %.2f us (median over launches)"
              % (100 * frac, float(np.median(t))))
    print("  tickets per workgroup      %s" % q(np.where(active, tickets, np.nan)))
    print("  32-token steps of wave 0   %s" % q(np.where(active, steps, np.nan)))
    # per-ticket durations (first launch kept): meeting k minus meeting k-1 (ticket 0: minus first data)
    kmax = words - 8
    meet = np.where(r[:, :, 8:] > 0, r[:, :, 8:] - t0[:, :, None], np.nan)
    dur = np.diff(np.concatenate([first[:, :, None], meet], axis=2), axis=2)
    print("  time from one meeting of the workgroup to the next, by position of the ticket in the workgroup:")
    for k in range(min(kmax, 8)):
        if np.isfinite(dur[:, :, k]).any():
            print("    ticket %d: n %5d  %s" % (k, int(np.isfinite(dur[:, :, k]).sum()), q(dur[:, :, k])))
    return 0


if __name__ == "__main__":
    sys.exit(main())
