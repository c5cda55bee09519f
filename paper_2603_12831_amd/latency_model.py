"""Decode-attention latency model of the paper's Profiler, fitted on this library's kernels.

The paper models the latency of decode attention as linear in the decode load and in the number of
decoding requests (latency-model section, the decode-attention equation):

    f_DA(c_DA, g) = a * c_DA + h * g + b,      c_DA = sum over decoding requests of (l_j + 1),

fits the coefficients by linear regression on profiled samples and reports the accuracy of the fit
(its accuracy table: average and P90).  Here c_DA is the sum of the context lengths this library is
given (they already count the current token) and the latency is that of the whole hot path on the
GPU: work list, paged decode attention, merge.

    python -m paper_2603_12831_amd.latency_model [--samples 60] [--seed 0] [--out file.json]

measures seeded synthetic batches on the GPU, fits on the first 70 % and reports accuracy on the rest.
"""
from __future__ import annotations

import argparse
import json
import sys
from typing import Dict, Sequence

import numpy as np


def fit(c_da: Sequence[float], g: Sequence[float], t: Sequence[float]) -> Dict[str, float]:
    """Least-squares coefficients (a, h, b) of t ~ a * c_da + h * g + b."""
    c = np.asarray(c_da, dtype=np.float64)
    n = np.asarray(g, dtype=np.float64)
    y = np.asarray(t, dtype=np.float64)
    if not (c.shape == n.shape == y.shape) or c.ndim != 1 or c.size < 3:
        raise ValueError("need three equally long 1-D sample arrays with at least 3 samples")
    design = np.stack([c, n, np.ones_like(c)], axis=1)
    coef, _, rank, _ = np.linalg.lstsq(design, y, rcond=None)
    if rank < 3:
        raise ValueError("samples do not determine the three coefficients (rank %d)" % rank)
    return {"a": float(coef[0]), "h": float(coef[1]), "b": float(coef[2])}


def predict(model: Dict[str, float], c_da, g) -> np.ndarray:
    return model["a"] * np.asarray(c_da, dtype=np.float64) + model["h"] * np.asarray(g, dtype=np.float64) + model["b"]


def accuracy(pred, meas) -> Dict[str, float]:
    """Per-sample accuracy 1 - |pred - meas| / meas; its mean, and the level 90 % of the samples reach."""
    p = np.asarray(pred, dtype=np.float64)
    m = np.asarray(meas, dtype=np.float64)
    acc = 1.0 - np.abs(p - m) / m
    return {"avg": float(acc.mean()), "p90": float(np.percentile(acc, 10.0)), "min": float(acc.min())}


def sample_batches(seed: int, n: int, max_tokens: int = 600_000, max_batch: int = 512):
    """Seeded decode batches: request count g uniform in [4, max_batch], context lengths lognormal around
    a per-batch median drawn log-uniformly from [128, 4096], clipped to [1, 8192], total capped."""
    rng = np.random.default_rng([seed, 77])
    out = []
    for _ in range(n):
        g = int(rng.integers(4, max_batch + 1))
        median = float(np.exp(rng.uniform(np.log(128.0), np.log(4096.0))))
        lengths = np.clip(np.rint(np.exp(np.log(median) + 0.6 * rng.standard_normal(g))), 1, 8192).astype(np.int32)
        while int(lengths.sum()) > max_tokens:
            lengths = lengths[: max(4, len(lengths) // 2)]
        out.append(lengths)
    return out


def measure(samples, reps: int = 7, hq: int = 32, hkv: int = 8, chunk_tokens: int = 1024, device="cuda:0"):
    """Median latency (ms) of list + decode attention + merge for each batch, on one shared page pool."""
    import torch
    from . import binding

    dev = torch.device(device)
    bs, d = 16, 128
    pool_pages = max(int(((s.astype(np.int64) + bs - 1) // bs).sum()) for s in samples)
    k_pool = torch.randn(pool_pages, hkv, bs, d, device=dev).bfloat16()
    v_pool = torch.randn(pool_pages, hkv, bs, d, device=dev).bfloat16()
    rng = np.random.default_rng(5)
    times = []
    for lengths in samples:
        B = len(lengths)
        need = (lengths.astype(np.int64) + bs - 1) // bs
        max_blocks = int(need.max())
        perm = rng.permutation(pool_pages).astype(np.int32)
        table = np.full((B, max_blocks), -1, dtype=np.int32)
        pos = 0
        for i, nb in enumerate(need):
            table[i, :nb] = perm[pos:pos + nb]
            pos += int(nb)
        max_chunks = int((int(lengths.max()) + chunk_tokens - 1) // chunk_tokens)
        q = torch.randn(B, hq, d, device=dev).bfloat16()
        bt = torch.from_numpy(table).to(dev)
        end = torch.from_numpy(lengths.astype(np.int32)).to(dev)
        part_o = torch.empty((B, max_chunks, hq, d), dtype=torch.float32, device=dev)
        part_lse = torch.empty((B, max_chunks, hq), dtype=torch.float32, device=dev)
        out_o = torch.empty((B, hq, d), dtype=torch.bfloat16, device=dev)
        out_lse = torch.empty((B, hq), dtype=torch.float32, device=dev)
        ws = torch.empty(binding.omni_decode_workspace_bytes(B, max_chunks, hkv), dtype=torch.uint8, device=dev)

        def once():
            binding.omni_paged_decode_attn(q, k_pool, v_pool, bt, None, end, sm_scale=d ** -0.5,
                                           chunk_tokens=chunk_tokens, max_chunks=max_chunks, part_o=part_o,
                                           part_lse=part_lse, workspace=ws)
            binding.omni_merge_partials(B, hq, d, [(part_o, part_lse, None, max_chunks)], out_o, out_lse)

        once()
        ts = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            once()
            e1.record()
            e1.synchronize()
            ts.append(e0.elapsed_time(e1))
        times.append(float(np.median(ts)))
    return np.array(times)


def profile_and_fit(n_samples: int = 60, seed: int = 0, train_frac: float = 0.7, keep_samples: bool = False,
                    **kw) -> Dict:
    samples = sample_batches(seed, n_samples)
    t = measure(samples, **kw)
    c = np.array([int(s.sum()) for s in samples], dtype=np.float64)
    g = np.array([len(s) for s in samples], dtype=np.float64)
    n_train = max(3, int(round(train_frac * n_samples)))
    model = fit(c[:n_train], g[:n_train], t[:n_train])
    held = slice(n_train, None) if n_train < n_samples else slice(0, None)
    extra = {"samples": {"c_da": c.tolist(), "g": g.tolist(), "ms": t.tolist()}} if keep_samples else {}
    return {**extra, "model_ms": model, "train_samples": n_train, "test_samples": int(len(c[held])),
            "accuracy_train": accuracy(predict(model, c[:n_train], g[:n_train]), t[:n_train]),
            "accuracy_test": accuracy(predict(model, c[held], g[held]), t[held]),
            "ns_per_context_token": model["a"] * 1e6, "us_per_request": model["h"] * 1e3,
            "us_fixed": model["b"] * 1e3,
            "implied_kv_GBps": 2 * kw.get("hkv", 8) * 128 * 2 / (model["a"] * 1e-3) / 1e9,
            "c_da_range": [float(c.min()), float(c.max())], "g_range": [float(g.min()), float(g.max())]}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--samples", type=int, default=60)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--out", default=None)
    ap.add_argument("--keep-samples", action="store_true", help="include the measured (c_DA, g, ms) samples")
    args = ap.parse_args()
    res = profile_and_fit(args.samples, args.seed, keep_samples=args.keep_samples)
    line = json.dumps(res)
    print(line)
    if args.out:
        with open(args.out, "w") as f:
            f.write(line + "\n")
    return 0


if __name__ == "__main__":
    sys.exit(main())
