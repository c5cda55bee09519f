"""Device-side plumbing around the binding: upload a workload, allocate the
partial / output buffers, issue the decode calls and the merge.  No arithmetic
of the method happens here — every step runs in the HIP library."""
from __future__ import annotations

from typing import List, Optional

import numpy as np
import torch

from . import binding
from .workloads import Workload


def to_device(a: np.ndarray, dtype: str, device) -> torch.Tensor:
    """Upload raw bits: uint16 arrays are bf16 patterns, float32 arrays are fp32."""
    if dtype == "bf16":
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)


class DeviceWorkload:
    """A workload resident in HBM plus the buffers one pass of the hot path writes."""

    def __init__(self, w: Workload, device="cuda:0", out_dtype: Optional[str] = None,
                 ext_o: Optional[np.ndarray] = None, ext_lse: Optional[np.ndarray] = None,
                 ext_offsets: Optional[np.ndarray] = None, n_pool_copies: int = 1, workspace: bool = True,
                 mode: str = "merge", pools_from: Optional["DeviceWorkload"] = None):
        """mode: how the final rows come about.
        "merge"  every chunk writes a partial row, omni_merge_partials makes the final rows (a single
                 one-chunk call with nothing else to merge writes them itself);
        "final"  the decode call also writes the final rows of the sequences it can finish (one non-empty
                 chunk), the masked merge does the others;
        "fused"  the decode call finishes every sequence (in-launch merge, external rows folded in).
        pools_from: take q, the pool copies and the block table from that object instead of uploading them
        again (the same batch with other ranges or another chunking)."""
        # workspace: False / 0 none (grid form), True / 1 a workspace whose list every call rebuilds,
        # 2 a workspace prepared once by omni_decode_plan and passed as planned to every call
        self.plan_first = workspace == 2 and workspace is not True
        self._planned = False
        if mode not in ("merge", "final", "fused"):
            raise ValueError("unknown mode %r" % mode)
        if mode != "merge" and len(w.calls) != 1:
            raise ValueError("mode %r needs a workload with one decode call" % mode)
        self.mode = mode
        self.w = w
        self.device = torch.device(device)
        if pools_from is not None:
            self.q, self.k_pools, self.v_pools = pools_from.q, pools_from.k_pools, pools_from.v_pools
            self.block_table = pools_from.block_table
        else:
            k_pool, v_pool, table = w.device_views()
            self.q = to_device(w.q, w.dtype, self.device)
            # several physical copies of the pools let a timing loop defeat cache residency
            self.k_pools = [to_device(k_pool, w.dtype, self.device) for _ in range(n_pool_copies)]
            self.v_pools = [to_device(v_pool, w.dtype, self.device) for _ in range(n_pool_copies)]
            self.block_table = torch.from_numpy(np.ascontiguousarray(table, dtype=np.int32)).to(self.device)
        B, Hq, D = w.batch, w.num_q_heads, w.head_dim
        self.calls = []
        for c in w.calls:
            self.calls.append(dict(
                begin=torch.from_numpy(np.ascontiguousarray(c.ctx_begin, dtype=np.int32)).to(self.device),
                end=torch.from_numpy(np.ascontiguousarray(c.ctx_end, dtype=np.int32)).to(self.device),
                chunk_tokens=c.chunk_tokens, max_chunks=c.max_chunks,
                part_o=torch.empty((B, c.max_chunks, Hq, D), dtype=torch.float32, device=self.device),
                part_lse=torch.empty((B, c.max_chunks, Hq), dtype=torch.float32, device=self.device),
                workspace=torch.zeros(binding.omni_decode_workspace_bytes(B, c.max_chunks, w.num_kv_heads),
                                      dtype=torch.uint8, device=self.device) if workspace else None))
        self.ext = None
        if ext_o is not None:
            self.ext = (torch.from_numpy(np.ascontiguousarray(ext_o, dtype=np.float32)).to(self.device),
                        torch.from_numpy(np.ascontiguousarray(ext_lse, dtype=np.float32)).to(self.device),
                        torch.from_numpy(np.ascontiguousarray(ext_offsets, dtype=np.int32)).to(self.device), 0)
        od = out_dtype or w.out_dtype
        self.out_o = torch.empty((B, Hq, D), dtype=torch.bfloat16 if od == "bf16" else torch.float32,
                                 device=self.device)
        self.out_lse = torch.empty((B, Hq), dtype=torch.float32, device=self.device)
        self.seq_final = torch.zeros(B, dtype=torch.int32, device=self.device)
        self._arg_cache, self._merge_call = {}, None
        # a single one-chunk call with nothing else to merge writes the final rows itself
        self.direct = len(self.calls) == 1 and self.calls[0]["max_chunks"] == 1 and self.ext is None
        if self.direct:
            self.mode = "merge"

    def poison_outputs(self):
        """Fill every output with NaN so that stale data cannot pass a check."""
        for c in self.calls:
            c["part_o"].fill_(float("nan"))
            c["part_lse"].fill_(float("nan"))
        self.out_o.fill_(float("nan"))
        self.out_lse.fill_(float("nan"))

    def decode_args(self, c, kernel: int, pool: int, planned: bool):
        final = self.direct or self.mode != "merge"
        return binding.make_decode_args(
            self.q, self.k_pools[pool], self.v_pools[pool], self.block_table, c["begin"], c["end"],
            sm_scale=self.w.sm_scale, chunk_tokens=c["chunk_tokens"], max_chunks=c["max_chunks"],
            part_o=None if self.direct else c["part_o"], part_lse=None if self.direct else c["part_lse"],
            out_o=self.out_o if final else None, out_lse=self.out_lse if final else None,
            kernel=kernel, workspace=c["workspace"], workspace_planned=planned,
            seq_final=self.seq_final if self.mode != "merge" else None, fuse_merge=self.mode == "fused",
            ext_srcs=[self.ext] if (self.mode != "merge" and self.ext is not None) else None)

    def _args(self, i: int, kernel: int, pool: int, planned: bool):
        """decode_args of call i, marshalled once per combination (the step loops call this every step)."""
        key = (i, kernel, pool, planned, self.mode, id(self.ext))
        a = self._arg_cache.get(key)
        if a is None:
            a = self._arg_cache[key] = self.decode_args(self.calls[i], kernel, pool, planned)
        return a

    def plan(self, stream=None):
        """Build the work list of every decode call once (it can then serve many attention passes)."""
        for i, c in enumerate(self.calls):
            if c["workspace"] is not None:
                binding.omni_decode_plan(self._args(i, binding.OMNI_KERNEL_AUTO, 0, False), stream)

    def run_attention(self, kernel: int = binding.OMNI_KERNEL_AUTO, pool: int = 0, stream=None,
                      planned: bool = False):
        for i in range(len(self.calls)):
            binding.omni_paged_decode_attn_raw(self._args(i, kernel, pool, planned), stream)

    def merge_sources(self) -> List:
        srcs = [self.ext] if self.ext is not None else []
        srcs += [(c["part_o"], c["part_lse"], None, c["max_chunks"]) for c in self.calls]
        return srcs

    def run_merge(self, stream=None):
        if self.direct or self.mode == "fused":
            return
        key = (self.mode, id(self.ext))
        if self._merge_call is None or self._merge_call[0] != key:
            w = self.w
            self._merge_call = (key, binding.PreparedMerge(
                w.batch, w.num_q_heads, w.head_dim, self.merge_sources(),
                self.seq_final if self.mode == "final" else None, self.out_o, self.out_lse))
        self._merge_call[1].run(stream)

    def run(self, kernel: int = binding.OMNI_KERNEL_AUTO, pool: int = 0, stream=None):
        """One pass of the whole hot path: every decode call, then the merge."""
        if self.plan_first and not self._planned:
            self.plan(stream)
            self._planned = True
        self.run_attention(kernel, pool, stream, planned=self.plan_first)
        self.run_merge(stream)

    def abandoned_waves(self) -> int:
        """Diagnostic word of the work lists: waves that gave a launch up (always 0 in a healthy run)."""
        torch.cuda.synchronize(self.device)
        return sum(int(c["workspace"][20:24].view(torch.int32).item()) for c in self.calls if c["workspace"] is not None)

    def results(self):
        torch.cuda.synchronize(self.device)
        return self.out_o.float().cpu().numpy().astype(np.float64), self.out_lse.cpu().numpy().astype(np.float64)
