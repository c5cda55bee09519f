"""Seeded synthetic inputs for paged decode attention and partial merging.

This module only *lays out data*: random values, bf16 bit patterns, page pools,
block tables, context ranges and chunk plans.  It contains none of the
attention or merge arithmetic, so the CPU oracle and the HIP path can both be
fed from it without sharing any of the method's code.

The shapes stand in for the serving loads the paper measures on (chat-length
latency-sensitive requests and long-document best-effort requests, evaluation
section: bf16 models, contexts from about one thousand to twelve thousand
tokens); no item of any dataset is reproduced, only length statistics.

bf16 tensors are carried on the host as ``uint16`` bit patterns (numpy has no
bf16).  Values are drawn in fp32 and rounded to bf16 once, round-to-nearest-
even, so every consumer sees the identical bits.
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

BLOCK_SIZE = 16


# ----------------------------------------------------------------------------
# representation helpers (format conversion only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal(shape, seed_seq, scale: float, dtype: str, workers: int = 8,
            boost_frac: float = 0.0, boost: float = 1.0) -> np.ndarray:
    """N(0, scale^2) tensor, generated in row slabs by independent child
    streams of ``seed_seq`` (the result does not depend on ``workers``).

    If ``boost_frac`` > 0 the tensor is viewed as rows of its last axis and a
    Bernoulli(boost_frac) subset of rows is multiplied by ``boost``.
    """
    shape = tuple(int(s) for s in shape)
    out = np.empty(shape, dtype=np.float32 if dtype == "f32" else np.uint16)
    n0 = shape[0]
    row_elems = int(np.prod(shape[1:])) if len(shape) > 1 else 1
    slab = max(1, (1 << 22) // max(1, row_elems))          # ~4M values per slab
    starts = list(range(0, n0, slab))
    children = np.random.SeedSequence(seed_seq).spawn(len(starts)) if starts else []

    def work(j):
        lo = starts[j]
        hi = min(n0, lo + slab)
        rng = np.random.default_rng(children[j])
        x = rng.standard_normal((hi - lo,) + shape[1:], dtype=np.float32)
        if scale != 1.0:
            x *= np.float32(scale)
        if boost_frac > 0.0:
            pick = rng.random(x.shape[:-1]) < boost_frac
            x[pick] *= np.float32(boost)
        out[lo:hi] = x if dtype == "f32" else f32_to_bf16_bits(x)

    if len(starts) <= 1 or workers <= 1:
        for j in range(len(starts)):
            work(j)
    else:
        with ThreadPoolExecutor(max_workers=workers) as ex:
            list(ex.map(work, range(len(starts))))
    return out


# ----------------------------------------------------------------------------
# workload container
# ----------------------------------------------------------------------------
@dataclass
class DecodeCall:
    """One call of the decode-attention entry point: per-sequence token range
    [ctx_begin, ctx_end) cut into chunks of ``chunk_tokens`` (0 = one chunk)."""
    ctx_begin: np.ndarray            # int32 [B]
    ctx_end: np.ndarray              # int32 [B]
    chunk_tokens: int
    max_chunks: int


@dataclass
class Workload:
    name: str
    batch: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    block_size: int
    dtype: str                       # "f32" | "bf16" : dtype of q / k_pool / v_pool
    out_dtype: str                   # dtype of the final O the config asks for
    sm_scale: float
    q: np.ndarray                    # [B, Hq, D]
    k_pool: np.ndarray               # [num_blocks, Hkv, bs, D]  (full logical contexts)
    v_pool: np.ndarray
    block_table: np.ndarray          # int32 [B, max_blocks], -1 = no page
    ctx_len: np.ndarray              # int32 [B] full context length (current token included)
    calls: List[DecodeCall]
    # pages resident on the GPU, if they differ from the full pool (hybrid batch)
    dev_k_pool: Optional[np.ndarray] = None
    dev_v_pool: Optional[np.ndarray] = None
    dev_block_table: Optional[np.ndarray] = None
    # externally produced partials: per sequence a list of [begin, end) token ranges
    ext_ranges: Optional[List[List[tuple]]] = None
    meta: Dict = field(default_factory=dict)

    @property
    def num_blocks(self) -> int:
        return int(self.k_pool.shape[0])

    @property
    def max_blocks_per_seq(self) -> int:
        return int(self.block_table.shape[1])

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def kv_bytes(self) -> int:
        """KV bytes one pass of all decode calls must read."""
        tok = sum(int(np.maximum(c.ctx_end.astype(np.int64) - c.ctx_begin, 0).sum()) for c in self.calls)
        return tok * 2 * self.num_kv_heads * self.head_dim * self.elem_bytes

    def device_views(self):
        if self.dev_k_pool is None:
            return self.k_pool, self.v_pool, self.block_table
        return self.dev_k_pool, self.dev_v_pool, self.dev_block_table


def _assign_pages(rng, lengths, num_blocks: int, block_size: int, max_blocks: Optional[int] = None):
    """Give every sequence ceil(L/bs) distinct pages taken from one random
    permutation of the pool; unused table entries are -1."""
    need = [(int(L) + block_size - 1) // block_size for L in lengths]
    total = sum(need)
    if total > num_blocks:
        raise ValueError("pool too small: need %d pages, have %d" % (total, num_blocks))
    perm = rng.permutation(num_blocks).astype(np.int32)
    mb = max(need + [1]) if max_blocks is None else max_blocks
    table = np.full((len(lengths), mb), -1, dtype=np.int32)
    pos = 0
    for i, n in enumerate(need):
        table[i, :n] = perm[pos:pos + n]
        pos += n
    return table


def _single_call(lengths, chunk_tokens: int) -> DecodeCall:
    lengths = np.asarray(lengths, dtype=np.int32)
    if chunk_tokens:
        max_chunks = max(1, int((int(lengths.max(initial=1)) + chunk_tokens - 1) // chunk_tokens))
    else:
        max_chunks = 1
    return DecodeCall(np.zeros_like(lengths), lengths.copy(), int(chunk_tokens), max_chunks)


def make_generic(seed: int, lengths, num_q_heads: int, num_kv_heads: int, head_dim: int,
                 dtype: str = "bf16", chunk_tokens: int = 0, pool_factor: float = 1.0,
                 value_scale: float = 1.0, sm_scale: Optional[float] = None,
                 out_dtype: str = "f32", name: str = "generic", ctx_begin=None,
                 boost_frac: float = 0.0, boost: float = 1.0, workers: int = 8) -> Workload:
    """Arbitrary ragged batch with the common recipe (used by the edge-case tests)."""
    lengths = np.asarray(lengths, dtype=np.int32)
    B = len(lengths)
    bs = BLOCK_SIZE
    rng = np.random.default_rng([seed, 0])
    need = int(sum((int(L) + bs - 1) // bs for L in lengths))
    num_blocks = max(1, int(math.ceil(need * pool_factor)))
    table = _assign_pages(rng, lengths, num_blocks, bs)
    q = _normal((B, num_q_heads, head_dim), [seed, 1], value_scale, dtype, workers)
    k = _normal((num_blocks, num_kv_heads, bs, head_dim), [seed, 2], value_scale, dtype, workers,
                boost_frac=boost_frac, boost=boost)
    v = _normal((num_blocks, num_kv_heads, bs, head_dim), [seed, 3], value_scale, dtype, workers)
    call = _single_call(lengths, chunk_tokens)
    if ctx_begin is not None:
        call.ctx_begin = np.asarray(ctx_begin, dtype=np.int32)
    return Workload(name=name, batch=B, num_q_heads=num_q_heads, num_kv_heads=num_kv_heads,
                    head_dim=head_dim, block_size=bs, dtype=dtype, out_dtype=out_dtype,
                    sm_scale=float(1.0 / math.sqrt(head_dim) if sm_scale is None else sm_scale),
                    q=q, k_pool=k, v_pool=v, block_table=table, ctx_len=lengths.copy(), calls=[call])


# ----------------------------------------------------------------------------
# the five named configurations
# ----------------------------------------------------------------------------
def make_cfg1(seed: int = 1) -> Workload:
    """Tiny fp32 GQA case: B4, 8 q heads / 2 kv heads, D64, contexts
    {17,100,256,511}; every sequence is cut into two chunks at a page-aligned
    point near its middle (two decode calls with explicit ranges), merged."""
    lengths = np.array([17, 100, 256, 511], dtype=np.int32)
    w = make_generic(seed, lengths, 8, 2, 64, dtype="f32", name="cfg1-tiny-f32")
    bs = w.block_size
    cut = np.array([bs * (((int(L) + 1) // 2 + bs - 1) // bs) for L in lengths], dtype=np.int32)
    cut = np.minimum(cut, lengths)
    zeros = np.zeros_like(lengths)
    w.calls = [DecodeCall(zeros, cut.copy(), 0, 1), DecodeCall(cut.copy(), lengths.copy(), 0, 1)]
    w.meta["cut"] = cut
    return w


def make_cfg2(seed: int = 2, batch: int = 64, lo: int = 512, hi: int = 4096, workers: int = 8) -> Workload:
    """7B-shaped MHA step: 32 q = 32 kv heads, D128, bf16, values N(0,1)/sqrt(128),
    contexts uniform in [lo, hi], pages scattered over a pool twice the needed
    size, one chunk per sequence, bf16 O + fp32 LSE."""
    rng = np.random.default_rng([seed, 9])
    lengths = rng.integers(lo, hi + 1, size=batch).astype(np.int32)
    return make_generic(seed, lengths, 32, 32, 128, dtype="bf16", chunk_tokens=0, pool_factor=2.0,
                        value_scale=1.0 / math.sqrt(128.0), out_dtype="bf16",
                        name="cfg2-mha-b%d" % batch, workers=workers)


def lognormal_lengths(rng, n: int, median: float, sigma: float, lo: int, hi: int) -> np.ndarray:
    x = np.exp(math.log(median) + sigma * rng.standard_normal(n))
    return np.clip(np.rint(x), lo, hi).astype(np.int32)


def make_cfg3(seed: int = 3, batch: int = 256, median: float = 1500.0, sigma: float = 0.8,
              lo: int = 64, hi: int = 8192, chunk_tokens: int = 1024, workers: int = 8) -> Workload:
    """8B-shaped GQA step: 32 q / 8 kv heads, D128, bf16 N(0,1), contexts
    lognormal(median 1500, sigma 0.8 in ln-space) clipped to [64, 8192], shuffled
    pool, split-KV chunks of 1024 tokens, then merge."""
    rng = np.random.default_rng([seed, 9])
    lengths = lognormal_lengths(rng, batch, median, sigma, lo, hi)
    return make_generic(seed, lengths, 32, 8, 128, dtype="bf16", chunk_tokens=chunk_tokens,
                        out_dtype="bf16", name="cfg3-gqa-b%d" % batch, workers=workers)


def make_cfg5(seed: int = 5, batch: int = 32, ctx: int = 32768, chunk_tokens: int = 1024,
              workers: int = 8) -> Workload:
    """Long-context 70B-layer shape: 64 q / 8 kv heads, D128, bf16, every context
    ``ctx`` tokens, permuted pages, chunks of 1024, 1% of key rows scaled x8."""
    lengths = np.full(batch, ctx, dtype=np.int32)
    return make_generic(seed, lengths, 64, 8, 128, dtype="bf16", chunk_tokens=chunk_tokens,
                        out_dtype="bf16", name="cfg5-long-b%d-L%d" % (batch, ctx),
                        boost_frac=0.01, boost=8.0, workers=workers)


def make_cfg4(seed: int = 4, n_ls: int = 32, n_be: int = 224, ls_lo: int = 256, ls_hi: int = 2048,
              be_lo: int = 1024, be_hi: int = 4096, tail_lo: int = 64, tail_hi: int = 256,
              workers: int = 8) -> Workload:
    """Hybrid piggyback batch (32 q / 8 kv heads, D128, bf16 N(0,1)).

    Rows [0, n_ls) are latency-sensitive: whole context in GPU pages.
    Rows [n_ls, n_ls+n_be) are best-effort: full context L ~ U[be_lo, be_hi];
    only the last ``tail`` ~ U{tail_lo..tail_hi} tokens are in GPU pages (the
    tail start is not page aligned); the prefix [0, L-tail) is cut into
    1..4 near-equal contiguous pieces whose partial O / LSE are produced off
    the GPU (``ext_ranges``).  ``k_pool``/``block_table`` hold every token (the
    view a full-context check needs); ``dev_*`` hold only the resident pages,
    renumbered into their own shuffled pool.
    """
    rng = np.random.default_rng([seed, 9])
    bs = BLOCK_SIZE
    B = n_ls + n_be
    ls_len = rng.integers(ls_lo, ls_hi + 1, size=n_ls)
    be_len = rng.integers(be_lo, be_hi + 1, size=n_be)
    tail = rng.integers(tail_lo, tail_hi + 1, size=n_be)
    tail = np.minimum(tail, be_len)
    n_ext = rng.integers(1, 5, size=n_be)
    lengths = np.concatenate([ls_len, be_len]).astype(np.int32)
    w = make_generic(seed, lengths, 32, 8, 128, dtype="bf16", out_dtype="bf16",
                     name="cfg4-hybrid-%dls-%dbe" % (n_ls, n_be), workers=workers)
    begin = np.zeros(B, dtype=np.int32)
    begin[n_ls:] = (be_len - tail).astype(np.int32)
    w.calls = [DecodeCall(begin, lengths.copy(), 0, 1)]
    ext: List[List[tuple]] = [[] for _ in range(B)]
    for j in range(n_be):
        prefix = int(be_len[j] - tail[j])
        n = int(n_ext[j])
        cuts = [(prefix * p) // n for p in range(n + 1)]
        ext[n_ls + j] = [(cuts[p], cuts[p + 1]) for p in range(n)]
    w.ext_ranges = ext
    # resident pages: logical page indices touched by [begin, end)
    first_pg = begin // bs
    last_pg = (lengths + bs - 1) // bs
    n_res = int((last_pg - first_pg).sum())
    perm = rng.permutation(n_res).astype(np.int32)
    dev_table = np.full_like(w.block_table, -1)
    src = np.empty(n_res, dtype=np.int64)
    pos = 0
    for i in range(B):
        n = int(last_pg[i] - first_pg[i])
        dev_table[i, first_pg[i]:last_pg[i]] = perm[pos:pos + n]
        src[perm[pos:pos + n]] = w.block_table[i, first_pg[i]:last_pg[i]]
        pos += n
    w.dev_k_pool = w.k_pool[src]
    w.dev_v_pool = w.v_pool[src]
    w.dev_block_table = dev_table
    w.meta.update(n_ls=n_ls, n_be=n_be, tail=tail.astype(np.int32), n_ext=n_ext.astype(np.int32))
    return w


def ext_row_offsets(w: Workload) -> np.ndarray:
    """CSR offsets [B+1] of the external partial rows of a hybrid workload."""
    counts = np.array([len(r) for r in (w.ext_ranges or [[]] * w.batch)], dtype=np.int32)
    off = np.zeros(w.batch + 1, dtype=np.int32)
    np.cumsum(counts, out=off[1:])
    return off


MAKERS = {"cfg1": make_cfg1, "cfg2": make_cfg2, "cfg3": make_cfg3, "cfg4": make_cfg4, "cfg5": make_cfg5}
