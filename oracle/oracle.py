"""ctypes front end of the CPU fp64 oracle (``oracle_attn.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, the smoke check and the
CPU-baseline leg of the benchmark.  It shares no code with the GPU library and
never imports it.  Operation definitions and citations are in the C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle_attn.c")
_LIB = os.path.join(_HERE, "liboracle_attn.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 (OpenMP only spreads independent work items)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        vp, i32, i64, dbl = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_double
        lib.oracle_paged_attn.argtypes = [i32, i32, i32, i32, i32, i32, dbl, vp, vp, vp, vp, i64, vp,
                                          vp, vp, i32]
        lib.oracle_paged_attn.restype = i32
        lib.oracle_merge.argtypes = [i64, i32, vp, vp, vp, vp, vp]
        lib.oracle_merge.restype = None
        lib.oracle_gather_kv.argtypes = [i32, i32, i32, i32, i32, vp, vp, vp, i32, i32, i32, vp, vp]
        lib.oracle_gather_kv.restype = None
        lib.oracle_queue_push.argtypes = [vp, vp, vp, i32, i32, vp, vp, i32]
        lib.oracle_queue_push.restype = i32
        lib.oracle_queue_pop.argtypes = [vp, vp, vp, i32, i32, vp, vp, i32]
        lib.oracle_queue_pop.restype = i32
        lib.oracle_store_rows.argtypes = [vp, i64, i32, vp, i32, vp, i32]
        lib.oracle_store_rows.restype = None
        lib.oracle_kv_append.argtypes = [i32, i32, i32, i32, i32, i64, i32, vp, vp, vp, vp, vp, vp]
        lib.oracle_kv_append.restype = None
        lib.oracle_kv_pages.argtypes = [i32, i32, i32, i64, i32, vp, vp, vp, i64, vp, vp, i32]
        lib.oracle_kv_pages.restype = None
        _lib = lib
    return _lib


def _ptr(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data)


def _check_pool(q, k_pool, v_pool, dtype):
    want = np.float32 if dtype == "f32" else np.uint16
    for a in (q, k_pool, v_pool):
        if a.dtype != want or not a.flags.c_contiguous:
            raise ValueError("oracle expects C-contiguous %s arrays" % np.dtype(want).name)


def paged_attn_items(q, k_pool, v_pool, block_table, items, sm_scale: float, dtype: str,
                     n_threads: int = 1):
    """Partial attention for explicit work items.

    items: int array [n, 4] of (sequence, query head, begin, end).
    Returns (O [n, D] float64, LSE [n] float64).
    """
    _check_pool(q, k_pool, v_pool, dtype)
    lib = _load()
    items = np.ascontiguousarray(items, dtype=np.int32).reshape(-1, 4)
    bt = np.ascontiguousarray(block_table, dtype=np.int32)
    _, hq, d = q.shape
    _, hkv, bs, _ = k_pool.shape
    n = items.shape[0]
    # host-side bounds check: every touched table entry must name a pool page
    for seq, _h, b, e in items:
        if e > b:
            pages = bt[seq, b // bs:(e + bs - 1) // bs]
            if b < 0 or (e + bs - 1) // bs > bt.shape[1] or pages.min() < 0 or pages.max() >= k_pool.shape[0]:
                raise ValueError("work item reads outside the block table / pool")
    o = np.empty((n, d), dtype=np.float64)
    lse = np.empty((n,), dtype=np.float64)
    rc = lib.oracle_paged_attn(hq, hkv, d, bs, bt.shape[1], 0 if dtype == "f32" else 1,
                               float(sm_scale), _ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(bt),
                               n, _ptr(items), _ptr(o), _ptr(lse), int(n_threads))
    if rc != 0:
        raise MemoryError("oracle_paged_attn failed")
    return o, lse


def paged_attn(q, k_pool, v_pool, block_table, begin, end, sm_scale: float, dtype: str,
               seqs: Optional[Sequence[int]] = None, heads: Optional[Sequence[int]] = None,
               n_threads: int = 1):
    """Attention of every (sequence in ``seqs``, head in ``heads``) over tokens
    [begin[i], end[i]).  Returns (O [len(seqs), len(heads), D], LSE [len(seqs), len(heads)])."""
    B, hq, d = q.shape
    seqs = np.arange(B) if seqs is None else np.asarray(seqs)
    heads = np.arange(hq) if heads is None else np.asarray(heads)
    begin = np.zeros(B, dtype=np.int32) if begin is None else np.asarray(begin)
    end = np.asarray(end)
    items = np.empty((len(seqs), len(heads), 4), dtype=np.int32)
    items[:, :, 0] = seqs[:, None]
    items[:, :, 1] = heads[None, :]
    items[:, :, 2] = begin[seqs][:, None]
    items[:, :, 3] = end[seqs][:, None]
    o, lse = paged_attn_items(q, k_pool, v_pool, block_table, items, sm_scale, dtype, n_threads)
    return o.reshape(len(seqs), len(heads), d), lse.reshape(len(seqs), len(heads))


def merge(part_o, part_lse, offsets):
    """Merge partial rows (CSR ``offsets`` [n_rows+1]) -> (O [n_rows, D], LSE [n_rows])."""
    lib = _load()
    po = np.ascontiguousarray(part_o, dtype=np.float64)
    pl = np.ascontiguousarray(part_lse, dtype=np.float64)
    off = np.ascontiguousarray(offsets, dtype=np.int64)
    n_rows = off.shape[0] - 1
    d = po.shape[-1]
    po = po.reshape(-1, d)
    if off[0] != 0 or off[-1] > po.shape[0] or np.any(np.diff(off) < 0) or pl.size != po.shape[0]:
        raise ValueError("bad CSR offsets")
    o = np.empty((n_rows, d), dtype=np.float64)
    lse = np.empty((n_rows,), dtype=np.float64)
    lib.oracle_merge(n_rows, d, _ptr(off), _ptr(po), _ptr(pl), _ptr(o), _ptr(lse))
    return o, lse


def gather_kv(k_pool, v_pool, block_table, seq: int, begin: int, end: int):
    """Rows of logical tokens [begin, end) of one sequence: ([n, Hkv, D], [n, Hkv, D]), raw dtype."""
    lib = _load()
    bt = np.ascontiguousarray(block_table, dtype=np.int32)
    _, hkv, bs, d = k_pool.shape
    n = max(0, end - begin)
    if n and (begin < 0 or (end + bs - 1) // bs > bt.shape[1]
              or bt[seq, begin // bs:(end + bs - 1) // bs].min() < 0
              or bt[seq, begin // bs:(end + bs - 1) // bs].max() >= k_pool.shape[0]):
        raise ValueError("gather reads outside the block table / pool")
    k_out = np.empty((n, hkv, d), dtype=k_pool.dtype)
    v_out = np.empty((n, hkv, d), dtype=v_pool.dtype)
    if n:
        lib.oracle_gather_kv(hkv, d, bs, bt.shape[1], k_pool.dtype.itemsize, _ptr(k_pool), _ptr(v_pool),
                             _ptr(bt), int(seq), int(begin), int(end), _ptr(k_out), _ptr(v_out))
    return k_out, v_out


def kv_append(k_pool, v_pool, block_table, k_new, v_new, positions):
    """In-place append of one token per sequence into writable pool arrays (see the C file)."""
    lib = _load()
    nb, hkv, bs, d = k_pool.shape
    bt = np.ascontiguousarray(block_table, dtype=np.int32)
    pos = np.ascontiguousarray(positions, dtype=np.int32)
    for a in (k_pool, v_pool, k_new, v_new):
        if not a.flags.c_contiguous or a.dtype != k_pool.dtype:
            raise ValueError("contiguous arrays of one dtype expected")
    if k_new.shape != (bt.shape[0], hkv, d) or v_new.shape != k_new.shape or pos.shape != (bt.shape[0],):
        raise ValueError("bad shapes")
    lib.oracle_kv_append(bt.shape[0], hkv, d, bs, bt.shape[1], nb, k_pool.dtype.itemsize, _ptr(k_pool), _ptr(v_pool),
                         _ptr(bt), _ptr(k_new), _ptr(v_new), _ptr(pos))


def kv_gather_pages(k_pool, v_pool, page_ids):
    lib = _load()
    nb, hkv, bs, d = k_pool.shape
    ids = np.ascontiguousarray(page_ids, dtype=np.int32)
    k_out = np.empty((len(ids), hkv, bs, d), dtype=k_pool.dtype)
    v_out = np.empty_like(k_out)
    lib.oracle_kv_pages(hkv, d, bs, nb, k_pool.dtype.itemsize, _ptr(k_pool), _ptr(v_pool), _ptr(ids), len(ids),
                        _ptr(k_out), _ptr(v_out), 0)
    return k_out, v_out


def kv_scatter_pages(k_pool, v_pool, page_ids, k_in, v_in):
    lib = _load()
    nb, hkv, bs, d = k_pool.shape
    ids = np.ascontiguousarray(page_ids, dtype=np.int32)
    k_in = np.ascontiguousarray(k_in, dtype=k_pool.dtype)
    v_in = np.ascontiguousarray(v_in, dtype=k_pool.dtype)
    if k_in.shape != (len(ids), hkv, bs, d) or v_in.shape != k_in.shape:
        raise ValueError("bad staging shape")
    lib.oracle_kv_pages(hkv, d, bs, nb, k_pool.dtype.itemsize, _ptr(k_pool), _ptr(v_pool), _ptr(ids), len(ids),
                        _ptr(k_in), _ptr(v_in), 1)


class Queue:
    """Host model of a row queue: ring [capacity, row_bytes] uint8, int32 tags, uint32 state words."""

    def __init__(self, capacity: int, row_bytes: int):
        self.data = np.zeros((capacity, row_bytes), dtype=np.uint8)
        self.tags = np.zeros(capacity, dtype=np.int32)
        self.state = np.zeros(4, dtype=np.uint32)

    def push(self, rows: np.ndarray, tags=None) -> int:
        rows = np.ascontiguousarray(rows, dtype=np.uint8).reshape(-1, self.data.shape[1])
        t = None if tags is None else np.ascontiguousarray(tags, dtype=np.int32)
        return _load().oracle_queue_push(_ptr(self.data), _ptr(self.tags), _ptr(self.state), self.data.shape[0],
                                         self.data.shape[1], _ptr(rows), None if t is None else _ptr(t), rows.shape[0])

    def pop(self, max_rows: int):
        rows = np.zeros((max_rows, self.data.shape[1]), dtype=np.uint8)
        tags = np.zeros(max_rows, dtype=np.int32)
        n = _load().oracle_queue_pop(_ptr(self.data), _ptr(self.tags), _ptr(self.state), self.data.shape[0],
                                     self.data.shape[1], _ptr(rows), _ptr(tags), max_rows)
        return rows[:n], tags[:n]


def store_save(store: np.ndarray, slot_ids, rows: np.ndarray):
    ids = np.ascontiguousarray(slot_ids, dtype=np.int32)
    rows = np.ascontiguousarray(rows, dtype=np.uint8).reshape(len(ids), store.shape[1])
    _load().oracle_store_rows(_ptr(store), store.shape[0], store.shape[1], _ptr(ids), len(ids), _ptr(rows), 1)


def store_load(store: np.ndarray, slot_ids) -> np.ndarray:
    ids = np.ascontiguousarray(slot_ids, dtype=np.int32)
    rows = np.empty((len(ids), store.shape[1]), dtype=np.uint8)
    _load().oracle_store_rows(_ptr(store), store.shape[0], store.shape[1], _ptr(ids), len(ids), _ptr(rows), 0)
    return rows
