"""ctypes binding of libomni_attn.so: argument marshalling only.

Functions carry the names of the C entry points declared in
``include/omni_attn.h``; tensors are torch CUDA tensors used purely as device
memory handles.  There is no fallback: if the library has not been built, or a
tensor is not on the GPU, the call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libomni_attn.so")

OMNI_F32, OMNI_BF16 = 0, 1
OMNI_KERNEL_AUTO, OMNI_KERNEL_VECTOR, OMNI_KERNEL_MFMA = 0, 1, 2
OMNI_OK, OMNI_ERR_NULL, OMNI_ERR_SHAPE, OMNI_ERR_DTYPE, OMNI_ERR_UNSUPPORTED, OMNI_ERR_LAUNCH = 0, -1, -2, -3, -4, -5
OMNI_ERR_TOO_LARGE = -6
OMNI_STATIC_SCRATCH_BYTES = 2 * 1024 * 1024

EXPORTS = ("omni_paged_decode_attn", "omni_paged_decode_attn_static", "omni_decode_workspace_bytes", "omni_decode_plan",
           "omni_decode_abandoned_waves", "omni_decode_kernel_name", "omni_merge_partials", "omni_merge_partials_masked",
           "omni_status_string", "omni_debug_gather_kv", "omni_debug_stream_read", "omni_debug_copy",
           "omni_debug_host_stream_read",
           "omni_kv_append", "omni_kv_gather_pages", "omni_kv_scatter_pages",
           "omni_queue_push", "omni_queue_pop", "omni_csr_from_tags", "omni_residual_save", "omni_residual_load",
           "omni_host_partial_attn", "omni_debug_sort_bin", "omni_debug_ticket_map",
           "omni_debug_decode_timeline_shape", "omni_debug_decode_timeline")


class OmniError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s" % (where, omni_status_string(status)))


class omni_partial_src(ctypes.Structure):
    _fields_ = [("o", ctypes.c_void_p), ("lse", ctypes.c_void_p), ("row_offsets", ctypes.c_void_p),
                ("dense_rows_per_seq", ctypes.c_int32)]


class omni_decode_args(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("block_size", ctypes.c_int32), ("max_blocks_per_seq", ctypes.c_int32),
        ("num_blocks", ctypes.c_int64), ("qkv_dtype", ctypes.c_int32), ("sm_scale", ctypes.c_float),
        ("q", ctypes.c_void_p), ("k_pool", ctypes.c_void_p), ("v_pool", ctypes.c_void_p),
        ("block_table", ctypes.c_void_p), ("ctx_begin", ctypes.c_void_p), ("ctx_end", ctypes.c_void_p),
        ("chunk_tokens", ctypes.c_int32), ("max_chunks", ctypes.c_int32),
        ("part_o", ctypes.c_void_p), ("part_lse", ctypes.c_void_p),
        ("out_o", ctypes.c_void_p), ("out_dtype", ctypes.c_int32), ("out_lse", ctypes.c_void_p),
        ("kernel", ctypes.c_int32),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_uint64),
        ("workspace_planned", ctypes.c_int32),
        ("seq_final", ctypes.c_void_p), ("fuse_merge", ctypes.c_int32),
        ("ext_srcs", ctypes.POINTER(omni_partial_src)), ("n_ext_srcs", ctypes.c_int32),
    ]


class omni_kv_cache(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("block_size", ctypes.c_int32), ("max_blocks_per_seq", ctypes.c_int32),
                ("num_blocks", ctypes.c_int64), ("dtype", ctypes.c_int32),
                ("k_pool", ctypes.c_void_p), ("v_pool", ctypes.c_void_p), ("block_table", ctypes.c_void_p)]


class omni_queue(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("tags", ctypes.c_void_p), ("state", ctypes.c_void_p),
                ("capacity", ctypes.c_int32), ("row_bytes", ctypes.c_int32)]


class omni_host_attn_args(ctypes.Structure):
    _fields_ = [("n_rows", ctypes.c_int32),
                ("batch", ctypes.c_int32), ("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("block_size", ctypes.c_int32), ("max_blocks_per_seq", ctypes.c_int32),
                ("num_blocks", ctypes.c_int64), ("qkv_dtype", ctypes.c_int32), ("sm_scale", ctypes.c_float),
                ("q", ctypes.c_void_p), ("k_pool", ctypes.c_void_p), ("v_pool", ctypes.c_void_p),
                ("block_table", ctypes.c_void_p), ("row_seq", ctypes.c_void_p), ("row_begin", ctypes.c_void_p),
                ("row_end", ctypes.c_void_p), ("part_o", ctypes.c_void_p), ("part_lse", ctypes.c_void_p),
                ("n_threads", ctypes.c_int32), ("isa_level", ctypes.c_int32)]


_lib = None


def load_library() -> ctypes.CDLL:
    """Load the HIP library (no GPU needed for loading).  Raises if it is absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libomni_attn.so is not built (run `python -m paper_2603_12831_amd.build`); "
                               "there is no fallback path")
        lib = ctypes.CDLL(LIB_PATH)
        vp = ctypes.c_void_p
        lib.omni_paged_decode_attn.argtypes = [ctypes.POINTER(omni_decode_args), vp]
        lib.omni_paged_decode_attn.restype = ctypes.c_int
        lib.omni_paged_decode_attn_static.argtypes = [ctypes.POINTER(omni_decode_args), vp]
        lib.omni_paged_decode_attn_static.restype = ctypes.c_int
        lib.omni_decode_plan.argtypes = [ctypes.POINTER(omni_decode_args), vp]
        lib.omni_decode_plan.restype = ctypes.c_int
        lib.omni_decode_workspace_bytes.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32]
        lib.omni_decode_workspace_bytes.restype = ctypes.c_uint64
        lib.omni_decode_kernel_name.argtypes = [ctypes.POINTER(omni_decode_args)]
        lib.omni_decode_kernel_name.restype = ctypes.c_char_p
        lib.omni_decode_abandoned_waves.argtypes = [vp, ctypes.POINTER(ctypes.c_uint32), vp]
        lib.omni_decode_abandoned_waves.restype = ctypes.c_int
        lib.omni_merge_partials_masked.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                                   ctypes.POINTER(omni_partial_src), ctypes.c_int32, vp, vp,
                                                   ctypes.c_int32, vp, vp]
        lib.omni_merge_partials_masked.restype = ctypes.c_int
        lib.omni_merge_partials.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                            ctypes.POINTER(omni_partial_src), ctypes.c_int32, vp,
                                            ctypes.c_int32, vp, vp]
        lib.omni_merge_partials.restype = ctypes.c_int
        lib.omni_status_string.argtypes = [ctypes.c_int]
        lib.omni_status_string.restype = ctypes.c_char_p
        lib.omni_debug_gather_kv.argtypes = [ctypes.POINTER(omni_decode_args), ctypes.c_int32, vp, vp, vp]
        lib.omni_debug_gather_kv.restype = ctypes.c_int
        lib.omni_debug_stream_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
        lib.omni_debug_stream_read.restype = ctypes.c_int
        lib.omni_debug_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
        lib.omni_debug_copy.restype = ctypes.c_int
        lib.omni_debug_host_stream_read.argtypes = [vp, ctypes.c_size_t, ctypes.c_int32, ctypes.POINTER(ctypes.c_uint64)]
        lib.omni_debug_host_stream_read.restype = ctypes.c_int
        lib.omni_debug_sort_bin.argtypes = [ctypes.c_int32, ctypes.c_int32]
        lib.omni_debug_sort_bin.restype = ctypes.c_int32
        lib.omni_debug_ticket_map.argtypes = [ctypes.c_uint32, ctypes.c_uint32, ctypes.c_int32, ctypes.c_uint32, vp,
                                              ctypes.c_uint64, ctypes.POINTER(ctypes.c_uint32)]
        lib.omni_debug_ticket_map.restype = ctypes.c_int
        lib.omni_debug_decode_timeline_shape.argtypes = [ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32)]
        lib.omni_debug_decode_timeline_shape.restype = ctypes.c_int
        lib.omni_debug_decode_timeline.argtypes = [ctypes.POINTER(omni_decode_args), vp, ctypes.c_uint64, vp]
        lib.omni_debug_decode_timeline.restype = ctypes.c_int
        qp = ctypes.POINTER(omni_queue)
        lib.omni_queue_push.argtypes = [qp, vp, vp, ctypes.c_int32, vp, vp]
        lib.omni_queue_push.restype = ctypes.c_int
        lib.omni_queue_pop.argtypes = [qp, vp, vp, ctypes.c_int32, vp, vp]
        lib.omni_queue_pop.restype = ctypes.c_int
        lib.omni_csr_from_tags.argtypes = [vp, vp, ctypes.c_int32, ctypes.c_int32, vp, vp]
        lib.omni_csr_from_tags.restype = ctypes.c_int
        lib.omni_residual_save.argtypes = [vp, ctypes.c_int64, ctypes.c_int32, vp, ctypes.c_int32, vp, vp]
        lib.omni_residual_save.restype = ctypes.c_int
        lib.omni_residual_load.argtypes = [vp, ctypes.c_int64, ctypes.c_int32, vp, ctypes.c_int32, vp, vp]
        lib.omni_residual_load.restype = ctypes.c_int
        kvp = ctypes.POINTER(omni_kv_cache)
        lib.omni_kv_append.argtypes = [kvp, vp, vp, vp, vp]
        lib.omni_kv_append.restype = ctypes.c_int
        lib.omni_kv_gather_pages.argtypes = [kvp, vp, ctypes.c_int64, vp, vp, vp]
        lib.omni_kv_gather_pages.restype = ctypes.c_int
        lib.omni_kv_scatter_pages.argtypes = [kvp, vp, ctypes.c_int64, vp, vp, vp]
        lib.omni_kv_scatter_pages.restype = ctypes.c_int
        lib.omni_host_partial_attn.argtypes = [ctypes.POINTER(omni_host_attn_args)]
        lib.omni_host_partial_attn.restype = ctypes.c_int
        _lib = lib
    return _lib


def _dev_ptr(t: Optional[torch.Tensor], name: str, dtype=None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("%s must be a GPU tensor" % name)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if dtype is not None and t.dtype != dtype:
        raise ValueError("%s must have dtype %s, got %s" % (name, dtype, t.dtype))
    return t.data_ptr()


def _stream_ptr(stream) -> Optional[int]:
    """Raw handle of `stream`, or of torch's current stream on the current device (0 / None = the default stream)."""
    if stream is None:
        try:        # the raw handle straight from torch's runtime: 0.1 us against 2.7 us for the Stream object
            return torch._C._cuda_getCurrentRawStream(torch._C._cuda_getDevice()) or None
        except AttributeError:
            stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def _dtype_code(t: torch.Tensor, name: str) -> int:
    if t.dtype == torch.float32:
        return OMNI_F32
    if t.dtype == torch.bfloat16:
        return OMNI_BF16
    raise ValueError("%s must be float32 or bfloat16" % name)


def omni_status_string(status: int) -> str:
    return load_library().omni_status_string(int(status)).decode()


def make_decode_args(q, k_pool, v_pool, block_table, ctx_begin, ctx_end, *, sm_scale: float,
                     chunk_tokens: int = 0, max_chunks: int = 1, part_o=None, part_lse=None, out_o=None,
                     out_lse=None, kernel: int = OMNI_KERNEL_AUTO, workspace=None,
                     workspace_planned: bool = False, seq_final=None, fuse_merge: bool = False,
                     ext_srcs: Optional[Sequence["PartialSrc"]] = None) -> omni_decode_args:
    """Fill the C argument struct from tensors (shapes are taken from the tensors)."""
    a = omni_decode_args()
    a.batch, a.num_q_heads, a.head_dim = q.shape
    a.num_blocks, a.num_kv_heads, a.block_size, d2 = k_pool.shape
    if d2 != a.head_dim or tuple(v_pool.shape) != tuple(k_pool.shape):
        raise ValueError("pool shapes do not match q / each other")
    if block_table.shape[0] != a.batch or ctx_end.shape[0] != a.batch:
        raise ValueError("block_table / ctx_end batch mismatch")
    a.max_blocks_per_seq = block_table.shape[1]
    a.qkv_dtype = _dtype_code(q, "q")
    if k_pool.dtype != q.dtype or v_pool.dtype != q.dtype:
        raise ValueError("q, k_pool, v_pool must share a dtype")
    a.sm_scale = float(sm_scale)
    a.q, a.k_pool, a.v_pool = _dev_ptr(q, "q"), _dev_ptr(k_pool, "k_pool"), _dev_ptr(v_pool, "v_pool")
    a.block_table = _dev_ptr(block_table, "block_table", torch.int32)
    a.ctx_begin = _dev_ptr(ctx_begin, "ctx_begin", torch.int32)
    a.ctx_end = _dev_ptr(ctx_end, "ctx_end", torch.int32)
    a.chunk_tokens, a.max_chunks = int(chunk_tokens), int(max_chunks)
    if part_o is not None and part_o.numel() != a.batch * a.max_chunks * a.num_q_heads * a.head_dim:
        raise ValueError("part_o has the wrong size")
    if part_lse is not None and part_lse.numel() != a.batch * a.max_chunks * a.num_q_heads:
        raise ValueError("part_lse has the wrong size")
    a.part_o = _dev_ptr(part_o, "part_o", torch.float32)
    a.part_lse = _dev_ptr(part_lse, "part_lse", torch.float32)
    if out_o is not None:
        if out_o.numel() != q.numel():
            raise ValueError("out_o has the wrong size")
        a.out_dtype = _dtype_code(out_o, "out_o")
    a.out_o = _dev_ptr(out_o, "out_o")
    if out_lse is not None and out_lse.numel() != a.batch * a.num_q_heads:
        raise ValueError("out_lse has the wrong size")
    a.out_lse = _dev_ptr(out_lse, "out_lse", torch.float32)
    a.kernel = int(kernel)
    a.workspace = _dev_ptr(workspace, "workspace")
    a.workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    a.workspace_planned = 1 if workspace_planned else 0
    if seq_final is not None and seq_final.numel() != a.batch:
        raise ValueError("seq_final must have one entry per sequence")
    a.seq_final = _dev_ptr(seq_final, "seq_final", torch.int32)
    a.fuse_merge = 1 if fuse_merge else 0
    if ext_srcs:
        a._ext_keepalive = make_partial_srcs(ext_srcs, a.batch, a.num_q_heads, a.head_dim)   # host array
        a.ext_srcs = ctypes.cast(a._ext_keepalive, ctypes.POINTER(omni_partial_src))
        a.n_ext_srcs = len(ext_srcs)
    return a


def omni_paged_decode_attn(q, k_pool, v_pool, block_table, ctx_begin, ctx_end, *, sm_scale: float,
                           chunk_tokens: int = 0, max_chunks: int = 1, part_o=None, part_lse=None,
                           out_o=None, out_lse=None, kernel: int = OMNI_KERNEL_AUTO, workspace=None,
                           workspace_planned: bool = False, seq_final=None, fuse_merge: bool = False,
                           ext_srcs=None, stream=None, check: bool = True) -> int:
    a = make_decode_args(q, k_pool, v_pool, block_table, ctx_begin, ctx_end, sm_scale=sm_scale,
                         chunk_tokens=chunk_tokens, max_chunks=max_chunks, part_o=part_o, part_lse=part_lse,
                         out_o=out_o, out_lse=out_lse, kernel=kernel, workspace=workspace,
                         workspace_planned=workspace_planned, seq_final=seq_final, fuse_merge=fuse_merge,
                         ext_srcs=ext_srcs)
    return omni_paged_decode_attn_raw(a, stream, check)


def omni_paged_decode_attn_raw(args: omni_decode_args, stream=None, check: bool = True) -> int:
    st = load_library().omni_paged_decode_attn(ctypes.byref(args), _stream_ptr(stream))
    if check and st != OMNI_OK:
        raise OmniError(st, "omni_paged_decode_attn")
    return st


def omni_paged_decode_attn_static(args: omni_decode_args, stream=None, check: bool = True) -> int:
    st = load_library().omni_paged_decode_attn_static(ctypes.byref(args), _stream_ptr(stream))
    if check and st != OMNI_OK:
        raise OmniError(st, "omni_paged_decode_attn_static")
    return st


def omni_decode_plan(args: omni_decode_args, stream=None, check: bool = True) -> int:
    st = load_library().omni_decode_plan(ctypes.byref(args), _stream_ptr(stream))
    if check and st != OMNI_OK:
        raise OmniError(st, "omni_decode_plan")
    return st


def omni_decode_workspace_bytes(batch: int, max_chunks: int, num_kv_heads: int) -> int:
    return int(load_library().omni_decode_workspace_bytes(int(batch), int(max_chunks), int(num_kv_heads)))


def omni_decode_kernel_name(args: omni_decode_args) -> str:
    return load_library().omni_decode_kernel_name(ctypes.byref(args)).decode()


def omni_decode_abandoned_waves(workspace=None, stream=None) -> int:
    """Reads and clears the diagnostic word of a work list (None: the library's static scratch)."""
    n = ctypes.c_uint32(0)
    st = load_library().omni_decode_abandoned_waves(_dev_ptr(workspace, "workspace"), ctypes.byref(n), _stream_ptr(stream))
    if st != OMNI_OK:
        raise OmniError(st, "omni_decode_abandoned_waves")
    return int(n.value)


PartialSrc = Tuple[torch.Tensor, torch.Tensor, Optional[torch.Tensor], int]


def make_partial_srcs(srcs: Sequence[PartialSrc], batch: int, num_q_heads: int, head_dim: int):
    arr = (omni_partial_src * max(1, len(srcs)))()
    for i, (o, lse, row_offsets, dense_rows) in enumerate(srcs):
        n_rows = lse.numel() // num_q_heads
        if o.numel() != n_rows * num_q_heads * head_dim:
            raise ValueError("partial source %d: o / lse sizes disagree" % i)
        if row_offsets is None and n_rows != batch * dense_rows:
            raise ValueError("partial source %d: dense rows do not cover the batch" % i)
        if row_offsets is not None and row_offsets.numel() != batch + 1:
            raise ValueError("partial source %d: row_offsets must have batch+1 entries" % i)
        arr[i].o = _dev_ptr(o, "src.o", torch.float32)
        arr[i].lse = _dev_ptr(lse, "src.lse", torch.float32)
        arr[i].row_offsets = _dev_ptr(row_offsets, "src.row_offsets", torch.int32)
        arr[i].dense_rows_per_seq = int(dense_rows)
    return arr


def omni_merge_partials(batch: int, num_q_heads: int, head_dim: int, srcs: Sequence[PartialSrc], out_o,
                        out_lse=None, stream=None, check: bool = True) -> int:
    """srcs: sequence of (o, lse, row_offsets or None, dense_rows_per_seq)."""
    arr = make_partial_srcs(srcs, batch, num_q_heads, head_dim)
    if out_o.numel() != batch * num_q_heads * head_dim:
        raise ValueError("out_o has the wrong size")
    st = load_library().omni_merge_partials(batch, num_q_heads, head_dim, arr, len(srcs),
                                            _dev_ptr(out_o, "out_o"), _dtype_code(out_o, "out_o"),
                                            _dev_ptr(out_lse, "out_lse", torch.float32), _stream_ptr(stream))
    if check and st != OMNI_OK:
        raise OmniError(st, "omni_merge_partials")
    return st


def omni_merge_partials_masked(batch: int, num_q_heads: int, head_dim: int, srcs: Sequence[PartialSrc], skip,
                               out_o, out_lse=None, stream=None, check: bool = True) -> int:
    """As omni_merge_partials; rows of sequences with skip[i] != 0 (int32 [batch] or None) are left alone."""
    arr = make_partial_srcs(srcs, batch, num_q_heads, head_dim)
    if out_o.numel() != batch * num_q_heads * head_dim:
        raise ValueError("out_o has the wrong size")
    if skip is not None and skip.numel() != batch:
        raise ValueError("skip must have one entry per sequence")
    st = load_library().omni_merge_partials_masked(batch, num_q_heads, head_dim, arr, len(srcs),
                                                   _dev_ptr(skip, "skip", torch.int32),
                                                   _dev_ptr(out_o, "out_o"), _dtype_code(out_o, "out_o"),
                                                   _dev_ptr(out_lse, "out_lse", torch.float32), _stream_ptr(stream))
    if check and st != OMNI_OK:
        raise OmniError(st, "omni_merge_partials_masked")
    return st


class PreparedMerge:
    """A merge call with its arguments marshalled once (a step loop then pays one foreign call per merge):
    `run(stream)` calls omni_merge_partials_masked (skip may be None) on the same buffers every time."""

    def __init__(self, batch: int, num_q_heads: int, head_dim: int, srcs: Sequence[PartialSrc], skip, out_o,
                 out_lse=None):
        if out_o.numel() != batch * num_q_heads * head_dim:
            raise ValueError("out_o has the wrong size")
        if skip is not None and skip.numel() != batch:
            raise ValueError("skip must have one entry per sequence")
        self._keep = (list(srcs), skip, out_o, out_lse)        # the tensors behind the raw pointers
        self._fn = load_library().omni_merge_partials_masked
        self._argv = (batch, num_q_heads, head_dim, make_partial_srcs(srcs, batch, num_q_heads, head_dim), len(srcs),
                      _dev_ptr(skip, "skip", torch.int32), _dev_ptr(out_o, "out_o"), _dtype_code(out_o, "out_o"),
                      _dev_ptr(out_lse, "out_lse", torch.float32))

    def run(self, stream=None, check: bool = True) -> int:
        st = self._fn(*self._argv, _stream_ptr(stream))
        if check and st != OMNI_OK:
            raise OmniError(st, "omni_merge_partials_masked")
        return st


def omni_debug_decode_timeline_shape():
    """(workgroups of a persistent launch on the current device, 64-bit stamp words per workgroup)"""
    n, w = ctypes.c_int32(0), ctypes.c_int32(0)
    st = load_library().omni_debug_decode_timeline_shape(ctypes.byref(n), ctypes.byref(w))
    if st != OMNI_OK:
        raise OmniError(st, "omni_debug_decode_timeline_shape")
    return n.value, w.value


def omni_debug_decode_timeline(args: omni_decode_args, stamps, stream=None, check: bool = True) -> int:
    """The decode call through the time-stamping kernel instance; stamps: zeroed int64 device tensor."""
    st = load_library().omni_debug_decode_timeline(ctypes.byref(args), _dev_ptr(stamps, "stamps", torch.int64),
                                                   stamps.numel(), _stream_ptr(stream))
    if check and st != OMNI_OK:
        raise OmniError(st, "omni_debug_decode_timeline")
    return st


def omni_debug_gather_kv(args: omni_decode_args, seq: int, k_out, v_out, stream=None, check: bool = True) -> int:
    st = load_library().omni_debug_gather_kv(ctypes.byref(args), int(seq), _dev_ptr(k_out, "k_out"),
                                             _dev_ptr(v_out, "v_out"), _stream_ptr(stream))
    if check and st != OMNI_OK:
        raise OmniError(st, "omni_debug_gather_kv")
    return st


def omni_debug_stream_read(src, sink, nbytes: Optional[int] = None, stream=None) -> int:
    n = src.numel() * src.element_size() if nbytes is None else int(nbytes)
    if sink.numel() * sink.element_size() < 16 or n > src.numel() * src.element_size():
        raise ValueError("sink needs 16 bytes; nbytes must not exceed src")
    st = load_library().omni_debug_stream_read(_dev_ptr(src, "src"), n, _dev_ptr(sink, "sink"), _stream_ptr(stream))
    if st != OMNI_OK:
        raise OmniError(st, "omni_debug_stream_read")
    return st


def omni_debug_copy(dst, src, nbytes: Optional[int] = None, stream=None) -> int:
    n = src.numel() * src.element_size() if nbytes is None else int(nbytes)
    if n > dst.numel() * dst.element_size() or n > src.numel() * src.element_size():
        raise ValueError("copy larger than its buffers")
    st = load_library().omni_debug_copy(_dev_ptr(dst, "dst"), _dev_ptr(src, "src"), n, _stream_ptr(stream))
    if st != OMNI_OK:
        raise OmniError(st, "omni_debug_copy")
    return st


def omni_debug_host_stream_read(array, n_threads: int = 0) -> int:
    """Reads a C-contiguous numpy array once with n_threads host threads; returns the fold of its words."""
    nbytes = array.nbytes // 8 * 8
    if not array.flags["C_CONTIGUOUS"]:
        raise ValueError("array must be C-contiguous")
    sink = ctypes.c_uint64(0)
    st = load_library().omni_debug_host_stream_read(array.ctypes.data, nbytes, int(n_threads), ctypes.byref(sink))
    if st != OMNI_OK:
        raise OmniError(st, "omni_debug_host_stream_read")
    return int(sink.value)


def make_kv_cache(k_pool, v_pool, block_table=None) -> omni_kv_cache:
    c = omni_kv_cache()
    c.num_blocks, c.num_kv_heads, c.block_size, c.head_dim = k_pool.shape
    if tuple(v_pool.shape) != tuple(k_pool.shape) or v_pool.dtype != k_pool.dtype:
        raise ValueError("k_pool and v_pool must match")
    c.dtype = _dtype_code(k_pool, "k_pool")
    c.k_pool, c.v_pool = _dev_ptr(k_pool, "k_pool"), _dev_ptr(v_pool, "v_pool")
    if block_table is not None:
        c.batch, c.max_blocks_per_seq = block_table.shape
        c.block_table = _dev_ptr(block_table, "block_table", torch.int32)
    return c


def omni_kv_append(k_pool, v_pool, block_table, k_new, v_new, positions, stream=None, check: bool = True) -> int:
    c = make_kv_cache(k_pool, v_pool, block_table)
    want = (c.batch, c.num_kv_heads, c.head_dim)
    if tuple(k_new.shape) != want or tuple(v_new.shape) != want or k_new.dtype != k_pool.dtype or v_new.dtype != k_pool.dtype:
        raise ValueError("k_new / v_new must be [batch, num_kv_heads, head_dim] of the pool dtype")
    if positions.numel() != c.batch:
        raise ValueError("positions must have one entry per sequence")
    st = load_library().omni_kv_append(ctypes.byref(c), _dev_ptr(k_new, "k_new"), _dev_ptr(v_new, "v_new"),
                                       _dev_ptr(positions, "positions", torch.int32), _stream_ptr(stream))
    if check and st != OMNI_OK:
        raise OmniError(st, "omni_kv_append")
    return st


def _kv_pages(fn_name, k_pool, v_pool, page_ids, k_stage, v_stage, stream, check):
    c = make_kv_cache(k_pool, v_pool)
    n = page_ids.numel()
    per_page = c.num_kv_heads * c.block_size * c.head_dim
    for t, name in ((k_stage, "k staging"), (v_stage, "v staging")):
        if t.numel() != n * per_page or t.dtype != k_pool.dtype:
            raise ValueError("%s must hold n_pages pages of the pool dtype" % name)
    st = getattr(load_library(), fn_name)(ctypes.byref(c), _dev_ptr(page_ids, "page_ids", torch.int32), n,
                                          _dev_ptr(k_stage, "k staging"), _dev_ptr(v_stage, "v staging"),
                                          _stream_ptr(stream))
    if check and st != OMNI_OK:
        raise OmniError(st, fn_name)
    return st


def omni_kv_gather_pages(k_pool, v_pool, page_ids, k_out, v_out, stream=None, check: bool = True) -> int:
    return _kv_pages("omni_kv_gather_pages", k_pool, v_pool, page_ids, k_out, v_out, stream, check)


def omni_kv_scatter_pages(k_pool, v_pool, page_ids, k_in, v_in, stream=None, check: bool = True) -> int:
    return _kv_pages("omni_kv_scatter_pages", k_pool, v_pool, page_ids, k_in, v_in, stream, check)


def make_queue(data, tags, state) -> omni_queue:
    """data: [capacity, row_bytes] uint8; tags: [capacity] int32 or None; state: [4] int32 (zeroed once)."""
    q = omni_queue()
    if data.dtype != torch.uint8 or data.dim() != 2 or state.numel() != 4 or state.element_size() != 4:
        raise ValueError("queue data must be a 2-D uint8 tensor and state four 32-bit words")
    q.capacity, q.row_bytes = data.shape
    q.data, q.state = _dev_ptr(data, "queue data"), _dev_ptr(state, "queue state")
    q.tags = _dev_ptr(tags, "queue tags", torch.int32)
    return q


def omni_queue_push(q: omni_queue, rows, tags=None, n_pushed=None, stream=None, check: bool = True) -> int:
    n = rows.shape[0]
    if rows.numel() * rows.element_size() != n * q.row_bytes or (tags is not None and tags.numel() != n):
        raise ValueError("rows / tags do not match the queue's row size")
    st = load_library().omni_queue_push(ctypes.byref(q), _dev_ptr(rows, "rows"), _dev_ptr(tags, "tags", torch.int32), n,
                                        _dev_ptr(n_pushed, "n_pushed", torch.int32), _stream_ptr(stream))
    if check and st != OMNI_OK:
        raise OmniError(st, "omni_queue_push")
    return st


def omni_queue_pop(q: omni_queue, rows_out, tags_out=None, n_popped=None, stream=None, check: bool = True) -> int:
    n = rows_out.shape[0]
    if rows_out.numel() * rows_out.element_size() != n * q.row_bytes or (tags_out is not None and tags_out.numel() != n):
        raise ValueError("rows_out / tags_out do not match the queue's row size")
    st = load_library().omni_queue_pop(ctypes.byref(q), _dev_ptr(rows_out, "rows_out"),
                                       _dev_ptr(tags_out, "tags_out", torch.int32), n,
                                       _dev_ptr(n_popped, "n_popped", torch.int32), _stream_ptr(stream))
    if check and st != OMNI_OK:
        raise OmniError(st, "omni_queue_pop")
    return st


def omni_csr_from_tags(tags, n_rows, batch: int, row_offsets, stream=None, check: bool = True) -> int:
    """tags int32 [max_rows], n_rows int32 [1] or None, row_offsets int32 [batch + 1] (all on the GPU)."""
    if row_offsets.numel() != batch + 1:
        raise ValueError("row_offsets must have batch + 1 entries")
    st = load_library().omni_csr_from_tags(_dev_ptr(tags, "tags", torch.int32), _dev_ptr(n_rows, "n_rows", torch.int32),
                                           tags.numel(), int(batch), _dev_ptr(row_offsets, "row_offsets", torch.int32),
                                           _stream_ptr(stream))
    if check and st != OMNI_OK:
        raise OmniError(st, "omni_csr_from_tags")
    return st


def _residual(fn_name, store, slot_ids, rows, stream, check):
    n = slot_ids.numel()
    row_bytes = store.shape[1] * store.element_size()
    if store.dim() != 2 or rows.numel() * rows.element_size() != n * row_bytes:
        raise ValueError("store must be [n_slots, row] and rows hold one store row per slot id")
    st = getattr(load_library(), fn_name)(_dev_ptr(store, "store"), store.shape[0], row_bytes,
                                          _dev_ptr(slot_ids, "slot_ids", torch.int32), n, _dev_ptr(rows, "rows"),
                                          _stream_ptr(stream))
    if check and st != OMNI_OK:
        raise OmniError(st, fn_name)
    return st


def omni_residual_save(store, slot_ids, rows, stream=None, check: bool = True) -> int:
    return _residual("omni_residual_save", store, slot_ids, rows, stream, check)


def omni_residual_load(store, slot_ids, rows_out, stream=None, check: bool = True) -> int:
    return _residual("omni_residual_load", store, slot_ids, rows_out, stream, check)


def omni_host_partial_attn(q, k_pool, v_pool, block_table, row_seq, row_begin, row_end, sm_scale: float,
                           dtype: str, n_threads: int = 0, check: bool = True, isa_level: int = 0):
    """Partial rows computed on the host's cores from KV in host memory.  q, k_pool, v_pool: C-contiguous
    numpy arrays (float32, or uint16 holding bf16 bit patterns when dtype == "bf16") in the layouts of the
    decode call; block_table int32 [batch, max_blocks]; row_seq / row_begin / row_end int32 [n_rows].
    isa_level: 0 best available, 1 plain, 2 AVX2 + FMA, 3 AVX-512.
    Returns (part_o [n_rows, Hq, D] float32, part_lse [n_rows, Hq] float32)."""
    import numpy as np
    want = np.uint16 if dtype == "bf16" else np.float32
    for name, arr in (("q", q), ("k_pool", k_pool), ("v_pool", v_pool)):
        if arr.dtype != want or not arr.flags["C_CONTIGUOUS"]:
            raise ValueError("%s must be a C-contiguous %s array" % (name, np.dtype(want).name))
    block_table = np.ascontiguousarray(block_table, dtype=np.int32)
    row_seq = np.ascontiguousarray(row_seq, dtype=np.int32)
    row_end = np.ascontiguousarray(row_end, dtype=np.int32)
    row_begin = None if row_begin is None else np.ascontiguousarray(row_begin, dtype=np.int32)
    n_rows = int(row_seq.shape[0])
    batch, hq, d = q.shape
    num_blocks, hkv, bs, _ = k_pool.shape
    part_o = np.empty((n_rows, hq, d), dtype=np.float32)
    part_lse = np.empty((n_rows, hq), dtype=np.float32)
    a = omni_host_attn_args(
        n_rows=n_rows, batch=batch, num_q_heads=hq, num_kv_heads=hkv, head_dim=d, block_size=bs,
        max_blocks_per_seq=block_table.shape[1], num_blocks=num_blocks,
        qkv_dtype=OMNI_BF16 if dtype == "bf16" else OMNI_F32, sm_scale=float(sm_scale),
        q=q.ctypes.data, k_pool=k_pool.ctypes.data, v_pool=v_pool.ctypes.data,
        block_table=block_table.ctypes.data, row_seq=row_seq.ctypes.data,
        row_begin=None if row_begin is None else row_begin.ctypes.data, row_end=row_end.ctypes.data,
        part_o=part_o.ctypes.data, part_lse=part_lse.ctypes.data, n_threads=int(n_threads), isa_level=int(isa_level))
    st = load_library().omni_host_partial_attn(ctypes.byref(a))
    if check and st != OMNI_OK:
        raise OmniError(st, "omni_host_partial_attn")
    return (part_o, part_lse) if check else st


def omni_debug_sort_bin(tokens: int, chunk_tokens: int) -> int:
    return int(load_library().omni_debug_sort_bin(int(tokens), int(chunk_tokens)))


def omni_debug_ticket_map(n_entries: int, n_long_entries: int, num_kv_heads: int, n_workgroups: int):
    """(items [n_tickets, 4] int32 with -1 = none, grouped [n_tickets] bool) of the persistent form's tickets."""
    import numpy as np
    cap = (n_entries * max(num_kv_heads, 1) + 4) * 8 + 8
    buf = np.full(cap, -7, dtype=np.int32)
    n = ctypes.c_uint32(0)
    st = load_library().omni_debug_ticket_map(n_entries, n_long_entries, num_kv_heads, n_workgroups,
                                              buf.ctypes.data_as(ctypes.c_void_p), cap, ctypes.byref(n))
    if st != OMNI_OK:
        raise OmniError(st, "omni_debug_ticket_map")
    pairs = buf[:n.value * 8].reshape(n.value, 4, 2)
    return pairs[:, :, 0].copy(), pairs[:, 0, 1].astype(bool)
