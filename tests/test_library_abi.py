"""The built HIP library loads without a GPU, exports every symbol the header
declares, and rejects bad arguments on the host before anything is launched."""
import ctypes
import os
import re

import pytest

from paper_2603_12831_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_header_symbols_are_exported():
    hdr = open(os.path.join(ROOT, "include", "omni_attn.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(omni_[a-z_]+)\s*\(", hdr))
    assert declared == set(binding.EXPORTS)
    lib = binding.load_library()
    for name in declared:
        assert getattr(lib, name) is not None


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header must compile as C99 (no C++ in the signatures) with warnings on."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    src = tmp_path / "use_header.c"
    src.write_text('#include "omni_attn.h"\n'
                   'int main(void) { omni_decode_args a; a.batch = 0; return (int)sizeof(a) == 0 || a.batch; }\n')
    r = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(ROOT, "include"),
                        "-fsyntax-only", str(src)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr


def test_status_strings():
    assert binding.omni_status_string(0) == "OMNI_OK"
    for code in (-1, -2, -3, -4, -5):
        assert binding.omni_status_string(code).startswith("OMNI_ERR_")
    assert "unknown" in binding.omni_status_string(-99)


def _args(**over):
    a = binding.omni_decode_args()
    a.batch, a.num_q_heads, a.num_kv_heads, a.head_dim, a.block_size, a.max_blocks_per_seq = 2, 8, 2, 64, 16, 4
    a.num_blocks, a.qkv_dtype, a.sm_scale = 8, binding.OMNI_F32, 0.125
    # never dereferenced on the host; every case below is rejected before a launch
    for f in ("q", "k_pool", "v_pool", "block_table", "ctx_end", "part_o", "part_lse"):
        setattr(a, f, 0x1000)
    a.chunk_tokens, a.max_chunks = 0, 1
    for k, v in over.items():
        setattr(a, k, v)
    return a


@pytest.mark.parametrize("over,code", [
    (dict(q=None), binding.OMNI_ERR_NULL),
    (dict(ctx_end=None), binding.OMNI_ERR_NULL),
    (dict(part_o=None, part_lse=None), binding.OMNI_ERR_NULL),          # no output at all
    (dict(part_lse=None), binding.OMNI_ERR_NULL),
    (dict(num_q_heads=7), binding.OMNI_ERR_SHAPE),
    (dict(batch=-1), binding.OMNI_ERR_SHAPE),
    (dict(chunk_tokens=24, max_chunks=2), binding.OMNI_ERR_SHAPE),      # not a multiple of the page
    (dict(chunk_tokens=0, max_chunks=2), binding.OMNI_ERR_SHAPE),
    (dict(max_chunks=0), binding.OMNI_ERR_SHAPE),
    (dict(qkv_dtype=5), binding.OMNI_ERR_DTYPE),
    (dict(head_dim=96), binding.OMNI_ERR_UNSUPPORTED),
    (dict(block_size=32, chunk_tokens=0), binding.OMNI_ERR_UNSUPPORTED),
    (dict(num_q_heads=64, num_kv_heads=2), binding.OMNI_ERR_UNSUPPORTED),  # G = 32
    (dict(kernel=9), binding.OMNI_ERR_SHAPE),
    (dict(kernel=binding.OMNI_KERNEL_MFMA), binding.OMNI_ERR_UNSUPPORTED),  # fp32, D64: no matrix-core path
])
def test_decode_argument_errors(over, code):
    lib = binding.load_library()
    assert lib.omni_paged_decode_attn(ctypes.byref(_args(**over)), None) == code
    assert lib.omni_paged_decode_attn(None, None) == binding.OMNI_ERR_NULL


def test_plan_argument_errors_and_workspace_size():
    lib = binding.load_library()
    assert lib.omni_decode_workspace_bytes(256, 8, 8) >= 16 * 256 * 8 + 4 * 256 * 8
    assert lib.omni_decode_workspace_bytes(0, 8, 8) == 0 and lib.omni_decode_workspace_bytes(4, -1, 8) == 0
    assert lib.omni_decode_workspace_bytes(4, 1, 0) == 0
    assert lib.omni_decode_plan(None, None) == binding.OMNI_ERR_NULL
    assert lib.omni_decode_plan(ctypes.byref(_args()), None) == binding.OMNI_ERR_NULL        # no workspace
    assert lib.omni_decode_plan(ctypes.byref(_args(workspace=0x1000, workspace_bytes=8)), None) == binding.OMNI_ERR_SHAPE
    assert lib.omni_decode_plan(ctypes.byref(_args(workspace=0x1008, workspace_bytes=1 << 20)), None) == binding.OMNI_ERR_SHAPE
    assert lib.omni_decode_plan(ctypes.byref(_args(workspace=0x1000, workspace_bytes=1 << 20, chunk_tokens=8,
                                                   max_chunks=2)), None) == binding.OMNI_ERR_SHAPE


def test_merge_and_aid_argument_errors():
    lib = binding.load_library()
    src = (binding.omni_partial_src * 1)()
    src[0].o, src[0].lse, src[0].dense_rows_per_seq = 0x1000, 0x1000, 1
    assert lib.omni_merge_partials(2, 8, 64, src, 0, 0x1000, 0, None, None) == binding.OMNI_ERR_SHAPE
    assert lib.omni_merge_partials(2, 8, 64, src, 5, 0x1000, 0, None, None) == binding.OMNI_ERR_SHAPE
    assert lib.omni_merge_partials(2, 8, 96, src, 1, 0x1000, 0, None, None) == binding.OMNI_ERR_SHAPE
    assert lib.omni_merge_partials(2, 8, 64, src, 1, None, 0, None, None) == binding.OMNI_ERR_NULL
    assert lib.omni_merge_partials(2, 8, 64, None, 1, 0x1000, 0, None, None) == binding.OMNI_ERR_NULL
    assert lib.omni_merge_partials(2, 8, 64, src, 1, 0x1000, 7, None, None) == binding.OMNI_ERR_DTYPE
    src[0].lse = None
    assert lib.omni_merge_partials(2, 8, 64, src, 1, 0x1000, 0, None, None) == binding.OMNI_ERR_NULL
    assert lib.omni_debug_gather_kv(ctypes.byref(_args()), 5, 0x1000, 0x1000, None) == binding.OMNI_ERR_SHAPE
    assert lib.omni_debug_gather_kv(ctypes.byref(_args()), 0, None, 0x1000, None) == binding.OMNI_ERR_NULL
    assert lib.omni_debug_stream_read(0x1000, 24, 0x1000, None) == binding.OMNI_ERR_SHAPE
    assert lib.omni_debug_stream_read(None, 32, 0x1000, None) == binding.OMNI_ERR_NULL
    assert lib.omni_debug_copy(0x1000, None, 32, None) == binding.OMNI_ERR_NULL


def test_binding_refuses_host_tensors():
    import torch
    q = torch.zeros(1, 4, 64)
    kv = torch.zeros(2, 2, 16, 64)
    bt = torch.zeros(1, 2, dtype=torch.int32)
    end = torch.ones(1, dtype=torch.int32)
    with pytest.raises(ValueError):
        binding.omni_paged_decode_attn(q, kv, kv, bt, None, end, sm_scale=1.0, out_o=torch.zeros(1, 4, 64))


def test_kv_cache_argument_errors():
    lib = binding.load_library()
    c = binding.omni_kv_cache()
    c.batch, c.num_kv_heads, c.head_dim, c.block_size, c.max_blocks_per_seq, c.num_blocks = 2, 2, 64, 16, 4, 8
    c.dtype, c.k_pool, c.v_pool, c.block_table = binding.OMNI_BF16, 0x1000, 0x1000, 0x1000
    assert lib.omni_kv_append(None, 0x1000, 0x1000, 0x1000, None) == binding.OMNI_ERR_NULL
    assert lib.omni_kv_append(ctypes.byref(c), None, 0x1000, 0x1000, None) == binding.OMNI_ERR_NULL
    assert lib.omni_kv_gather_pages(ctypes.byref(c), None, 3, 0x1000, 0x1000, None) == binding.OMNI_ERR_NULL
    assert lib.omni_kv_gather_pages(ctypes.byref(c), 0x1000, -1, 0x1000, 0x1000, None) == binding.OMNI_ERR_SHAPE
    assert lib.omni_kv_scatter_pages(ctypes.byref(c), 0x1000, 3, 0x1000, None, None) == binding.OMNI_ERR_NULL
    c.block_size = 32
    assert lib.omni_kv_append(ctypes.byref(c), 0x1000, 0x1000, 0x1000, None) == binding.OMNI_ERR_UNSUPPORTED
    c.block_size, c.head_dim = 16, 4                                 # 8-byte rows cannot be moved in 16-byte pieces
    assert lib.omni_kv_gather_pages(ctypes.byref(c), 0x1000, 3, 0x1000, 0x1000, None) == binding.OMNI_ERR_UNSUPPORTED
    c.head_dim, c.dtype = 64, 9
    assert lib.omni_kv_scatter_pages(ctypes.byref(c), 0x1000, 3, 0x1000, 0x1000, None) == binding.OMNI_ERR_DTYPE
    c.dtype, c.block_table = binding.OMNI_F32, None
    assert lib.omni_kv_append(ctypes.byref(c), 0x1000, 0x1000, 0x1000, None) == binding.OMNI_ERR_NULL


def test_queue_and_store_argument_errors():
    lib = binding.load_library()
    q = binding.omni_queue()
    q.data, q.state, q.capacity, q.row_bytes = 0x1000, 0x1000, 8, 64
    assert lib.omni_queue_push(None, 0x1000, None, 1, None, None) == binding.OMNI_ERR_NULL
    assert lib.omni_queue_push(ctypes.byref(q), None, None, 2, None, None) == binding.OMNI_ERR_NULL
    assert lib.omni_queue_pop(ctypes.byref(q), None, None, 2, None, None) == binding.OMNI_ERR_NULL
    assert lib.omni_queue_push(ctypes.byref(q), 0x1000, None, -1, None, None) == binding.OMNI_ERR_SHAPE
    q.row_bytes = 24
    assert lib.omni_queue_pop(ctypes.byref(q), 0x1000, None, 2, None, None) == binding.OMNI_ERR_SHAPE
    q.row_bytes, q.state = 64, None
    assert lib.omni_queue_pop(ctypes.byref(q), 0x1000, None, 2, None, None) == binding.OMNI_ERR_NULL
    assert lib.omni_residual_save(0x1000, 0, 64, 0x1000, 2, 0x1000, None) == binding.OMNI_ERR_SHAPE
    assert lib.omni_residual_save(0x1000, 4, 20, 0x1000, 2, 0x1000, None) == binding.OMNI_ERR_SHAPE
    assert lib.omni_residual_load(None, 4, 64, 0x1000, 2, 0x1000, None) == binding.OMNI_ERR_NULL
    assert lib.omni_residual_load(0x1000, 4, 64, 0x1000, 0, None, None) == binding.OMNI_OK
