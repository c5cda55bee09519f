"""The allocation-free decode entry point (work list in the library's own static scratch) against the
ordinary entry point with a caller workspace: same kernels, so partial rows, merged rows and LSE must be
equal bit for bit — on two calls in a row, the second on a smaller batch (the scratch keeps the first
call's list), and both within the oracle's tolerance."""
import ctypes

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import oracle
from paper_2603_12831_amd import binding, workloads as wl
from paper_2603_12831_amd.runner import DeviceWorkload

pytestmark = pytest.mark.gpu


def _run(w, static):
    dw = DeviceWorkload(w, out_dtype="f32", workspace=not static)
    dw.poison_outputs()
    for c in dw.calls:
        args = dw.decode_args(c, binding.OMNI_KERNEL_AUTO, 0, False)
        if static:
            binding.omni_paged_decode_attn_static(args)
        else:
            binding.omni_paged_decode_attn_raw(args)
    dw.run_merge()
    o, lse = dw.results()
    parts = [(c["part_o"].cpu().numpy(), c["part_lse"].cpu().numpy()) for c in dw.calls]
    return o, lse, parts


def test_static_scratch_entry_matches_workspace_entry():
    if not torch.cuda.is_available():
        pytest.fail("needs a GPU")
    binding.load_library()
    big = wl.make_cfg3(batch=48, median=500, lo=1, hi=3000, chunk_tokens=256)
    big.calls[0].ctx_end[5] = 0                                   # an empty sequence among them
    small = wl.make_cfg3(seed=13, batch=7, median=200, lo=1, hi=700, chunk_tokens=128)
    for w in (big, small):                                        # the second call: fewer, shorter rows
        o_s, l_s, p_s = _run(w, static=True)
        o_w, l_w, p_w = _run(w, static=False)
        assert np.array_equal(o_s, o_w) and np.array_equal(l_s, l_w)
        for (po_s, pl_s), (po_w, pl_w) in zip(p_s, p_w):
            live = np.isfinite(pl_w)
            assert np.array_equal(pl_s, pl_w)
            assert np.array_equal(po_s[live], po_w[live])
        exp_o, exp_l = oracle.paged_attn(w.q, w.k_pool, w.v_pool, w.block_table, None, w.calls[0].ctx_end,
                                         w.sm_scale, w.dtype, n_threads=8)
        fin = np.isfinite(exp_l)
        assert np.array_equal(np.isfinite(l_s), fin)
        assert np.max(np.abs(o_s - exp_o)) <= 2e-3 and np.max(np.abs(l_s[fin] - exp_l[fin])) <= 2e-3


def test_static_scratch_entry_rejects_what_does_not_fit():
    if not torch.cuda.is_available():
        pytest.fail("needs a GPU")
    w = wl.make_generic(14, [40, 10], 8, 2, 128, dtype="bf16", chunk_tokens=16)
    dw = DeviceWorkload(w, out_dtype="f32", workspace=False)
    args = dw.decode_args(dw.calls[0], binding.OMNI_KERNEL_AUTO, 0, False)
    # claim a chunk stride whose list cannot fit the scratch: rejected on the host, nothing launched
    args.max_chunks = 65535
    assert binding.omni_decode_workspace_bytes(2, 65535, 2) > binding.OMNI_STATIC_SCRATCH_BYTES
    assert binding.omni_paged_decode_attn_static(args, check=False) == binding.OMNI_ERR_TOO_LARGE
    assert "scratch" in binding.omni_status_string(binding.OMNI_ERR_TOO_LARGE)
    assert binding.load_library().omni_paged_decode_attn_static(None, None) == binding.OMNI_ERR_NULL
