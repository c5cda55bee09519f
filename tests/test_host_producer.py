"""Host-side partial producer (omni_host_partial_attn) against the oracle.

The producer is host code (no GPU call), so these run without a GPU; the hybrid-batch test at the end
feeds its rows to the GPU merge and is marked gpu."""
import ctypes

import numpy as np
import pytest

from oracle import oracle
from paper_2603_12831_amd import binding, workloads as wl

TOL = {"f32": 1e-5, "bf16": 2e-3}


@pytest.fixture(scope="module", autouse=True)
def _lib():
    binding.load_library()


def rows_for(w, rng, n_rows, max_len):
    seq = rng.integers(0, w.batch, size=n_rows).astype(np.int32)
    end = np.array([rng.integers(0, w.ctx_len[s] + 1) for s in seq], dtype=np.int32)
    length = rng.integers(0, max_len + 1, size=n_rows)
    begin = np.maximum(end - length, 0).astype(np.int32)
    return seq, begin, end


def oracle_rows(w, seq, begin, end):
    items = [(int(s), h, int(b), int(e)) for s, b, e in zip(seq, begin, end) for h in range(w.num_q_heads)]
    o, lse = oracle.paged_attn_items(w.q, w.k_pool, w.v_pool, w.block_table, items, w.sm_scale, w.dtype, n_threads=8)
    return o.reshape(len(seq), w.num_q_heads, w.head_dim), lse.reshape(len(seq), w.num_q_heads)


def check_rows(got_o, got_l, exp_o, exp_l, tol):
    fin = np.isfinite(exp_l)
    assert np.array_equal(np.isfinite(got_l), fin)
    assert np.all(got_l[~fin] == -np.inf)
    assert np.all(got_o[~fin] == 0.0)
    assert float(np.max(np.abs(got_o[fin] - exp_o[fin]), initial=0.0)) <= tol
    assert float(np.max(np.abs(got_l[fin] - exp_l[fin]), initial=0.0)) <= tol


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(8, 2, 64), (8, 8, 128), (32, 8, 128), (16, 1, 128), (6, 3, 64), (12, 4, 128), (10, 2, 64),
                                   (14, 2, 128), (12, 1, 64)])
def test_rows_match_oracle(shape, dtype):
    """Ragged rows: unaligned begins and ends, empty rows, ranges longer than a 512-token slice (so that
    slices are folded), several rows per sequence."""
    hq, hkv, d = shape
    rng = np.random.default_rng([70, hq, hkv, d])
    lengths = rng.integers(1, 1500, size=7)
    w = wl.make_generic(70 + hq, lengths, hq, hkv, d, dtype=dtype, pool_factor=1.5)
    seq, begin, end = rows_for(w, rng, 24, 1400)
    begin[0], end[0] = 5, 5                                   # empty
    begin[1], end[1] = 0, int(w.ctx_len[seq[1]])              # whole context
    got_o, got_l = binding.omni_host_partial_attn(w.q, w.k_pool, w.v_pool, w.block_table, seq, begin, end,
                                                  w.sm_scale, dtype, n_threads=8)
    exp_o, exp_l = oracle_rows(w, seq, begin, end)
    check_rows(got_o, got_l, exp_o, exp_l, TOL[dtype])


@pytest.mark.parametrize("level", [1, 2, 3])
@pytest.mark.parametrize("dtype,shape", [("bf16", (8, 2, 128)), ("f32", (6, 1, 64)), ("bf16", (10, 2, 64)), ("f32", (12, 4, 128))])
def test_every_instruction_set_level(level, dtype, shape):
    """The plain, AVX2 and AVX-512 forms of the inner loops each against the oracle (a level the CPU lacks
    is refused, not emulated), and each independent of the thread count."""
    hq, hkv, d = shape
    rng = np.random.default_rng([75, hq, hkv, d])
    w = wl.make_generic(75 + hq, rng.integers(1, 1200, size=5), hq, hkv, d, dtype=dtype, pool_factor=1.5)
    seq, begin, end = rows_for(w, rng, 14, 1100)
    args = (w.q, w.k_pool, w.v_pool, w.block_table, seq, begin, end, w.sm_scale, dtype)
    st = binding.omni_host_partial_attn(*args, n_threads=4, check=False, isa_level=level)
    if st == binding.OMNI_ERR_UNSUPPORTED:
        pytest.skip("this CPU lacks instruction-set level %d" % level)
    got_o, got_l = binding.omni_host_partial_attn(*args, n_threads=4, isa_level=level)
    exp_o, exp_l = oracle_rows(w, seq, begin, end)
    check_rows(got_o, got_l, exp_o, exp_l, TOL[dtype])
    one_o, one_l = binding.omni_host_partial_attn(*args, n_threads=1, isa_level=level)
    assert np.array_equal(one_o, got_o) and np.array_equal(one_l, got_l)


def test_result_does_not_depend_on_thread_count():
    rng = np.random.default_rng(71)
    w = wl.make_generic(71, rng.integers(200, 2000, size=5), 8, 2, 128, dtype="bf16")
    seq, begin, end = rows_for(w, rng, 12, 2000)
    ref = binding.omni_host_partial_attn(w.q, w.k_pool, w.v_pool, w.block_table, seq, begin, end, w.sm_scale,
                                         "bf16", n_threads=1)
    for n in (2, 5, 16, 0):
        got = binding.omni_host_partial_attn(w.q, w.k_pool, w.v_pool, w.block_table, seq, begin, end,
                                             w.sm_scale, "bf16", n_threads=n)
        assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])


def test_absent_pages_and_clamped_ranges():
    """A table entry that names no pool page removes its 16 tokens; ends past the table are clamped."""
    w = wl.make_generic(72, [100, 260], 4, 2, 64, dtype="f32")
    table = w.block_table.copy()
    table[0, 2] = -1
    table[1, 5] = w.k_pool.shape[0] + 3
    cap = table.shape[1] * w.block_size
    seq = np.array([0, 1, 1], dtype=np.int32)
    begin = np.array([0, 0, -7], dtype=np.int32)
    end = np.array([100, 260, cap + 50], dtype=np.int32)
    got_o, got_l = binding.omni_host_partial_attn(w.q, w.k_pool, w.v_pool, table, seq, begin, end, w.sm_scale, "f32")
    # the oracle sees the same token sets as explicit pieces around the holes
    def union(seq_i, pieces):
        items = [(seq_i, h, b, e) for (b, e) in pieces for h in range(w.num_q_heads)]
        o, l = oracle.paged_attn_items(w.q, w.k_pool, w.v_pool, w.block_table, items, w.sm_scale, "f32")
        o = o.reshape(len(pieces), w.num_q_heads, -1).transpose(1, 0, 2)      # [head][piece][D]
        l = l.reshape(len(pieces), w.num_q_heads).T
        return oracle.merge(o, l, np.arange(w.num_q_heads + 1) * len(pieces))
    e0 = union(0, [(0, 32), (48, 100)])
    e1 = union(1, [(0, 80), (96, 260)])
    e2 = union(1, [(0, 80), (96, cap)])                        # clamped to the table's 17 pages
    for r, (eo, el) in enumerate([e0, e1, e2]):
        assert np.max(np.abs(got_o[r] - eo)) <= 1e-5 and np.max(np.abs(got_l[r] - el)) <= 1e-5


def test_argument_errors():
    w = wl.make_generic(73, [40], 4, 2, 64, dtype="f32")
    one = np.array([0], dtype=np.int32)
    args = dict(q=w.q, k_pool=w.k_pool, v_pool=w.v_pool, block_table=w.block_table, row_seq=one, row_begin=None,
                row_end=np.array([40], dtype=np.int32), sm_scale=w.sm_scale, dtype="f32", check=False)
    lib = binding.load_library()
    assert lib.omni_host_partial_attn(None) == binding.OMNI_ERR_NULL
    bad = dict(args, row_seq=np.array([1], dtype=np.int32))
    assert binding.omni_host_partial_attn(**bad) == binding.OMNI_ERR_SHAPE
    a = binding.omni_host_attn_args(n_rows=0)
    assert lib.omni_host_partial_attn(ctypes.byref(a)) == binding.OMNI_OK
    a = binding.omni_host_attn_args(n_rows=1, batch=1, num_q_heads=4, num_kv_heads=2, head_dim=64, block_size=16,
                                    max_blocks_per_seq=3, num_blocks=3)
    assert lib.omni_host_partial_attn(ctypes.byref(a)) == binding.OMNI_ERR_NULL
    w2 = wl.make_generic(73, [40], 4, 2, 64, dtype="f32")
    k32 = np.ascontiguousarray(w2.k_pool.reshape(w2.k_pool.shape[0], 2, 8, 128))
    with pytest.raises(binding.OmniError):
        binding.omni_host_partial_attn(w2.q, k32, k32, w2.block_table, one, None, np.array([40], dtype=np.int32),
                                       w2.sm_scale, "f32")


@pytest.mark.gpu
def test_hybrid_batch_with_host_produced_prefix_partials():
    """Config-4-shaped batch: the prefix partials of the best-effort rows come from the host producer
    (KV in host memory), the tails and the latency-sensitive rows from the GPU kernel; the merge must give
    attention over the full contexts."""
    import torch
    from paper_2603_12831_amd.runner import DeviceWorkload
    if not torch.cuda.is_available():
        pytest.fail("needs a GPU")
    w = wl.make_cfg4(n_ls=3, n_be=9, ls_lo=20, ls_hi=300, be_lo=300, be_hi=1500, tail_lo=5, tail_hi=70)
    seq = np.array([i for i, rs in enumerate(w.ext_ranges) for _ in rs], dtype=np.int32)
    begin = np.array([b for rs in w.ext_ranges for (b, _) in rs], dtype=np.int32)
    end = np.array([e for rs in w.ext_ranges for (_, e) in rs], dtype=np.int32)
    ext_o, ext_l = binding.omni_host_partial_attn(w.q, w.k_pool, w.v_pool, w.block_table, seq, begin, end,
                                                  w.sm_scale, w.dtype, n_threads=8)
    dw = DeviceWorkload(w, out_dtype="f32", ext_o=ext_o, ext_lse=ext_l, ext_offsets=wl.ext_row_offsets(w))
    dw.poison_outputs()
    dw.run()
    got_o, got_l = dw.results()
    full_end = np.max(np.stack([c.ctx_end for c in w.calls]), axis=0)
    exp_o, exp_l = oracle.paged_attn(w.q, w.k_pool, w.v_pool, w.block_table, np.zeros_like(full_end), full_end,
                                     w.sm_scale, w.dtype, n_threads=8)
    assert float(np.max(np.abs(got_o - exp_o))) <= TOL["bf16"]
    assert float(np.max(np.abs(got_l - exp_l))) <= TOL["bf16"]
