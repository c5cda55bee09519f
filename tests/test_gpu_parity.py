"""GPU parity: the HIP path, called through the C ABI, against the CPU fp64 oracle
on the same seeded inputs.

Tolerances (max abs error on O and on LSE, compared on fp32 outputs unless the
config asks for bf16 output):
  * fp32 inputs: 1e-5;
  * bf16 inputs with fp32 accumulation: 2e-3.
Integer work (which pages and slots are read) is checked bit-exactly through
the gather aid and through attention over integer-coded values.
"""
import math

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import oracle
from paper_2603_12831_amd import binding, workloads as wl
from paper_2603_12831_amd.runner import DeviceWorkload, to_device

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-3}
THREADS = 16
# (kernel selector, give a workspace): the vector kernel in its grid form and launched by a work list, and
# both launch forms of the automatic choice (which is the matrix-core kernel for bf16 at head_dim 128 and
# some head_dim-64 shapes, the vector kernel otherwise); workspace 2 = a workspace prepared once
# (omni_decode_plan) and passed as planned to every call
KERNELS = [pytest.param((binding.OMNI_KERNEL_VECTOR, False), id="vector"),
           pytest.param((binding.OMNI_KERNEL_VECTOR, True), id="vector-listed"),
           pytest.param((binding.OMNI_KERNEL_VECTOR, 2), id="vector-listed-planned"),
           pytest.param((binding.OMNI_KERNEL_AUTO, False), id="auto-grid"),
           pytest.param((binding.OMNI_KERNEL_AUTO, True), id="auto-persistent"),
           pytest.param((binding.OMNI_KERNEL_AUTO, 2), id="auto-persistent-planned")]
BENCH_FORM = (binding.OMNI_KERNEL_AUTO, True)          # what bench.py times: the list is rebuilt by every step
PLANNED_LIST = (binding.OMNI_KERNEL_AUTO, 2)           # the same kernel on a list built once


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("these tests need a GPU (run with -m gpu on an MI355X box)")
    binding.load_library()


def union_range(w):
    b = np.min(np.stack([c.ctx_begin for c in w.calls]), axis=0)
    e = np.max(np.stack([c.ctx_end for c in w.calls]), axis=0)
    return b, e


def expected_full(w, begin=None, end=None, seqs=None, heads=None):
    if begin is None:
        begin, end = union_range(w)
        if w.ext_ranges is not None:
            begin = np.zeros_like(begin)
    return oracle.paged_attn(w.q, w.k_pool, w.v_pool, w.block_table, begin, end, w.sm_scale, w.dtype,
                             seqs=seqs, heads=heads, n_threads=THREADS)


def ext_partials_from_oracle(w):
    """Externally produced partials of a hybrid batch: the oracle's fp64 partial over each
    prefix piece, rounded to fp32 (the format such partials arrive in)."""
    items = []
    for i, ranges in enumerate(w.ext_ranges):
        for (b, e) in ranges:
            for h in range(w.num_q_heads):
                items.append((i, h, b, e))
    o, lse = oracle.paged_attn_items(w.q, w.k_pool, w.v_pool, w.block_table, items, w.sm_scale, w.dtype,
                                     n_threads=THREADS)
    n = len(items) // w.num_q_heads
    return (o.reshape(n, w.num_q_heads, w.head_dim).astype(np.float32),
            lse.reshape(n, w.num_q_heads).astype(np.float32), wl.ext_row_offsets(w))


def check(got_o, got_l, exp_o, exp_l, tol, what=""):
    assert got_o.shape == exp_o.shape and got_l.shape == exp_l.shape
    fin = np.isfinite(exp_l)
    assert np.array_equal(np.isfinite(got_l), fin), "%s: finite pattern of LSE differs" % what
    assert np.all(got_l[~fin] == -np.inf)
    assert np.all(np.isfinite(got_o)), "%s: non-finite O" % what
    eo = float(np.max(np.abs(got_o - exp_o))) if got_o.size else 0.0
    el = float(np.max(np.abs(got_l[fin] - exp_l[fin]))) if fin.any() else 0.0
    assert eo <= tol and el <= tol, "%s: max abs err O %.3g LSE %.3g > %.1g" % (what, eo, el, tol)
    return eo, el


def run_and_check(w, kernel, out_dtype="f32", tol=None, ext=None, expected=None):
    ext = ext or (None, None, None)
    dw = DeviceWorkload(w, out_dtype=out_dtype, ext_o=ext[0], ext_lse=ext[1], ext_offsets=ext[2],
                        workspace=kernel[1])
    dw.poison_outputs()
    dw.run(kernel=kernel[0])
    got_o, got_l = dw.results()
    assert dw.abandoned_waves() == 0
    exp_o, exp_l = expected if expected is not None else expected_full(w)
    return check(got_o, got_l, exp_o, exp_l, tol or TOL[w.dtype], w.name), dw


# ---------------------------------------------------------------------------
# config 1 (tiny fp32, two chunks per sequence, merged) and its partials
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("kernel", KERNELS)
def test_cfg1_merged_and_partials(kernel):
    w = wl.make_cfg1()
    (_, dw) = run_and_check(w, kernel)
    for c, dc in zip(w.calls, dw.calls):
        exp_o, exp_l = expected_full(w, c.ctx_begin, c.ctx_end)
        po = dc["part_o"].cpu().numpy().astype(np.float64)[:, 0]
        pl = dc["part_lse"].cpu().numpy().astype(np.float64)[:, 0]
        check(po, pl, exp_o, exp_l, 1e-5, "cfg1 partial")


# ---------------------------------------------------------------------------
# scaled-down versions of configs 2-5: several pages per wave, ragged tails
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("kernel", KERNELS)
def test_small_cfg2_direct_bf16_output(kernel):
    w = wl.make_cfg2(batch=5, lo=30, hi=700)
    run_and_check(w, kernel, out_dtype="bf16")
    run_and_check(w, kernel, out_dtype="f32")


@pytest.mark.parametrize("kernel", KERNELS)
@pytest.mark.parametrize("chunk", [64, 256, 1024])
def test_small_cfg3_chunked(kernel, chunk):
    w = wl.make_cfg3(batch=12, median=300, lo=1, hi=1500, chunk_tokens=chunk)
    (_, dw) = run_and_check(w, kernel)
    # every partial against the oracle's partial over the same chunk
    c = w.calls[0]
    po = dw.calls[0]["part_o"].cpu().numpy().astype(np.float64)
    pl = dw.calls[0]["part_lse"].cpu().numpy().astype(np.float64)
    for ci in range(c.max_chunks):
        b = np.minimum(c.ctx_begin + ci * chunk, c.ctx_end)
        e = np.minimum(b + chunk, c.ctx_end)
        exp_o, exp_l = expected_full(w, b, e)
        live = e > b
        assert np.all(pl[~live, ci] == -np.inf)
        check(po[live, ci], pl[live, ci], exp_o[live], exp_l[live], 2e-3, "chunk %d" % ci)


@pytest.mark.parametrize("kernel", KERNELS)
def test_small_cfg5_wide_softmax_range(kernel):
    w = wl.make_cfg5(batch=2, ctx=2048 + 48, chunk_tokens=256)
    run_and_check(w, kernel)


@pytest.mark.parametrize("kernel", KERNELS)
def test_small_cfg4_hybrid(kernel):
    w = wl.make_cfg4(n_ls=3, n_be=9, ls_lo=20, ls_hi=300, be_lo=300, be_hi=900, tail_lo=5, tail_hi=70)
    run_and_check(w, kernel, ext=ext_partials_from_oracle(w))


@pytest.mark.parametrize("kernel", KERNELS)
@pytest.mark.parametrize("shape", [(8, 8, 64), (8, 1, 128), (16, 1, 64), (6, 3, 128), (4, 4, 128), (32, 2, 128)])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_head_layouts(kernel, shape, dtype):
    hq, hkv, d = shape
    w = wl.make_generic(21, [1, 16, 17, 200, 333], hq, hkv, d, dtype=dtype, chunk_tokens=128, pool_factor=1.5)
    run_and_check(w, kernel)


@pytest.mark.parametrize("kernel", KERNELS)
@pytest.mark.parametrize("shape", [(8, 8), (4, 2), (6, 2), (16, 4), (12, 4), (32, 8)])
def test_head_dim_64_bf16(kernel, shape):
    """bf16 head_dim 64 with an even number of kv heads and up to four query heads per kv head runs on the
    matrix-core kernel as kv-head pairs (the automatic choice): ragged ranges that start past token 0,
    chunked and unchunked, rows written as partials, as final fp32 rows and as final bf16 rows."""
    hq, hkv = shape
    rng = np.random.default_rng([67, hq, hkv])
    lengths = rng.integers(1, 700, size=11)
    lengths[:3] = [1, 16, 33]
    begin = rng.integers(0, 2, size=11) * rng.integers(0, 30, size=11)
    w = wl.make_generic(67 + hq, lengths + begin, hq, hkv, 64, dtype="bf16", ctx_begin=begin, pool_factor=1.4)
    exp = expected_full(w, begin=w.calls[0].ctx_begin, end=w.calls[0].ctx_end)
    if kernel[0] == binding.OMNI_KERNEL_AUTO:
        dw = DeviceWorkload(w, workspace=kernel[1])
        args = dw.decode_args(dw.calls[0], kernel[0], 0, False)
        assert binding.omni_decode_kernel_name(args).startswith("decode_mfma")
    run_and_check(w, kernel, expected=exp, out_dtype="f32")
    run_and_check(w, kernel, expected=exp, out_dtype="bf16",
                  tol=TOL["bf16"] + float(np.max(np.abs(exp[0]))) * 2.0 ** -9)
    w.calls[0].chunk_tokens, w.calls[0].max_chunks = 96, 8
    (_, dw) = run_and_check(w, kernel, expected=exp)
    # every partial row against the oracle's partial over the same chunk
    c = w.calls[0]
    po = dw.calls[0]["part_o"].cpu().numpy().astype(np.float64)
    pl = dw.calls[0]["part_lse"].cpu().numpy().astype(np.float64)
    for ci in range(c.max_chunks):
        b = np.minimum(c.ctx_begin + ci * 96, c.ctx_end)
        e = np.minimum(b + 96, c.ctx_end)
        live = e > b
        assert np.all(pl[~live, ci] == -np.inf)
        if live.any():
            exp_o, exp_l = expected_full(w, b, e)
            check(po[live, ci], pl[live, ci], exp_o[live], exp_l[live], 2e-3, "chunk %d" % ci)


# ---------------------------------------------------------------------------
# edge cases
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("kernel", KERNELS)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_edge_lengths_and_offsets(kernel, dtype):
    lengths = [1, 2, 15, 16, 17, 31, 32, 33, 63, 64, 65, 100, 0, 129, 1000]
    begins = [0, 1, 14, 0, 16, 5, 31, 32, 0, 63, 17, 99, 0, 128, 333]
    w = wl.make_generic(31, np.maximum(lengths, 1), 8, 2, 128, dtype=dtype, pool_factor=2.0)
    w.calls[0].ctx_end = np.array(lengths, dtype=np.int32)
    w.calls[0].ctx_begin = np.array(begins, dtype=np.int32)
    run_and_check(w, kernel)
    # the same ranges, chunked: chunk boundaries relative to a non-aligned begin
    w.calls[0].chunk_tokens, w.calls[0].max_chunks = 64, 16
    run_and_check(w, kernel)


@pytest.mark.parametrize("kernel", KERNELS)
def test_empty_and_reversed_ranges_give_zero_and_minus_inf(kernel):
    w = wl.make_generic(32, [40, 40, 40], 4, 2, 128, dtype="bf16")
    w.calls[0].ctx_begin = np.array([0, 40, 30], dtype=np.int32)
    w.calls[0].ctx_end = np.array([0, 40, 10], dtype=np.int32)
    for chunk, mc in [(0, 1), (16, 4)]:
        w.calls[0].chunk_tokens, w.calls[0].max_chunks = chunk, mc
        dw = DeviceWorkload(w, out_dtype="f32", workspace=kernel[1])
        dw.poison_outputs()
        dw.run(kernel=kernel[0])
        o, l = dw.results()
        assert np.all(o == 0) and np.all(l == -np.inf)


@pytest.mark.parametrize("kernel", KERNELS)
def test_chunks_beyond_max_chunks_are_not_attended(kernel):
    w = wl.make_generic(33, [300, 90], 8, 2, 128, dtype="bf16")
    w.calls[0].chunk_tokens, w.calls[0].max_chunks = 64, 2
    exp = expected_full(w, np.zeros(2, dtype=np.int32), np.array([128, 90], dtype=np.int32))
    run_and_check(w, kernel, expected=exp)


@pytest.mark.parametrize("kernel", KERNELS)
def test_absent_pages_and_clamped_ranges(kernel):
    """A table entry outside the pool removes its 16 tokens; ctx_end beyond the table is clamped."""
    w = wl.make_generic(34, [160, 64], 8, 2, 128, dtype="bf16")
    bt = w.block_table.copy()
    bt[0, 3] = -1
    bt[0, 7] = w.num_blocks + 5
    w2 = wl.make_generic(34, [160, 64], 8, 2, 128, dtype="bf16")
    w2.block_table = bt
    w2.calls[0].ctx_end = np.array([160, 100000], dtype=np.int32)      # row 1 has 4 pages: clamps to 64
    # expected: merge of the oracle's partials over the surviving ranges
    pieces = [(0, 48), (64, 112), (128, 160)]
    o0, l0 = [], []
    for (b, e) in pieces:
        o, l = expected_full(w, np.array([b, 0]), np.array([e, 0]), seqs=[0])
        o0.append(o[0]); l0.append(l[0])
    exp_o, exp_l = expected_full(w)
    for h in range(w.num_q_heads):
        mo, ml = oracle.merge(np.stack([x[h] for x in o0]), [x[h] for x in l0], [0, 3])
        exp_o[0, h], exp_l[0, h] = mo[0], ml[0]
    run_and_check(w2, kernel, expected=(exp_o, exp_l))


@pytest.mark.parametrize("kernel", KERNELS)
def test_garbage_outside_the_range_is_never_used(kernel):
    """Slots past ctx_end, slots before ctx_begin and unused pages hold NaN: results unchanged."""
    w = wl.make_generic(35, [5, 40, 100, 257], 8, 2, 128, dtype="bf16", pool_factor=1.5)
    begins = np.array([0, 7, 33, 1], dtype=np.int32)
    w.calls[0].ctx_begin = begins
    exp = expected_full(w)
    nan = np.uint16(0x7FC0)
    keep = np.zeros(w.k_pool.shape[:1] + (16,), dtype=bool)
    for i, L in enumerate(w.ctx_len):
        for t in range(int(begins[i]), int(L)):
            keep[w.block_table[i, t // 16], t % 16] = True
    for pool in (w.k_pool, w.v_pool):
        pool[~keep[:, None, :].repeat(w.num_kv_heads, axis=1)] = nan
    for chunk, mc in [(0, 1), (32, 9)]:
        w.calls[0].chunk_tokens, w.calls[0].max_chunks = chunk, mc
        run_and_check(w, kernel, expected=exp)


def relocate_pools(dw, n_pages_big):
    """The workload's pages moved to the far end of pools of n_pages_big pages (allocated on the device: the
    rest holds zeros), the block table shifted with them."""
    small = dw.k_pools[0].shape[0]
    base = n_pages_big - small
    for pools in (dw.k_pools, dw.v_pools):
        big = torch.zeros((n_pages_big,) + tuple(pools[0].shape[1:]), dtype=pools[0].dtype, device=dw.device)
        big[base:].copy_(pools[0])
        pools[0] = big
    dw.block_table = torch.where(dw.block_table >= 0, dw.block_table + base, dw.block_table)
    dw._arg_cache.clear()
    return base


@pytest.mark.parametrize("kernel", KERNELS)
@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("bf16", 64), ("f32", 128)])
def test_pages_beyond_4_gib_into_the_pools(kernel, dtype, d):
    """Byte offsets of pages do not fit 32 bits: every page of the batch lies past 4 GiB in K and V pools of 4.5 GiB."""
    hkv = 2
    w = wl.make_generic(36, [700, 33, 2048, 1, 1500], 8, hkv, d, dtype=dtype, chunk_tokens=512, pool_factor=1.5)
    exp = expected_full(w)
    page_bytes = hkv * 16 * d * (2 if dtype == "bf16" else 4)
    n_big = (9 << 29) // page_bytes
    dw = DeviceWorkload(w, workspace=kernel[1])
    base = relocate_pools(dw, n_big)
    assert base * page_bytes > (1 << 32)
    dw.poison_outputs()
    dw.run(kernel=kernel[0])
    got_o, got_l = dw.results()
    assert dw.abandoned_waves() == 0
    check(got_o, got_l, exp[0], exp[1], TOL[dtype], "pools of 4.5 GiB")
    # the gather aid reads the same pages bit for bit
    c = dw.calls[0]
    args = binding.make_decode_args(dw.q, dw.k_pools[0], dw.v_pools[0], dw.block_table, c["begin"], c["end"],
                                    sm_scale=w.sm_scale, chunk_tokens=c["chunk_tokens"], max_chunks=c["max_chunks"],
                                    part_o=c["part_o"], part_lse=c["part_lse"])
    L = int(w.ctx_len[2])
    k_out = torch.zeros((L, hkv, d), dtype=dw.q.dtype, device=dw.device)
    v_out = torch.zeros_like(k_out)
    binding.omni_debug_gather_kv(args, 2, k_out, v_out)
    torch.cuda.synchronize()
    ek, ev = oracle.gather_kv(w.k_pool, w.v_pool, w.block_table, 2, 0, L)
    view = (lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)) if dtype == "bf16" else (lambda t: t.cpu().numpy())
    assert np.array_equal(view(k_out).view(np.uint8), ek.view(np.uint8))
    assert np.array_equal(view(v_out).view(np.uint8), ev.view(np.uint8))
    del dw
    torch.cuda.empty_cache()


# ---------------------------------------------------------------------------
# integer work: gather and index-revealing attention are bit-exact
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_gather_is_bit_exact(dtype):
    w = wl.make_generic(41, [1, 16, 17, 100, 511], 8, 2, 64, dtype=dtype, pool_factor=2.0)
    begins = np.array([0, 0, 3, 16, 255], dtype=np.int32)
    w.calls[0].ctx_begin = begins
    dw = DeviceWorkload(w)
    c = dw.calls[0]
    args = binding.make_decode_args(dw.q, dw.k_pools[0], dw.v_pools[0], dw.block_table, c["begin"], c["end"],
                                    sm_scale=w.sm_scale, part_o=c["part_o"], part_lse=c["part_lse"])
    for i, L in enumerate(w.ctx_len):
        n = int(L - begins[i])
        k_out = torch.zeros((n, w.num_kv_heads, w.head_dim), dtype=dw.q.dtype, device=dw.device)
        v_out = torch.zeros_like(k_out)
        binding.omni_debug_gather_kv(args, i, k_out, v_out)
        torch.cuda.synchronize()
        ek, ev = oracle.gather_kv(w.k_pool, w.v_pool, w.block_table, i, int(begins[i]), int(L))
        view = (lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)) if dtype == "bf16" else \
               (lambda t: t.cpu().numpy())
        assert np.array_equal(view(k_out).view(np.uint8), ek.view(np.uint8))
        assert np.array_equal(view(v_out).view(np.uint8), ev.view(np.uint8))


@pytest.mark.parametrize("kernel", KERNELS)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_index_revealing_attention_is_exact(kernel, dtype):
    """q = 0 makes every weight exactly 1/n; V rows hold small integer codes of (sequence, token),
    distinct per dim group, so n * O must be the exact integer sum of the codes of the tokens read."""
    lengths = [1, 16, 17, 64, 128, 250]
    w = wl.make_generic(42, lengths, 8, 2, 128, dtype=dtype, pool_factor=2.0)
    begins = np.array([0, 0, 5, 16, 1, 100], dtype=np.int32)
    w.calls[0].ctx_begin = begins
    q = np.zeros(w.q.shape, dtype=np.float32)
    v = np.full(w.v_pool.shape, 200.0, dtype=np.float32)      # a wrong page or slot shows up as 200
    for i, L in enumerate(lengths):
        for t in range(L):
            v[w.block_table[i, t // 16], :, t % 16, :] = (t % 64) + (i % 2)          # <= 64: exact in bf16
    w.q = q if dtype == "f32" else wl.f32_to_bf16_bits(q)
    w.v_pool = v if dtype == "f32" else wl.f32_to_bf16_bits(v)
    dw = DeviceWorkload(w, out_dtype="f32", workspace=kernel[1])
    dw.run(kernel=kernel[0])
    o, lse = dw.results()
    for i, L in enumerate(lengths):
        n = L - int(begins[i])
        want = sum((t % 64) + (i % 2) for t in range(int(begins[i]), L))
        # power-of-two counts divide exactly; otherwise allow the division's rounding only
        assert np.all(np.abs(o[i] * n - want) <= 1e-6 * max(1, want) * 8), (i, o[i, 0, 0] * n, want)
        assert np.all(np.abs(lse[i] - math.log(n)) < 1e-6)


@pytest.mark.parametrize("kernel", KERNELS)
def test_deterministic_and_placement_independent(kernel):
    w = wl.make_cfg3(batch=8, median=400, lo=10, hi=1500, chunk_tokens=256)
    dw = DeviceWorkload(w, out_dtype="f32", workspace=kernel[1])
    dw.run(kernel=kernel[0])
    o1, l1 = dw.results()
    dw.poison_outputs()
    dw.run(kernel=kernel[0])
    o2, l2 = dw.results()
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)
    # move every page to a new physical home, table updated: bit-identical outputs
    perm = np.random.default_rng(0).permutation(w.num_blocks)
    k2, v2 = np.empty_like(w.k_pool), np.empty_like(w.v_pool)
    k2[perm], v2[perm] = w.k_pool, w.v_pool
    w.k_pool, w.v_pool = k2, v2
    w.block_table = np.where(w.block_table >= 0, perm[np.maximum(w.block_table, 0)], -1).astype(np.int32)
    dw3 = DeviceWorkload(w, out_dtype="f32", workspace=kernel[1])
    dw3.run(kernel=kernel[0])
    o3, l3 = dw3.results()
    assert np.array_equal(o1, o3) and np.array_equal(l1, l3)


@pytest.mark.parametrize("kernel", KERNELS[3:])
@pytest.mark.parametrize("shape", [(16, 1, 128), (8, 8, 128), (6, 3, 128), (24, 3, 128), (32, 2, 128),
                                   (56, 8, 128), (28, 4, 128), (16, 2, 128)])
def test_matrix_core_group_sizes(kernel, shape):
    """GQA ratios 16, 1, 2, 8 and 16 (the last needs the large LDS window) with ragged chunked contexts; then
    the layer shapes of the paper's two models: 56 q / 8 kv heads (ratio 7) whole and halved for two GPUs,
    64 q / 8 kv heads quartered for four."""
    hq, hkv, d = shape
    rng = np.random.default_rng(hq * 100 + hkv)
    lengths = rng.integers(1, 900, size=9)
    w = wl.make_generic(61, lengths, hq, hkv, d, dtype="bf16", chunk_tokens=160, pool_factor=1.3)
    run_and_check(w, kernel)
    w.calls[0].chunk_tokens, w.calls[0].max_chunks = 0, 1
    run_and_check(w, kernel)


@pytest.mark.parametrize("kernel", KERNELS)
def test_one_context_of_131072_tokens(kernel):
    """8 192 pages in one table row: as one range (4 096 steps of one item), as 128 chunks of 1 024 and as
    2 048 chunks of 64 (the merge then folds 2 048 rows per head); a second, short sequence beside it."""
    w = wl.make_generic(64, [131072, 77], 8, 2, 128, dtype="bf16", pool_factor=1.1, boost_frac=0.01, boost=8.0)
    exp = expected_full(w)
    for chunk, mc in [(0, 1), (1024, 128), (64, 2048)]:
        w.calls[0].chunk_tokens, w.calls[0].max_chunks = chunk, mc
        run_and_check(w, kernel, expected=exp)


def test_work_list_with_many_sequences():
    """More sequences than the list kernel keeps in LDS (2048), most of them short, some empty."""
    rng = np.random.default_rng(62)
    lengths = rng.integers(0, 40, size=2500)
    lengths[::97] = 0
    lengths[5] = 700
    w = wl.make_generic(62, np.maximum(lengths, 1), 4, 1, 128, dtype="bf16", chunk_tokens=32)
    w.calls[0].ctx_end = lengths.astype(np.int32)
    run_and_check(w, BENCH_FORM)
    run_and_check(w, PLANNED_LIST)
    run_and_check(w, (binding.OMNI_KERNEL_AUTO, False))


def test_ticket_handover_across_item_lengths():
    """More items than resident workgroups, with lengths that put 1 to 10 steps of 32 tokens in an item
    (a wave then has none, one, two or three steps of it) in every order: the hand-over from one item to
    the next - ticket drawn early for single-step items, late otherwise, picked up by each wave on its
    own - must serve every item exactly once.  Run twice on one work list."""
    rng = np.random.default_rng(63)
    pool = np.array([1, 16, 31, 33, 64, 65, 96, 128, 129, 160, 161, 192, 224, 256, 257, 288, 300, 320])
    lengths = rng.choice(pool, size=440)
    begin = rng.integers(0, 2, size=440) * rng.integers(0, 20, size=440)
    w = wl.make_generic(63, lengths + begin, 8, 4, 128, dtype="bf16", ctx_begin=begin)
    exp = expected_full(w, begin=w.calls[0].ctx_begin, end=w.calls[0].ctx_end)
    (_, _), dw = run_and_check(w, BENCH_FORM, expected=exp)
    dw.poison_outputs()
    dw.run(kernel=BENCH_FORM[0])
    got_o, got_l = dw.results()
    check(got_o, got_l, exp[0], exp[1], TOL["bf16"], "second pass")
    # same ranges cut into 64-token chunks: items of one and two steps only, several thousand of them
    w.calls[0].chunk_tokens, w.calls[0].max_chunks = 64, 6
    run_and_check(w, BENCH_FORM, expected=exp)


@pytest.mark.parametrize("shape", [(6, 3, 401), (16, 1, 1100), (5, 5, 230), (32, 2, 600)])
def test_short_ranges_four_to_a_ticket(shape):
    """Enough ranges of up to 256 tokens for every workgroup to get a ticket of four of them (one per wave),
    behind a few longer ones that are still one item per ticket: item counts that leave the last ticket
    partly filled, kv-head counts that make a ticket straddle ranges of different lengths, waves with
    one to nine steps under one ticket, group sizes 1 to 16; final rows written directly (bf16 and fp32)
    and partial rows merged."""
    hq, hkv, batch = shape
    rng = np.random.default_rng([64, hq, hkv])
    lengths = rng.integers(1, 257, size=batch)
    lengths[rng.integers(0, batch, size=7)] = rng.integers(257, 700, size=7)
    begin = rng.integers(0, 2, size=batch) * rng.integers(0, 40, size=batch)
    w = wl.make_generic(64 + hq, lengths + begin, hq, hkv, 128, dtype="bf16", ctx_begin=begin)
    exp = expected_full(w, begin=w.calls[0].ctx_begin, end=w.calls[0].ctx_end)
    # rows stored as bf16 carry that format's rounding (half an ulp: 2^-9 relative) on top of the bound
    run_and_check(w, BENCH_FORM, expected=exp, out_dtype="bf16",
                  tol=TOL["bf16"] + float(np.max(np.abs(exp[0]))) * 2.0 ** -9)
    run_and_check(w, BENCH_FORM, expected=exp, out_dtype="f32")
    w.calls[0].chunk_tokens, w.calls[0].max_chunks = 128, 6
    run_and_check(w, BENCH_FORM, expected=exp)


@pytest.mark.parametrize("case", range(24))
def test_seeded_random_batches(case):
    """Seeded random batches through the form bench.py times: kv-head counts 1-8, group sizes 1-16, batches
    of many short ranges, few long ones and mixtures, ranges that start past token 0, unchunked and chunked
    (64 .. 1024 tokens, sometimes with a spare chunk slot); every batch is run twice on its buffers."""
    rng = np.random.default_rng([65, case])
    hkv = int(rng.choice([1, 2, 3, 4, 8]))
    hq = hkv * int(rng.choice([1, 2, 4, 5, 8, 16]))
    kind = case % 4
    if kind == 0:
        lengths = rng.integers(1, 300, size=int(rng.integers(300, 1500)))
    elif kind == 1:
        lengths = rng.integers(1, 2500, size=int(rng.integers(50, 400)))
    elif kind == 2:
        n = int(rng.integers(200, 900))
        lengths = np.where(rng.random(n) < 0.1, rng.integers(300, 3000, size=n), rng.integers(1, 260, size=n))
    else:
        lengths = rng.integers(1, 6000, size=int(rng.integers(1, 40)))
    lengths = lengths[:max(1, 40000 // hq)]                  # keeps the oracle quick
    begin = (rng.random(len(lengths)) < 0.3) * rng.integers(0, 50, size=len(lengths))
    w = wl.make_generic(6500 + case, lengths + begin, hq, hkv, 128, dtype="bf16", ctx_begin=begin)
    chunk = int(rng.choice([0, 64, 128, 256, 512, 1024]))
    if chunk:
        longest = int((lengths + begin).max())
        w.calls[0].chunk_tokens, w.calls[0].max_chunks = chunk, (longest + chunk - 1) // chunk + int(rng.integers(0, 2))
    exp = expected_full(w, begin=w.calls[0].ctx_begin, end=w.calls[0].ctx_end)
    for form in (BENCH_FORM, PLANNED_LIST):
        (_, _), dw = run_and_check(w, form, expected=exp)
        dw.poison_outputs()
        dw.run(kernel=form[0])
        got_o, got_l = dw.results()
        check(got_o, got_l, exp[0], exp[1], TOL["bf16"], "second pass")
        assert dw.abandoned_waves() == 0


def test_step_captured_in_a_graph_replays_exactly():
    """One whole step (work list, decode attention, merge) recorded into a graph on a side stream and
    replayed several times, with other work of the library and synchronisations in between: every replay
    must reproduce the directly launched step bit for bit (the work list's counters are put back by the
    kernel itself, nothing is allocated or cleared by the host between calls)."""
    w = wl.make_cfg3(batch=40, median=600, lo=1, hi=4000, chunk_tokens=512)
    exp = expected_full(w)
    (_, _), dw = run_and_check(w, BENCH_FORM, expected=exp)
    eager_o, eager_l = dw.results()
    other = DeviceWorkload(wl.make_generic(66, [300, 17, 1200], 8, 2, 128, dtype="bf16", chunk_tokens=256), out_dtype="f32")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        dw.run(kernel=BENCH_FORM[0])                           # warm-up on the capturing stream
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        dw.run(kernel=BENCH_FORM[0])
    for replay in range(4):
        dw.poison_outputs()
        other.run(kernel=BENCH_FORM[0])                        # unrelated launches between replays
        torch.cuda.synchronize()
        graph.replay()
        got_o, got_l = dw.results()
        assert np.array_equal(got_o, eager_o) and np.array_equal(got_l, eager_l), "replay %d differs" % replay
        assert dw.abandoned_waves() == 0
    check(got_o, got_l, exp[0], exp[1], TOL["bf16"], "graph replay")


def test_workspace_too_small_is_rejected():
    w = wl.make_generic(63, [100, 50], 8, 2, 128, dtype="bf16", chunk_tokens=32)
    dw = DeviceWorkload(w, out_dtype="f32")
    c = dw.calls[0]
    small = torch.empty(64, dtype=torch.uint8, device=dw.device)
    st = binding.omni_paged_decode_attn(dw.q, dw.k_pools[0], dw.v_pools[0], dw.block_table, c["begin"], c["end"],
                                        sm_scale=w.sm_scale, chunk_tokens=32, max_chunks=c["max_chunks"],
                                        part_o=c["part_o"], part_lse=c["part_lse"], workspace=small, check=False)
    assert st == binding.OMNI_ERR_SHAPE
    # the vector kernel ignores a workspace
    wf = wl.make_generic(63, [100, 50], 8, 2, 64, dtype="f32", chunk_tokens=32)
    run_and_check(wf, (binding.OMNI_KERNEL_AUTO, True))


def test_plan_once_serves_many_passes():
    """One work list (omni_decode_plan) reused by several attention passes over the same ranges,
    as the layers of one decoding iteration would: results equal the self-planning call bit for bit."""
    w = wl.make_cfg3(batch=24, median=500, lo=1, hi=3000, chunk_tokens=512)
    w.calls[0].ctx_end[3] = 0                                   # an empty sequence among them
    ref = DeviceWorkload(w, out_dtype="f32")
    ref.run()
    o_ref, l_ref = ref.results()
    check(o_ref, l_ref, *expected_full(w), 2e-3, "self-planned")
    dw = DeviceWorkload(w, out_dtype="f32")
    dw.plan()
    for layer in range(3):
        dw.poison_outputs()
        dw.run_attention(planned=True)
        dw.run_merge()
        o, l = dw.results()
        assert np.array_equal(o, o_ref) and np.array_equal(l, l_ref)
    # another "layer": different q and KV, same ranges, same plan
    w2 = wl.make_cfg3(batch=24, median=500, lo=1, hi=3000, chunk_tokens=512)
    w2.calls = w.calls
    w2.q = wl._normal(w.q.shape, [77, 1], 1.0, "bf16")
    w2.k_pool = wl._normal(w.k_pool.shape, [77, 2], 1.0, "bf16")
    w2.v_pool = wl._normal(w.v_pool.shape, [77, 3], 1.0, "bf16")
    dw.q.copy_(to_device(w2.q, "bf16", dw.device))
    dw.k_pools[0].copy_(to_device(w2.k_pool, "bf16", dw.device))
    dw.v_pools[0].copy_(to_device(w2.v_pool, "bf16", dw.device))
    dw.poison_outputs()
    dw.run_attention(planned=True)
    dw.run_merge()
    o, l = dw.results()
    check(o, l, *expected_full(w2), 2e-3, "second layer on a reused plan")


# ---------------------------------------------------------------------------
# the merge on its own
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("out_dtype", [torch.float32, torch.bfloat16])
def test_merge_random_sources(d, out_dtype):
    rng = np.random.default_rng(50 + d)
    B, H = 37, 6
    dev = torch.device("cuda:0")
    # source 0: CSR with 0..5 rows per sequence; source 1: dense 3 rows; source 2: dense 1 row; source 3: CSR
    srcs_np, kinds = [], ("csr", 3, 1, "csr")
    for kind in kinds:
        if kind == "csr":
            counts = rng.integers(0, 6, size=B)
            off = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
        else:
            off = np.arange(B + 1, dtype=np.int32) * kind
        n = int(off[-1])
        o = rng.standard_normal((n, H, d)).astype(np.float32)
        lse = (rng.standard_normal((n, H)) * 6).astype(np.float32)
        lse[rng.random((n, H)) < 0.25] = -np.inf
        for i in (0, 11):                                            # sequences with no live partial at all
            lse[off[i]:off[i + 1]] = -np.inf
        o[lse == -np.inf] = np.nan                                   # must never be read
        srcs_np.append((o, lse, off))
    srcs_t = [(torch.from_numpy(o).to(dev), torch.from_numpy(lse).to(dev),
               torch.from_numpy(off).to(dev) if kind == "csr" else None, 0 if kind == "csr" else kind)
              for (o, lse, off), kind in zip(srcs_np, kinds)]
    for n_srcs in (1, 2, 4):
        out_o = torch.full((B, H, d), float("nan"), dtype=out_dtype, device=dev)
        out_l = torch.full((B, H), float("nan"), dtype=torch.float32, device=dev)
        binding.omni_merge_partials(B, H, d, srcs_t[:n_srcs], out_o, out_l)
        torch.cuda.synchronize()
        po, pl, offs = [], [], [0]
        for i in range(B):
            for h in range(H):
                for (o, lse, off) in srcs_np[:n_srcs]:
                    po.append(np.nan_to_num(o[off[i]:off[i + 1], h], nan=0.0))
                    pl.append(lse[off[i]:off[i + 1], h])
                offs.append(offs[-1] + sum(int(s[2][i + 1] - s[2][i]) for s in srcs_np[:n_srcs]))
        exp_o, exp_l = oracle.merge(np.concatenate(po), np.concatenate(pl), offs)
        tol = 1e-5 if out_dtype == torch.float32 else 2.0 ** -8 * 5
        check(out_o.float().cpu().numpy().astype(np.float64).reshape(B * H, d),
              out_l.cpu().numpy().astype(np.float64).reshape(B * H), exp_o, exp_l, tol, "merge")
        assert np.all(exp_l[:H] == -np.inf)                          # sequence 0 had nothing live
        # without the LSE output
        out2 = torch.full((B, H, d), float("nan"), dtype=out_dtype, device=dev)
        binding.omni_merge_partials(B, H, d, srcs_t[:n_srcs], out2, None)
        torch.cuda.synchronize()
        assert torch.equal(out2, out_o)


# ---------------------------------------------------------------------------
# full-size configurations, in the launch configuration the benchmark times
# ---------------------------------------------------------------------------
def test_full_cfg2():
    w = wl.make_cfg2(workers=THREADS)
    (eo, el), _ = run_and_check(w, BENCH_FORM, out_dtype="bf16")
    print("cfg2 max abs err O %.3g LSE %.3g" % (eo, el))


def test_full_cfg3():
    w = wl.make_cfg3(workers=THREADS)
    (eo, el), dw = run_and_check(w, BENCH_FORM, out_dtype="f32")
    print("cfg3 max abs err O %.3g LSE %.3g" % (eo, el))
    # the bf16 output the config asks for is the correctly rounded fp32 result, up to one step
    exp_o, _ = expected_full(w)
    dwb = DeviceWorkload(w, out_dtype="bf16")
    dwb.run()
    # the grid form and the planned-list form on the full size too
    run_and_check(w, (binding.OMNI_KERNEL_AUTO, False), out_dtype="f32")
    run_and_check(w, PLANNED_LIST, out_dtype="f32")
    ob, _ = dwb.results()
    assert np.max(np.abs(ob - exp_o) / np.maximum(np.abs(exp_o), 2.0 ** -6)) <= 2.0 ** -8 + 1e-3


def test_full_cfg4():
    w = wl.make_cfg4(workers=THREADS)
    (eo, el), _ = run_and_check(w, BENCH_FORM, out_dtype="f32", ext=ext_partials_from_oracle(w))
    print("cfg4 max abs err O %.3g LSE %.3g" % (eo, el))


def test_full_cfg5_all_sequences():
    """Every head of all 32 sequences at the full size (32 chunks of 1024 tokens merged per row)."""
    w = wl.make_cfg5(workers=THREADS)
    dw = DeviceWorkload(w, out_dtype="f32")
    dw.poison_outputs()
    dw.run()
    got_o, got_l = dw.results()
    assert dw.abandoned_waves() == 0
    exp_o, exp_l = expected_full(w)
    eo, el = check(got_o, got_l, exp_o, exp_l, 2e-3, "cfg5")
    print("cfg5 max abs err over all %d x %d rows: O %.3g LSE %.3g" % (w.batch, w.num_q_heads, eo, el))
