"""GPU parity of the decode call's final rows: sequences the call can finish itself (one non-empty chunk)
written directly with the others left to the masked merge, and the fused form in which the attention
launch finishes every sequence (partials of several chunks merged by the workgroup that comes last, rows
computed elsewhere folded in).  Everything against the CPU fp64 oracle, and the routes against each other."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import oracle
from paper_2603_12831_amd import binding, workloads as wl
from paper_2603_12831_amd.runner import DeviceWorkload
from test_gpu_parity import (BENCH_FORM, KERNELS, PLANNED_LIST, THREADS, TOL, check, expected_full,
                             ext_partials_from_oracle)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("these tests need a GPU (run with -m gpu on an MI355X box)")
    binding.load_library()


def run_mode(w, mode, kernel=BENCH_FORM, out_dtype="f32", ext=None, passes=1):
    ext = ext or (None, None, None)
    dw = DeviceWorkload(w, out_dtype=out_dtype, ext_o=ext[0], ext_lse=ext[1], ext_offsets=ext[2],
                        workspace=kernel[1], mode=mode)
    for _ in range(passes):
        dw.poison_outputs()
        dw.seq_final.fill_(-7)
        dw.run(kernel=kernel[0])
    o, l = dw.results()
    if kernel[1]:
        assert dw.abandoned_waves() == 0
    return o, l, dw


def live_chunk_count(w):
    c = w.calls[0]
    tok = np.maximum(c.ctx_end.astype(np.int64) - c.ctx_begin, 0)
    ct = c.chunk_tokens if c.chunk_tokens else 1 << 30
    return np.minimum((tok + ct - 1) // ct, c.max_chunks)


def mixed_batch(seed=71, dtype="bf16", hq=8, hkv=2, d=128, chunk=128):
    """Ranges of zero, one and several chunks, some starting past token 0."""
    lengths = np.array([1, 40, 128, 129, 300, 127, 0, 513, 64, 1000, 128, 5, 260, 90, 0, 384])
    begin = np.array([0, 3, 0, 0, 17, 0, 0, 1, 60, 0, 1, 0, 4, 0, 0, 0])
    w = wl.make_generic(seed, np.maximum(lengths + begin, 1), hq, hkv, d, dtype=dtype, chunk_tokens=chunk,
                        ctx_begin=begin, pool_factor=1.3)
    w.calls[0].ctx_end = (lengths + begin).astype(np.int32)
    w.calls[0].max_chunks = int((int(lengths.max()) + chunk - 1) // chunk)
    return w


@pytest.mark.parametrize("kernel", KERNELS)
@pytest.mark.parametrize("out_dtype", ["f32", "bf16"])
def test_final_rows_of_single_chunk_sequences(kernel, out_dtype):
    """Mixed batch: the call writes the final rows of the sequences with at most one non-empty chunk and
    says so in seq_final; those rows equal the merged route bit for bit and their partial rows are never
    written; the masked merge completes the batch."""
    w = mixed_batch()
    exp = expected_full(w, begin=w.calls[0].ctx_begin, end=w.calls[0].ctx_end)
    o_m, l_m, _ = run_mode(w, "merge", kernel, out_dtype)
    dw = DeviceWorkload(w, out_dtype=out_dtype, workspace=kernel[1], mode="final")
    dw.poison_outputs()
    dw.seq_final.fill_(-7)
    if dw.plan_first:
        dw.plan()
    dw.run_attention(kernel=kernel[0], planned=dw.plan_first)
    torch.cuda.synchronize()
    single = live_chunk_count(w) <= 1
    assert np.array_equal(dw.seq_final.cpu().numpy(), single.astype(np.int32))
    o_a = dw.out_o.float().cpu().numpy().astype(np.float64)
    l_a = dw.out_lse.cpu().numpy().astype(np.float64)
    # finished rows are there already, bit-identical to the merged route; the others untouched (NaN)
    assert np.array_equal(o_a[single], o_m[single]) and np.array_equal(l_a[single], l_m[single])
    assert np.all(np.isnan(o_a[~single])) and np.all(np.isnan(l_a[~single]))
    po = dw.calls[0]["part_o"].cpu().numpy()
    pl = dw.calls[0]["part_lse"].cpu().numpy()
    assert np.all(np.isnan(po[single])), "a finished sequence wrote a partial row"
    assert np.all(pl[single] == -np.inf)
    dw.run_merge()
    o_f, l_f = dw.results()
    assert np.array_equal(o_f, o_m) and np.array_equal(l_f, l_m)
    tol = TOL["bf16"] + (float(np.max(np.abs(exp[0]))) * 2.0 ** -9 if out_dtype == "bf16" else 0.0)
    check(o_f, l_f, exp[0], exp[1], tol, "final rows + masked merge")


@pytest.mark.parametrize("dtype,shape", [("f32", (8, 2, 64)), ("bf16", (8, 8, 64)), ("f32", (4, 4, 128))])
def test_final_rows_vector_kernel(dtype, shape):
    hq, hkv, d = shape
    w = mixed_batch(seed=72, dtype=dtype, hq=hq, hkv=hkv, d=d, chunk=64)
    exp = expected_full(w, begin=w.calls[0].ctx_begin, end=w.calls[0].ctx_end)
    o_m, l_m, _ = run_mode(w, "merge", (binding.OMNI_KERNEL_VECTOR, False))
    o_f, l_f, dw = run_mode(w, "final", (binding.OMNI_KERNEL_VECTOR, False))
    assert np.array_equal(dw.seq_final.cpu().numpy(), (live_chunk_count(w) <= 1).astype(np.int32))
    assert np.array_equal(o_f, o_m) and np.array_equal(l_f, l_m)
    check(o_f, l_f, exp[0], exp[1], TOL[dtype], "vector kernel final rows")


@pytest.mark.parametrize("out_dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(8, 2, 128), (16, 1, 160), (6, 3, 64), (8, 8, 256)])
def test_fused_form_finishes_every_sequence(out_dtype, shape):
    """The attention launch alone: sequences of zero, one and several chunks, run three times on the same
    buffers and work list (the arrival counters must come back to zero), equal to the oracle and, to
    rounding of the different merge order, to the two-launch route."""
    hq, hkv, chunk = shape
    w = mixed_batch(seed=73 + hq, hq=hq, hkv=hkv, chunk=chunk)
    exp = expected_full(w, begin=w.calls[0].ctx_begin, end=w.calls[0].ctx_end)
    tol = TOL["bf16"] + (float(np.max(np.abs(exp[0]))) * 2.0 ** -9 if out_dtype == "bf16" else 0.0)
    o_m, l_m, _ = run_mode(w, "merge", out_dtype=out_dtype)
    o_r, l_r, _ = run_mode(w, "fused", PLANNED_LIST, out_dtype=out_dtype, passes=2)
    o_f, l_f, dw = run_mode(w, "fused", out_dtype=out_dtype, passes=3)
    assert np.all(dw.seq_final.cpu().numpy() == 1)
    assert np.array_equal(o_r, o_f) and np.array_equal(l_r, l_f)
    check(o_f, l_f, exp[0], exp[1], tol, "fused form")
    single = live_chunk_count(w) <= 1
    assert np.array_equal(o_f[single], o_m[single]) and np.array_equal(l_f[single], l_m[single])
    # a planned list reused by the fused form
    dw.plan()
    for _ in range(2):
        dw.poison_outputs()
        dw.run_attention(planned=True)
        o_p, l_p = dw.results()
        assert np.array_equal(o_p, o_f) and np.array_equal(l_p, l_f)


def test_fused_form_many_chunks_is_deterministic():
    """Rows of up to 40 chunks with many more items than workgroups: the merge must find every partial row
    of the launch in place whichever workgroup comes last; repeated runs are bit-identical."""
    rng = np.random.default_rng(74)
    lengths = rng.integers(1, 2600, size=300)
    lengths[::7] = rng.integers(1, 60, size=len(lengths[::7]))
    w = wl.make_generic(74, lengths, 16, 4, 128, dtype="bf16", chunk_tokens=64)
    exp = expected_full(w, begin=w.calls[0].ctx_begin, end=w.calls[0].ctx_end)
    o1, l1, dw = run_mode(w, "fused")
    check(o1, l1, exp[0], exp[1], TOL["bf16"], "fused, many chunks")
    for _ in range(4):
        dw.poison_outputs()
        dw.run()
        o2, l2 = dw.results()
        assert np.array_equal(o1, o2) and np.array_equal(l1, l2)
    assert dw.abandoned_waves() == 0


def test_fused_form_folds_rows_computed_elsewhere():
    """Hybrid batch: resident tails on the GPU, prefix partials from the oracle (fp32) as an external
    source folded in by the attention launch; also with the tails cut into chunks, and with sequences
    whose resident range is empty (their rows come from the external source alone)."""
    w = wl.make_cfg4(n_ls=5, n_be=20, ls_lo=20, ls_hi=600, be_lo=300, be_hi=900, tail_lo=5, tail_hi=200)
    ext = ext_partials_from_oracle(w)
    exp = expected_full(w)
    o_m, l_m, _ = run_mode(w, "merge", ext=ext)
    check(o_m, l_m, exp[0], exp[1], TOL["bf16"], "two launches")
    o_f, l_f, _ = run_mode(w, "fused", ext=ext, passes=2)
    check(o_f, l_f, exp[0], exp[1], TOL["bf16"], "fused hybrid")
    w.calls[0].chunk_tokens, w.calls[0].max_chunks = 64, 12
    o_c, l_c, _ = run_mode(w, "fused", ext=ext, passes=2)
    check(o_c, l_c, exp[0], exp[1], TOL["bf16"], "fused hybrid, chunked tails")
    # two best-effort rows without resident tokens, one latency-sensitive row without any context at all
    w.calls[0].chunk_tokens, w.calls[0].max_chunks = 0, 1
    n_ls = w.meta["n_ls"]
    end = w.calls[0].ctx_end.copy()
    for i in (n_ls + 1, n_ls + 4):
        end[i] = w.calls[0].ctx_begin[i]
    end[2] = 0
    w.calls[0].ctx_end = end
    exp2 = expected_full(w, begin=np.zeros_like(end), end=end)
    o_e, l_e, _ = run_mode(w, "fused", ext=ext)
    assert np.all(o_e[2] == 0) and np.all(l_e[2] == -np.inf)
    check(o_e, l_e, exp2[0], exp2[1], TOL["bf16"], "fused hybrid, empty resident ranges")


@pytest.mark.parametrize("kernel", KERNELS + [(binding.OMNI_KERNEL_VECTOR, False)])
def test_final_rows_leave_sequences_with_rows_elsewhere_to_the_merge(kernel):
    """Hybrid batch with the sources named but not folded in: the call finishes the sequences that have
    neither a second chunk nor rows elsewhere, says so in seq_final, and the masked merge puts the others
    together from every part - also where the resident range is a single chunk, or empty."""
    w = wl.make_cfg4(n_ls=5, n_be=20, ls_lo=20, ls_hi=600, be_lo=300, be_hi=900, tail_lo=5, tail_hi=200)
    ext = ext_partials_from_oracle(w)
    has_ext = np.array([len(rs) > 0 for rs in w.ext_ranges])
    exp = expected_full(w)
    for chunk_tokens, max_chunks in ((0, 1), (64, 12)):
        w.calls[0].chunk_tokens, w.calls[0].max_chunks = chunk_tokens, max_chunks
        o_m, l_m, _ = run_mode(w, "merge", kernel, ext=ext)
        o_f, l_f, dw = run_mode(w, "final", kernel, ext=ext, passes=2)
        final = (live_chunk_count(w) <= 1) & ~has_ext
        assert final.any() and not final.all()
        assert np.array_equal(dw.seq_final.cpu().numpy(), final.astype(np.int32))
        assert np.array_equal(o_f, o_m) and np.array_equal(l_f, l_m)
        check(o_f, l_f, exp[0], exp[1], TOL["bf16"], "final rows, hybrid batch, chunk %d" % chunk_tokens)
    # two best-effort rows without resident tokens (their rows elsewhere are all there is), one
    # latency-sensitive row without any context at all (finished here: O = 0, LSE = -inf)
    w.calls[0].chunk_tokens, w.calls[0].max_chunks = 0, 1
    n_ls = w.meta["n_ls"]
    end = w.calls[0].ctx_end.copy()
    for i in (n_ls + 1, n_ls + 4):
        end[i] = w.calls[0].ctx_begin[i]
    end[2] = 0
    w.calls[0].ctx_end = end
    exp2 = expected_full(w, begin=np.zeros_like(end), end=end)
    o_e, l_e, dw = run_mode(w, "final", kernel, ext=ext)
    fin = dw.seq_final.cpu().numpy()
    assert fin[2] == 1 and fin[n_ls + 1] == 0 and fin[n_ls + 4] == 0
    assert np.all(o_e[2] == 0) and np.all(l_e[2] == -np.inf)
    check(o_e, l_e, exp2[0], exp2[1], TOL["bf16"], "final rows, hybrid batch, empty resident ranges")


def test_final_rows_with_sources_need_seq_final_and_partials():
    w = wl.make_cfg4(n_ls=3, n_be=6, ls_lo=20, ls_hi=100, be_lo=300, be_hi=400, tail_lo=5, tail_hi=50)
    ext = ext_partials_from_oracle(w)
    dw = DeviceWorkload(w, out_dtype="f32", ext_o=ext[0], ext_lse=ext[1], ext_offsets=ext[2], mode="final")
    args = dw.decode_args(dw.calls[0], binding.OMNI_KERNEL_AUTO, 0, False)
    args.seq_final = None
    assert binding.omni_paged_decode_attn_raw(args, check=False) == binding.OMNI_ERR_NULL
    args = dw.decode_args(dw.calls[0], binding.OMNI_KERNEL_AUTO, 0, False)
    args.part_o, args.part_lse = None, None
    assert binding.omni_paged_decode_attn_raw(args, check=False) == binding.OMNI_ERR_NULL


def hybrid_batch(seed, hq, hkv, pieces, dtype="bf16"):
    """Sequences whose last tokens are resident and whose prefix comes as pieces[i] rows computed elsewhere
    (0 = the whole context is resident)."""
    rng = np.random.default_rng([seed, hq, hkv])
    n = len(pieces)
    lengths = rng.integers(200, 900, size=n)
    tail = rng.integers(3, 150, size=n)
    w = wl.make_generic(seed, lengths, hq, hkv, 128, dtype=dtype, pool_factor=1.3)
    begin = np.where(np.array(pieces) > 0, lengths - tail, 0).astype(np.int32)
    w.calls = [wl.DecodeCall(begin, lengths.astype(np.int32), 0, 1)]
    ext = []
    for i, k in enumerate(pieces):
        cuts = [(int(begin[i]) * j) // k for j in range(k + 1)] if k else []
        ext.append([(cuts[j], cuts[j + 1]) for j in range(k)])
    w.ext_ranges = ext
    return w


@pytest.mark.parametrize("shape", [(8, 8), (8, 4), (6, 2), (16, 4), (16, 2), (32, 2)])
def test_fused_form_hybrid_batches_of_every_head_group(shape):
    """Rows from elsewhere through the LDS slots (up to four rows, up to four heads per kv head) and through
    the merge routine (more rows, more heads), one to six rows per sequence and sequences without any, for
    every group size up to 16 and both with the list built by the call and with a planned one."""
    hq, hkv = shape
    pieces = [1, 2, 3, 4, 0, 5, 6, 1, 4, 0, 2, 3, 4, 4, 1, 6, 2, 0, 3, 1]
    w = hybrid_batch(77, hq, hkv, pieces)
    ext = ext_partials_from_oracle(w)
    exp = expected_full(w)
    o_m, l_m, _ = run_mode(w, "merge", ext=ext)
    check(o_m, l_m, exp[0], exp[1], TOL["bf16"], "two launches")
    for kernel in (BENCH_FORM, PLANNED_LIST):
        o_f, l_f, dw = run_mode(w, "fused", kernel, ext=ext, passes=3)
        assert np.all(dw.seq_final.cpu().numpy() == 1)
        check(o_f, l_f, exp[0], exp[1], TOL["bf16"], "fused hybrid, G = %d" % (hq // hkv))
    # the tails cut into chunks: the last workgroup of a (sequence, kv head) merges chunks and rows
    c = w.calls[0]
    c.chunk_tokens, c.max_chunks = 32, int((int((c.ctx_end - c.ctx_begin).max()) + 31) // 32)
    o_c, l_c, _ = run_mode(w, "fused", ext=ext, passes=2)
    check(o_c, l_c, exp[0], exp[1], TOL["bf16"], "fused hybrid, chunked tails, G = %d" % (hq // hkv))


def test_fused_form_dense_external_source():
    """The external source given as a fixed number of rows per sequence instead of row offsets."""
    w = hybrid_batch(78, 16, 4, [3] * 12)
    ext = ext_partials_from_oracle(w)
    exp = expected_full(w)
    dw = DeviceWorkload(w, out_dtype="f32", ext_o=ext[0], ext_lse=ext[1], ext_offsets=ext[2], mode="fused")
    dw.ext = (dw.ext[0], dw.ext[1], None, 3)
    for _ in range(2):
        dw.poison_outputs()
        dw.run()
    o, l = dw.results()
    check(o, l, exp[0], exp[1], TOL["bf16"], "fused hybrid, dense source")
    assert dw.abandoned_waves() == 0


@pytest.mark.parametrize("mode", ["final", "fused"])
def test_long_context_in_many_chunks(mode):
    """One context of 131 072 tokens in 128 and in 2 048 chunks beside a one-chunk sequence: the in-launch
    merge (fused) folds up to 2 048 rows per head, the other route leaves them to the masked merge."""
    w = wl.make_generic(65, [131072, 50], 8, 2, 128, dtype="bf16", pool_factor=1.1, boost_frac=0.01, boost=8.0)
    exp = expected_full(w)
    for chunk, mc in [(1024, 128), (64, 2048)]:
        w.calls[0].chunk_tokens, w.calls[0].max_chunks = chunk, mc
        o, l, dw = run_mode(w, mode, passes=2)
        check(o, l, exp[0], exp[1], TOL["bf16"], "%s, %d chunks" % (mode, mc))
        assert np.array_equal(dw.seq_final.cpu().numpy(), np.array([mode == "fused", 1], dtype=np.int32))


def test_fused_form_needs_the_persistent_kernel():
    w = mixed_batch(seed=75)
    dw = DeviceWorkload(w, out_dtype="f32", workspace=False, mode="fused")
    args = dw.decode_args(dw.calls[0], binding.OMNI_KERNEL_AUTO, 0, False)
    assert binding.omni_paged_decode_attn_raw(args, check=False) == binding.OMNI_ERR_UNSUPPORTED
    wf = mixed_batch(seed=75, dtype="f32", d=64)
    dwf = DeviceWorkload(wf, out_dtype="f32", workspace=True, mode="fused")
    args = dwf.decode_args(dwf.calls[0], binding.OMNI_KERNEL_AUTO, 0, False)
    assert binding.omni_paged_decode_attn_raw(args, check=False) == binding.OMNI_ERR_UNSUPPORTED
    # final rows for part of the batch without a seq_final array: refused
    dw2 = DeviceWorkload(w, out_dtype="f32", mode="final")
    args = dw2.decode_args(dw2.calls[0], binding.OMNI_KERNEL_AUTO, 0, False)
    args.seq_final = None
    assert binding.omni_paged_decode_attn_raw(args, check=False) == binding.OMNI_ERR_NULL


def test_fused_step_in_a_graph_replays_exactly():
    w = wl.make_cfg3(batch=40, median=600, lo=1, hi=4000, chunk_tokens=512)
    exp = expected_full(w)
    o_e, l_e, dw = run_mode(w, "fused")
    check(o_e, l_e, exp[0], exp[1], TOL["bf16"], "fused eager")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        dw.run()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        dw.run()
    for replay in range(4):
        dw.poison_outputs()
        torch.cuda.synchronize()
        graph.replay()
        o, l = dw.results()
        assert np.array_equal(o, o_e) and np.array_equal(l, l_e), "replay %d differs" % replay


@pytest.mark.parametrize("name", ["cfg3", "cfg4", "cfg5"])
def test_full_size_final_rows(name):
    """The full-size configurations as bench.py times them: final rows from the attention call where it can
    finish a sequence, the masked merge for the rest, work list rebuilt by the call."""
    w = wl.MAKERS[name](workers=THREADS)
    ext = ext_partials_from_oracle(w) if w.ext_ranges is not None else None
    o, l, dw = run_mode(w, "final", ext=ext, passes=2)
    exp = expected_full(w)
    eo, el = check(o, l, exp[0], exp[1], 2e-3, name + " final rows")
    fin = int(dw.seq_final.sum().item())
    print("%s final rows: %d of %d sequences finished by the call, max abs err O %.3g LSE %.3g"
          % (name, fin, w.batch, eo, el))
    assert fin == {"cfg3": 82, "cfg4": 32, "cfg5": 0}[name]


@pytest.mark.parametrize("name", ["cfg3", "cfg4", "cfg5"])
def test_full_size_fused(name):
    """The full-size configurations through the fused form."""
    w = wl.MAKERS[name](workers=THREADS)
    ext = ext_partials_from_oracle(w) if w.ext_ranges is not None else None
    o, l, dw = run_mode(w, "fused", ext=ext, passes=2)
    exp = expected_full(w)
    eo, el = check(o, l, exp[0], exp[1], 2e-3, name + " fused")
    print("%s fused: max abs err O %.3g LSE %.3g" % (name, eo, el))


def test_timeline_instance_matches_the_plain_kernel():
    """The time-stamping instance gives the plain call's rows bit for bit, and stamps that are ordered."""
    w = wl.make_cfg3(batch=40, median=600, lo=1, hi=4000, chunk_tokens=512)
    o_p, l_p, dw = run_mode(w, "final")
    n_wg, words = binding.omni_debug_decode_timeline_shape()
    assert n_wg >= 1 and words >= 16
    stamps = torch.zeros(n_wg * words, dtype=torch.int64, device="cuda")
    dw.poison_outputs()
    args = dw.decode_args(dw.calls[0], binding.OMNI_KERNEL_AUTO, 0, False)
    binding.omni_debug_decode_timeline(args, stamps)
    dw.run_merge()
    o_t, l_t = dw.results()
    assert np.array_equal(o_t, o_p) and np.array_equal(l_t, l_p)
    assert dw.abandoned_waves() == 0
    st = stamps.cpu().numpy().reshape(n_wg, words)
    busy = st[:, 2] > 0
    assert busy.any()
    assert np.all(st[busy, 0] <= st[busy, 1]) and np.all(st[busy, 1] <= st[busy, 2])
    assert np.all(st[busy, 3] >= st[busy, 1]) and np.all(st[busy, 4] >= 1)
    n_items = int(live_chunk_count(w).sum()) * w.num_kv_heads
    assert int(st[busy, 4].sum()) == n_items            # (no short-range grouping in this batch: a ticket is an item)
    # too small a stamp buffer, and forms without a stamping instance
    assert binding.omni_debug_decode_timeline(args, stamps[: n_wg * words - 1], check=False) == binding.OMNI_ERR_SHAPE
    dwg = DeviceWorkload(w, out_dtype="f32", workspace=False, mode="final")
    argsg = dwg.decode_args(dwg.calls[0], binding.OMNI_KERNEL_AUTO, 0, False)
    assert binding.omni_debug_decode_timeline(argsg, stamps, check=False) == binding.OMNI_ERR_UNSUPPORTED
