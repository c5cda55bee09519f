"""Row queues and residual store: oracle pins (CPU, against a Python deque / dict model) and bit-exact GPU
parity through the C ABI on a seeded random sequence of operations."""
import collections

import numpy as np
import pytest

from oracle import oracle


def _ops(seed, n_ops, capacity, max_rows):
    rng = np.random.default_rng(seed)
    ops = []
    for _ in range(n_ops):
        if rng.random() < 0.55:
            ops.append(("push", int(rng.integers(0, max_rows + 1))))
        else:
            ops.append(("pop", int(rng.integers(0, max_rows + 1))))
    return ops, rng


def test_oracle_queue_behaves_like_a_bounded_fifo():
    cap, rb = 13, 32
    q = oracle.Queue(cap, rb)
    model = collections.deque()
    ops, rng = _ops(0, 400, cap, 9)
    next_tag = 0
    for kind, n in ops:
        if kind == "push":
            rows = rng.integers(0, 256, size=(n, rb), dtype=np.uint8)
            tags = np.arange(next_tag, next_tag + n, dtype=np.int32)
            got = q.push(rows, tags)
            if len(model) + n <= cap:
                assert got == n
                model.extend((rows[i].tobytes(), int(tags[i])) for i in range(n))
                next_tag += n
            else:
                assert got == 0                                     # all or nothing
        else:
            rows, tags = q.pop(n)
            want = [model.popleft() for _ in range(min(n, len(model)))]
            assert len(rows) == len(want)
            for i, (b, t) in enumerate(want):
                assert rows[i].tobytes() == b and int(tags[i]) == t
        assert int(q.state[1] - q.state[0]) == len(model)
    assert int(q.state[1]) > 3 * cap                                # the ring wrapped several times


def test_oracle_store_is_a_keyed_row_store():
    rng = np.random.default_rng(1)
    store = np.zeros((50, 48), dtype=np.uint8)
    model = {}
    for _ in range(30):
        ids = rng.integers(-3, 54, size=7)
        ids[1] = ids[0]                                             # a duplicate: the later row wins
        rows = rng.integers(0, 256, size=(7, 48), dtype=np.uint8)
        oracle.store_save(store, ids, rows)
        for i, s in enumerate(ids):
            if 0 <= s < 50:
                model[int(s)] = rows[i].copy()
        probe = rng.integers(-3, 54, size=9)
        got = oracle.store_load(store, probe)
        for i, s in enumerate(probe):
            want = model.get(int(s), np.zeros(48, dtype=np.uint8)) if 0 <= s < 50 else np.zeros(48, dtype=np.uint8)
            assert np.array_equal(got[i], want)


@pytest.mark.gpu
def test_gpu_queue_and_store_match_the_oracle():
    torch = pytest.importorskip("torch")
    from paper_2603_12831_amd import binding
    assert torch.cuda.is_available()
    dev = torch.device("cuda:0")
    cap, rb = 97, 32 * 128 * 2                                      # rows = one request's attention result (bf16)
    host = oracle.Queue(cap, rb)
    data = torch.zeros((cap, rb), dtype=torch.uint8, device=dev)
    tags = torch.zeros(cap, dtype=torch.int32, device=dev)
    state = torch.zeros(4, dtype=torch.int32, device=dev)
    q = binding.make_queue(data, tags, state)
    n_dev = torch.zeros(1, dtype=torch.int32, device=dev)
    ops, rng = _ops(5, 120, cap, 60)
    tag0 = 0
    for kind, n in ops:
        if kind == "push":
            rows = rng.integers(0, 256, size=(n, rb), dtype=np.uint8)
            tg = np.arange(tag0, tag0 + n, dtype=np.int32)
            tag0 += n
            want = host.push(rows, tg)
            binding.omni_queue_push(q, torch.from_numpy(rows).to(dev), torch.from_numpy(tg).to(dev), n_dev)
            assert int(n_dev.item()) == want
        else:
            want_rows, want_tags = host.pop(n)
            out = torch.full((n, rb), 0xAB, dtype=torch.uint8, device=dev)
            out_t = torch.full((n,), -5, dtype=torch.int32, device=dev)
            binding.omni_queue_pop(q, out, out_t, n_dev)
            k = int(n_dev.item())
            assert k == len(want_rows)
            assert np.array_equal(out[:k].cpu().numpy(), want_rows) and np.array_equal(out_t[:k].cpu().numpy(), want_tags)
            assert bool((out[k:] == 0xAB).all())                    # rows beyond the popped count untouched
        st = state.cpu().numpy().view(np.uint32)
        assert st[0] == host.state[0] and st[1] == host.state[1] and st[2] == 0
    assert np.array_equal(data.cpu().numpy(), host.data) and np.array_equal(tags.cpu().numpy(), host.tags)

    # residual store: 400 requests x 4 layers of bf16 hidden rows (8192 bytes)
    n_slots, row = 1600, 4096
    store_h = np.zeros((n_slots, row * 2), dtype=np.uint8)
    store_d = torch.zeros((n_slots, row), dtype=torch.bfloat16, device=dev)
    for it in range(4):
        ids = rng.permutation(n_slots)[:400].astype(np.int32)
        ids[7], ids[9] = -1, n_slots
        rows = rng.integers(0, 256, size=(400, row * 2), dtype=np.uint8)
        oracle.store_save(store_h, ids, rows)
        binding.omni_residual_save(store_d, torch.from_numpy(ids).to(dev),
                                   torch.from_numpy(rows).to(dev).view(torch.bfloat16))
        probe = rng.integers(-2, n_slots + 2, size=400).astype(np.int32)
        out = torch.empty((400, row), dtype=torch.bfloat16, device=dev)
        binding.omni_residual_load(store_d, torch.from_numpy(probe).to(dev), out)
        assert np.array_equal(out.view(torch.uint8).cpu().numpy().reshape(400, -1), oracle.store_load(store_h, probe))
    assert np.array_equal(store_d.view(torch.uint8).cpu().numpy().reshape(n_slots, -1), store_h)


@pytest.mark.gpu
def test_gpu_rows_from_the_output_queue_feed_the_merge():
    """The piggybacking data path end to end on a config-4-shaped batch: the host producer computes the
    prefix partials of the best-effort rows (KV in host memory), they are pushed into device-resident output
    queues (O rows and LSE rows, tagged with the sequence number) in three instalments, popped, given their
    CSR offsets on the device from the tags and the popped count, and merged with the GPU's tail partials:
    the result must be attention over the full contexts (oracle), and the popped rows the pushed ones."""
    torch = pytest.importorskip("torch")
    from paper_2603_12831_amd import binding, workloads as wl
    from paper_2603_12831_amd.runner import DeviceWorkload
    assert torch.cuda.is_available()
    dev = torch.device("cuda:0")
    w = wl.make_cfg4(n_ls=4, n_be=23, ls_lo=20, ls_hi=400, be_lo=300, be_hi=1500, tail_lo=5, tail_hi=90)
    seq = np.array([i for i, rs in enumerate(w.ext_ranges) for _ in rs], dtype=np.int32)
    begin = np.array([b for rs in w.ext_ranges for (b, _) in rs], dtype=np.int32)
    end = np.array([e for rs in w.ext_ranges for (_, e) in rs], dtype=np.int32)
    ext_o, ext_l = binding.omni_host_partial_attn(w.q, w.k_pool, w.v_pool, w.block_table, seq, begin, end,
                                                  w.sm_scale, w.dtype, n_threads=8)
    n, hq, d = len(seq), w.num_q_heads, w.head_dim
    cap = n + 5
    # (the queue struct holds addresses only: the tensors must stay alive beside it)
    mem_o = (torch.zeros((cap, hq * d * 4), dtype=torch.uint8, device=dev), torch.zeros(cap, dtype=torch.int32, device=dev),
             torch.zeros(4, dtype=torch.int32, device=dev))
    mem_l = (torch.zeros((cap, hq * 4), dtype=torch.uint8, device=dev), torch.zeros(cap, dtype=torch.int32, device=dev),
             torch.zeros(4, dtype=torch.int32, device=dev))
    qo, ql = binding.make_queue(*mem_o), binding.make_queue(*mem_l)
    o_dev = torch.from_numpy(ext_o).to(dev)
    l_dev = torch.from_numpy(ext_l).to(dev)
    tags = torch.from_numpy(seq).to(dev)
    cuts = [0, n // 3, n // 3 + 1, n]
    for a, b in zip(cuts[:-1], cuts[1:]):                            # the producer's rows arrive in instalments
        binding.omni_queue_push(qo, o_dev[a:b].reshape(b - a, -1).view(torch.uint8), tags[a:b])
        binding.omni_queue_push(ql, l_dev[a:b].reshape(b - a, -1).view(torch.uint8), tags[a:b])
    # the consumer: pop whatever is there (room for more rows than came), offsets from the tags, merge
    got_o = torch.full((cap, hq, d), float("nan"), dtype=torch.float32, device=dev)
    got_l = torch.full((cap, hq), float("nan"), dtype=torch.float32, device=dev)
    got_t = torch.full((cap,), -9, dtype=torch.int32, device=dev)
    n_o = torch.zeros(1, dtype=torch.int32, device=dev)
    n_l = torch.zeros(1, dtype=torch.int32, device=dev)
    binding.omni_queue_pop(qo, got_o.view(torch.uint8).reshape(cap, -1), got_t, n_o)
    binding.omni_queue_pop(ql, got_l.view(torch.uint8).reshape(cap, -1), None, n_l)
    offsets = torch.full((w.batch + 1,), -1, dtype=torch.int32, device=dev)
    binding.omni_csr_from_tags(got_t, n_o, w.batch, offsets)
    # (built as a batch with an external source, which is then the popped rows as they lie on the device)
    dw = DeviceWorkload(w, out_dtype="f32", ext_o=np.zeros((1, hq, d), dtype=np.float32),
                        ext_lse=np.zeros((1, hq), dtype=np.float32), ext_offsets=np.zeros(w.batch + 1, dtype=np.int32))
    dw.ext = (got_o, got_l, offsets, 0)
    dw.poison_outputs()
    dw.run()
    res_o, res_l = dw.results()
    assert int(n_o.item()) == n and int(n_l.item()) == n
    assert np.array_equal(offsets.cpu().numpy(), wl.ext_row_offsets(w))
    assert np.array_equal(offsets.cpu().numpy(), np.searchsorted(seq, np.arange(w.batch + 1)))
    assert torch.equal(got_o[:n], o_dev) and torch.equal(got_l[:n], l_dev)
    full_end = np.max(np.stack([c.ctx_end for c in w.calls]), axis=0)
    exp_o, exp_l = oracle.paged_attn(w.q, w.k_pool, w.v_pool, w.block_table, np.zeros_like(full_end), full_end,
                                     w.sm_scale, w.dtype, n_threads=8)
    assert float(np.max(np.abs(res_o - exp_o))) <= 2e-3 and float(np.max(np.abs(res_l - exp_l))) <= 2e-3
