"""Host-side checks of the synthetic input recipes (no arithmetic of the method)."""
import numpy as np

from paper_2603_12831_amd import workloads as wl


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.0e38, 1e-40], dtype=np.float32)
    b = wl.f32_to_bf16_bits(x)
    back = wl.bf16_bits_to_f32(b)
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7 -> even mantissa (1.0); 1 + 3*2^-8 ties up to 1 + 2^-6
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == np.float32(1.015625) and back[3] == -2.5
    torch = __import__("torch")
    t = torch.from_numpy(x).to(torch.bfloat16).float().numpy()
    assert np.array_equal(t[:5], back[:5])
    y = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    assert np.array_equal(torch.from_numpy(y).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16),
                          wl.f32_to_bf16_bits(y))


def _check_tables(w):
    bs = w.block_size
    used = []
    for i in range(w.batch):
        n = (int(w.ctx_len[i]) + bs - 1) // bs
        row = w.block_table[i]
        assert np.all(row[:n] >= 0) and np.all(row[:n] < w.num_blocks) and np.all(row[n:] == -1)
        used.extend(row[:n].tolist())
    assert len(set(used)) == len(used)                       # no page is shared


def test_cfg1_recipe():
    w = wl.make_cfg1()
    assert (w.batch, w.num_q_heads, w.num_kv_heads, w.head_dim, w.dtype) == (4, 8, 2, 64, "f32")
    assert w.ctx_len.tolist() == [17, 100, 256, 511] and w.num_blocks == 57
    assert w.meta["cut"].tolist() == [16, 64, 128, 256]
    assert w.kv_bytes() == 905216
    _check_tables(w)
    w2 = wl.make_cfg1()
    assert np.array_equal(w.k_pool, w2.k_pool) and np.array_equal(w.block_table, w2.block_table)


def test_scaled_down_recipes():
    w = wl.make_cfg2(batch=3, lo=40, hi=90)
    assert w.num_q_heads == w.num_kv_heads == 32 and w.dtype == "bf16" and w.k_pool.dtype == np.uint16
    need = int(((w.ctx_len + 15) // 16).sum())
    assert w.num_blocks == 2 * need and w.calls[0].chunk_tokens == 0
    _check_tables(w)
    assert abs(float(wl.bf16_bits_to_f32(w.k_pool).std()) - 1 / np.sqrt(128)) < 2e-3
    w = wl.make_cfg3(batch=16, median=150, lo=16, hi=600, chunk_tokens=64)
    assert w.calls[0].max_chunks == (int(w.ctx_len.max()) + 63) // 64 and w.num_q_heads // w.num_kv_heads == 4
    _check_tables(w)
    w = wl.make_cfg5(batch=2, ctx=512, chunk_tokens=128)
    k = wl.bf16_bits_to_f32(w.k_pool)
    rows = np.sqrt((k.astype(np.float64) ** 2).mean(axis=-1))
    frac = float((rows > 4).mean())
    assert 0.003 < frac < 0.03 and w.num_q_heads == 64


def test_generation_does_not_depend_on_worker_count():
    a = wl._normal((37, 2, 16, 128), [5, 2], 1.0, "bf16", workers=1)
    b = wl._normal((37, 2, 16, 128), [5, 2], 1.0, "bf16", workers=4)
    assert np.array_equal(a, b)


def test_cfg4_recipe():
    w = wl.make_cfg4(n_ls=3, n_be=5, ls_lo=20, ls_hi=70, be_lo=300, be_hi=500, tail_lo=10, tail_hi=40)
    _check_tables(w)
    c = w.calls[0]
    assert np.all(c.ctx_begin[:3] == 0) and np.array_equal(c.ctx_end, w.ctx_len)
    assert np.array_equal(w.ctx_len[3:] - c.ctx_begin[3:], w.meta["tail"])
    off = wl.ext_row_offsets(w)
    assert off[3] == 0 and off[-1] == int(w.meta["n_ext"].sum())
    for i in range(3, 8):
        r = w.ext_ranges[i]
        assert r[0][0] == 0 and r[-1][1] == c.ctx_begin[i]
        assert all(r[p][1] == r[p + 1][0] for p in range(len(r) - 1))
    # resident pages hold exactly the bits of the corresponding full-pool pages
    bs = w.block_size
    for i in range(w.batch):
        for lp in range(w.max_blocks_per_seq):
            dp = w.dev_block_table[i, lp]
            resident = c.ctx_begin[i] // bs <= lp < (w.ctx_len[i] + bs - 1) // bs
            assert (dp >= 0) == resident
            if resident:
                assert np.array_equal(w.dev_k_pool[dp], w.k_pool[w.block_table[i, lp]])
                assert np.array_equal(w.dev_v_pool[dp], w.v_pool[w.block_table[i, lp]])
    assert w.dev_k_pool.shape[0] == int((w.dev_block_table >= 0).sum())


def test_traffic_file_generator_reads_counter_tables(tmp_path):
    """paper_2603_12831_amd.hbm_traffic: per-kernel means of a counter CSV; the fused instance of the persistent
    kernel is a different kernel and is left out of the plain kernel's mean."""
    from paper_2603_12831_amd import hbm_traffic
    rows = [("void omni::(anonymous namespace)::copy_kernel(void*)", 524300.0),
            ("void omni::(anonymous namespace)::copy_kernel(void*)", 524306.0),
            ("void omni::(anonymous namespace)::decode_mfma_persistent_kernel<false, false, false>(omni::DecodeParams)", 100.0),
            ("void omni::(anonymous namespace)::decode_mfma_persistent_kernel<false, false, false>(omni::DecodeParams)", 300.0),
            ("void omni::(anonymous namespace)::decode_mfma_persistent_kernel<true, false, false>(omni::DecodeParams)", 9000.0),
            ("void omni::(anonymous namespace)::merge_kernel<128>(omni::MergeParams)", 7.0)]
    path = tmp_path / "p_counter_collection.csv"
    with open(path, "w") as f:
        f.write("Kernel_Name,Counter_Name,Counter_Value\n")
        for k, v in rows:
            f.write('"%s",FETCH_SIZE,%s\n' % (k, v))
    mean, n = hbm_traffic.mean_per_kernel(str(path))
    assert n == {"copy": 2, "decode": 2}
    assert mean["copy"] == 524303.0 and mean["decode"] == 200.0
