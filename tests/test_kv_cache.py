"""KV append and page gather / scatter: oracle pins (CPU) and bit-exact GPU parity through the C ABI."""
import numpy as np
import pytest

from oracle import oracle
from paper_2603_12831_amd import workloads as wl


def _cache(seed=0, dtype="bf16", lengths=(5, 16, 40, 100), hkv=2, d=64):
    w = wl.make_generic(seed, list(lengths), 4, hkv, d, dtype=dtype, pool_factor=2.0)
    return w


def test_oracle_append_then_attention_sees_the_token():
    """Appending token L then reading range [L, L+1) must return exactly the appended v row, and the
    gather of that token must return the appended k, v bits; every other pool byte is untouched."""
    w = _cache(1, "f32", lengths=(5, 16, 40, 100))
    lengths = np.array([4, 15, 39, 99])                              # context before the append
    rng = np.random.default_rng(0)
    k_new = rng.standard_normal((4, 2, 64)).astype(np.float32)
    v_new = rng.standard_normal((4, 2, 64)).astype(np.float32)
    k0, v0 = w.k_pool.copy(), w.v_pool.copy()
    oracle.kv_append(w.k_pool, w.v_pool, w.block_table, k_new, v_new, lengths)
    changed = np.zeros(w.k_pool.shape[:3], dtype=bool)
    for i, L in enumerate(lengths):
        page, slot = w.block_table[i, L // 16], L % 16
        changed[page, :, slot] = True
        assert np.array_equal(w.k_pool[page, :, slot], k_new[i]) and np.array_equal(w.v_pool[page, :, slot], v_new[i])
        kk, vv = oracle.gather_kv(w.k_pool, w.v_pool, w.block_table, i, int(L), int(L) + 1)
        assert np.array_equal(kk[0], k_new[i]) and np.array_equal(vv[0], v_new[i])
        o, _ = oracle.paged_attn(w.q, w.k_pool, w.v_pool, w.block_table, lengths, lengths + 1, 1.0, "f32", seqs=[i])
        assert np.array_equal(o[0, 0], v_new[i, 0].astype(np.float64))
    assert np.array_equal(w.k_pool[~changed], k0[~changed]) and np.array_equal(w.v_pool[~changed], v0[~changed])


def test_oracle_append_skips_positions_without_a_slot():
    w = _cache(2, "bf16")
    k0, v0 = w.k_pool.copy(), w.v_pool.copy()
    k_new = np.full((4, 2, 64), 0x3F80, dtype=np.uint16)
    bt = w.block_table.copy()
    bt[2, 0] = w.num_blocks + 3
    oracle.kv_append(w.k_pool, w.v_pool, bt, k_new, k_new, np.array([-1, bt.shape[1] * 16, 3, 10 ** 6]))
    assert np.array_equal(w.k_pool, k0) and np.array_equal(w.v_pool, v0)


def test_oracle_page_gather_scatter_against_fancy_indexing_and_round_trip():
    w = _cache(3, "bf16", lengths=(300, 200))
    ids = np.array([5, 0, w.num_blocks - 1, 7, -1, w.num_blocks], dtype=np.int32)
    k, v = oracle.kv_gather_pages(w.k_pool, w.v_pool, ids)
    ok = (ids >= 0) & (ids < w.num_blocks)
    assert np.array_equal(k[ok], w.k_pool[ids[ok]]) and np.array_equal(v[ok], w.v_pool[ids[ok]])
    assert not k[~ok].any() and not v[~ok].any()
    # scatter into an empty pool at other places, gather back: identity on the valid pages
    k2, v2 = np.zeros_like(w.k_pool), np.zeros_like(w.v_pool)
    dest = np.array([9, 3, 1, 4, 2, -5], dtype=np.int32)
    oracle.kv_scatter_pages(k2, v2, dest, k, v)
    for j in range(5):
        assert np.array_equal(k2[dest[j]], k[j]) and np.array_equal(v2[dest[j]], v[j])
    untouched = np.setdiff1d(np.arange(w.num_blocks), dest[:5])
    assert not k2[untouched].any() and not v2[untouched].any()


# ---------------------------------------------------------------------------------------------------
@pytest.mark.gpu
@pytest.mark.parametrize("dtype,hkv,d", [("bf16", 8, 128), ("f32", 2, 64), ("bf16", 1, 64)])
def test_gpu_append_and_pages_bit_exact(dtype, hkv, d):
    torch = pytest.importorskip("torch")
    from paper_2603_12831_amd import binding
    from paper_2603_12831_amd.runner import to_device
    assert torch.cuda.is_available()
    rng = np.random.default_rng(7)
    lengths = rng.integers(1, 400, size=37)
    w = wl.make_generic(9, lengths + 1, 4 * hkv if hkv < 8 else 32, hkv, d, dtype=dtype, pool_factor=1.5)
    dev = torch.device("cuda:0")
    kp, vp = to_device(w.k_pool, dtype, dev), to_device(w.v_pool, dtype, dev)
    bt_np = w.block_table.copy()
    bt_np[3, 0] = -1                                                 # one sequence whose page is absent
    positions = lengths.astype(np.int32)
    positions[3] = 2
    positions[5] = -4
    positions[6] = bt_np.shape[1] * 16
    k_new = wl._normal((len(lengths), hkv, d), [9, 50], 1.0, dtype)
    v_new = wl._normal((len(lengths), hkv, d), [9, 51], 1.0, dtype)
    binding.omni_kv_append(kp, vp, torch.from_numpy(bt_np).to(dev), to_device(k_new, dtype, dev),
                           to_device(v_new, dtype, dev), torch.from_numpy(positions).to(dev))
    ek, ev = w.k_pool.copy(), w.v_pool.copy()
    oracle.kv_append(ek, ev, bt_np, k_new, v_new, positions)
    bits = (lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)) if dtype == "bf16" else (lambda t: t.cpu().numpy())
    assert np.array_equal(bits(kp).view(np.uint8), ek.view(np.uint8))
    assert np.array_equal(bits(vp).view(np.uint8), ev.view(np.uint8))
    assert not np.array_equal(ek, w.k_pool)                          # something was appended

    ids = rng.permutation(w.num_blocks)[: w.num_blocks // 2].astype(np.int32)
    ids[1] = -1
    ids[4] = w.num_blocks
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    ks = torch.full((len(ids), hkv, 16, d), 7.0, dtype=tdt, device=dev)
    vs = torch.full_like(ks, 7.0)
    ids_t = torch.from_numpy(ids).to(dev)
    binding.omni_kv_gather_pages(kp, vp, ids_t, ks, vs)
    gk, gv = oracle.kv_gather_pages(ek, ev, ids)
    assert np.array_equal(bits(ks).view(np.uint8), gk.view(np.uint8))
    assert np.array_equal(bits(vs).view(np.uint8), gv.view(np.uint8))
    # swap-in to other pages of a second pool
    kp2, vp2 = torch.zeros_like(kp), torch.zeros_like(vp)
    dest = rng.permutation(w.num_blocks)[: len(ids)].astype(np.int32)
    dest[2] = -7
    binding.omni_kv_scatter_pages(kp2, vp2, torch.from_numpy(dest).to(dev), ks, vs)
    ek2, ev2 = np.zeros_like(ek), np.zeros_like(ev)
    oracle.kv_scatter_pages(ek2, ev2, dest, gk, gv)
    torch.cuda.synchronize()
    assert np.array_equal(bits(kp2).view(np.uint8), ek2.view(np.uint8))
    assert np.array_equal(bits(vp2).view(np.uint8), ev2.view(np.uint8))
    # zero pages is a no-op
    binding.omni_kv_gather_pages(kp, vp, ids_t[:0], ks[:0], vs[:0])


@pytest.mark.gpu
def test_gpu_append_then_decode_matches_oracle():
    """The step before the hot path feeding it: append the new token on the GPU, then decode attention over
    the grown context equals the oracle on the oracle-appended cache."""
    torch = pytest.importorskip("torch")
    from paper_2603_12831_amd import binding
    from paper_2603_12831_amd.runner import DeviceWorkload, to_device
    w = wl.make_cfg3(batch=10, median=300, lo=2, hi=900, chunk_tokens=256)
    old = (w.ctx_len - 1).astype(np.int32)                           # the last token is the one being appended
    k_new = wl._normal((10, 8, 128), [3, 60], 1.0, "bf16")
    v_new = wl._normal((10, 8, 128), [3, 61], 1.0, "bf16")
    dw = DeviceWorkload(w, out_dtype="f32")
    binding.omni_kv_append(dw.k_pools[0], dw.v_pools[0], dw.block_table, to_device(k_new, "bf16", dw.device),
                           to_device(v_new, "bf16", dw.device), torch.from_numpy(old).to(dw.device))
    dw.run()
    got_o, got_l = dw.results()
    oracle.kv_append(w.k_pool, w.v_pool, w.block_table, k_new, v_new, old)
    exp_o, exp_l = oracle.paged_attn(w.q, w.k_pool, w.v_pool, w.block_table, None, w.ctx_len, w.sm_scale, "bf16",
                                     n_threads=8)
    assert np.max(np.abs(got_o - exp_o)) <= 2e-3 and np.max(np.abs(got_l - exp_l)) <= 2e-3


@pytest.mark.gpu
def test_gpu_append_and_pages_beyond_4_gib_into_the_pools():
    """Pools of 4.5 GiB whose used pages all lie past 4 GiB: the appended token and the gathered / scattered
    pages land bit for bit where the oracle puts them on the small pools."""
    torch = pytest.importorskip("torch")
    from paper_2603_12831_amd import binding
    from paper_2603_12831_amd.runner import to_device
    dtype, hkv, d = "bf16", 2, 128
    rng = np.random.default_rng(11)
    lengths = rng.integers(1, 300, size=9)
    w = wl.make_generic(12, lengths + 1, 8, hkv, d, dtype=dtype, pool_factor=1.5)
    dev = torch.device("cuda:0")
    n_big = (9 << 29) // (hkv * 16 * d * 2)
    base = n_big - w.num_blocks
    assert base * hkv * 16 * d * 2 > (1 << 32)

    def big(pool):
        t = torch.zeros((n_big, hkv, 16, d), dtype=torch.bfloat16, device=dev)
        t[base:].copy_(to_device(pool, dtype, dev))
        return t
    kp, vp = big(w.k_pool), big(w.v_pool)
    bt_big = np.where(w.block_table >= 0, w.block_table + base, -1).astype(np.int32)
    positions = lengths.astype(np.int32)
    k_new = wl._normal((len(lengths), hkv, d), [12, 50], 1.0, dtype)
    v_new = wl._normal((len(lengths), hkv, d), [12, 51], 1.0, dtype)
    binding.omni_kv_append(kp, vp, torch.from_numpy(bt_big).to(dev), to_device(k_new, dtype, dev),
                           to_device(v_new, dtype, dev), torch.from_numpy(positions).to(dev))
    ek, ev = w.k_pool.copy(), w.v_pool.copy()
    oracle.kv_append(ek, ev, w.block_table, k_new, v_new, positions)
    bits = lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(bits(kp[base:]), ek) and np.array_equal(bits(vp[base:]), ev)
    assert not bits(kp[base - 64:base]).any()                        # nothing landed in front of them

    ids = rng.permutation(w.num_blocks)[: w.num_blocks // 2].astype(np.int32)
    ks = torch.full((len(ids), hkv, 16, d), 7.0, dtype=torch.bfloat16, device=dev)
    vs = torch.full_like(ks, 7.0)
    binding.omni_kv_gather_pages(kp, vp, torch.from_numpy(ids + base).to(dev), ks, vs)
    gk, gv = oracle.kv_gather_pages(ek, ev, ids)
    assert np.array_equal(bits(ks), gk) and np.array_equal(bits(vs), gv)
    dest = rng.permutation(w.num_blocks)[: len(ids)].astype(np.int32)
    kp[base:].zero_()
    vp[base:].zero_()
    binding.omni_kv_scatter_pages(kp, vp, torch.from_numpy(dest + base).to(dev), ks, vs)
    ek2, ev2 = np.zeros_like(ek), np.zeros_like(ev)
    oracle.kv_scatter_pages(ek2, ev2, dest, gk, gv)
    torch.cuda.synchronize()
    assert np.array_equal(bits(kp[base:]), ek2) and np.array_equal(bits(vp[base:]), ev2)
    del kp, vp
    torch.cuda.empty_cache()
