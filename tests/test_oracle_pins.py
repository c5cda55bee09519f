"""Pins of the CPU oracle against things that are not the oracle.

Each test would fail for a plausible mistake in ``oracle/oracle_attn.c``:
wrong page/slot arithmetic, wrong GQA head mapping, missing scale, a dropped
max-subtraction, unnormalised partials, log base, transposed operands.
The expected values come from dense numpy/scipy evaluation (library softmax
and logsumexp on independently gathered rows), a library attention routine,
closed forms, or a hand-worked example.
"""
import math
import os

import numpy as np
import pytest
import scipy.special

from oracle import oracle
from paper_2603_12831_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def dense_rows(w, seq, kv_head, begin, end):
    """Independent gather: logical rows [begin, end) of one kv head as float64."""
    t = np.arange(begin, end)
    pages = w.block_table[seq, t // w.block_size]
    slots = t % w.block_size
    k = w.k_pool[pages, kv_head, slots]
    v = w.v_pool[pages, kv_head, slots]
    if w.dtype == "bf16":
        k, v = wl.bf16_bits_to_f32(k), wl.bf16_bits_to_f32(v)
    return k.astype(np.float64), v.astype(np.float64)


def brute(w, seq, head, begin, end):
    g = w.num_q_heads // w.num_kv_heads
    k, v = dense_rows(w, seq, head // g, begin, end)
    q = w.q[seq, head]
    if w.dtype == "bf16":
        q = wl.bf16_bits_to_f32(q)
    s = (k @ q.astype(np.float64)) * w.sm_scale
    return scipy.special.softmax(s) @ v, scipy.special.logsumexp(s)


def test_golden_two_token_example():
    q = np.array([[[1.0, 0.0]]], dtype=np.float32)
    k = np.zeros((1, 1, 16, 2), dtype=np.float32)
    v = np.zeros((1, 1, 16, 2), dtype=np.float32)
    k[0, 0, 1, 0] = np.float32(math.log(3.0))
    v[0, 0, 0] = (4, 0)
    v[0, 0, 1] = (0, 8)
    bt = np.zeros((1, 1), dtype=np.int32)
    o, lse = oracle.paged_attn(q, k, v, bt, None, [2], 1.0, "f32")
    ln3 = float(np.float32(math.log(3.0)))          # the stored key is fp32-rounded
    p1 = math.exp(ln3) / (1 + math.exp(ln3))
    assert abs(o[0, 0, 0] - 4 * (1 - p1)) < 1e-14 and abs(o[0, 0, 1] - 8 * p1) < 1e-14
    assert np.allclose(o[0, 0], [1.0, 6.0], atol=1e-6)          # file values, fp32 key rounding
    assert abs(lse[0, 0] - math.log(4.0)) < 1e-7
    o0, l0 = oracle.paged_attn(q, k, v, bt, [0], [1], 1.0, "f32")
    o1, l1 = oracle.paged_attn(q, k, v, bt, [1], [2], 1.0, "f32")
    assert np.array_equal(o0[0, 0], [4.0, 0.0]) and l0[0, 0] == 0.0
    assert np.array_equal(o1[0, 0], [0.0, 8.0]) and abs(l1[0, 0] - ln3) < 1e-15
    mo, ml = oracle.merge(np.stack([o0[0, 0], o1[0, 0]]), [l0[0, 0], l1[0, 0]], [0, 2])
    assert np.allclose(mo[0], [1.0, 6.0], atol=1e-6) and abs(ml[0] - math.log(4.0)) < 1e-7
    txt = open(os.path.join(GOLDEN, "two_token_closed_form.txt")).read()
    assert "O 1 6" in txt and "LSE ln4" in txt


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_bruteforce_cfg1_shape(dtype):
    w = wl.make_cfg1()
    if dtype == "bf16":
        w = wl.make_generic(11, w.ctx_len, 8, 2, 64, dtype="bf16", pool_factor=1.7, sm_scale=0.31)
    o, lse = oracle.paged_attn(w.q, w.k_pool, w.v_pool, w.block_table, None, w.ctx_len, w.sm_scale, w.dtype)
    for i in range(w.batch):
        for j in range(w.num_q_heads):
            bo, bl = brute(w, i, j, 0, int(w.ctx_len[i]))
            assert np.max(np.abs(o[i, j] - bo)) < 1e-12
            assert abs(lse[i, j] - bl) < 1e-12


def test_bruteforce_all_small_lengths_and_ranges():
    lengths = np.arange(1, 41)
    w = wl.make_generic(7, lengths, 6, 3, 8, dtype="f32", pool_factor=1.5, sm_scale=0.7)
    rng = np.random.default_rng(0)
    items = []
    for i, L in enumerate(lengths):
        for j in range(w.num_q_heads):
            b = int(rng.integers(0, L))
            e = int(rng.integers(b + 1, L + 1))
            items.append((i, j, b, e))
            items.append((i, j, 0, int(L)))
    o, lse = oracle.paged_attn_items(w.q, w.k_pool, w.v_pool, w.block_table, items, w.sm_scale, "f32")
    for n, (i, j, b, e) in enumerate(items):
        bo, bl = brute(w, i, j, b, e)
        assert np.max(np.abs(o[n] - bo)) < 1e-12 and abs(lse[n] - bl) < 1e-12


def test_bf16_inputs_equal_widened_f32_inputs():
    w = wl.make_generic(5, [33, 70], 4, 2, 64, dtype="bf16")
    wf = (wl.bf16_bits_to_f32(w.q), wl.bf16_bits_to_f32(w.k_pool), wl.bf16_bits_to_f32(w.v_pool))
    a = oracle.paged_attn(w.q, w.k_pool, w.v_pool, w.block_table, None, w.ctx_len, w.sm_scale, "bf16")
    b = oracle.paged_attn(*wf, w.block_table, None, w.ctx_len, w.sm_scale, "f32")
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_library_attention_routine_contiguous():
    torch = pytest.importorskip("torch")
    L, hq, hkv, d = 77, 4, 2, 64
    w = wl.make_generic(3, [L], hq, hkv, d, dtype="f32")
    w.block_table[0, :] = np.arange(w.block_table.shape[1])          # contiguous, un-permuted
    o, _ = oracle.paged_attn(w.q, w.k_pool, w.v_pool, w.block_table, None, w.ctx_len, w.sm_scale, "f32")
    k = torch.from_numpy(w.k_pool).double().permute(1, 0, 2, 3).reshape(hkv, -1, d)[:, :L]
    v = torch.from_numpy(w.v_pool).double().permute(1, 0, 2, 3).reshape(hkv, -1, d)[:, :L]
    q = torch.from_numpy(w.q[0]).double().reshape(hkv, hq // hkv, d)
    ref = torch.nn.functional.scaled_dot_product_attention(q, k, v)   # default scale 1/sqrt(d)
    assert np.max(np.abs(ref.reshape(hq, d).numpy() - o[0])) < 1e-12


def _one_seq(L, d=16, hq=2, hkv=1, seed=0):
    return wl.make_generic(seed, [L], hq, hkv, d, dtype="f32", pool_factor=2.0)


def test_identical_keys_give_mean_of_values():
    L = 37
    w = _one_seq(L)
    key = w.k_pool[0, 0, 0].copy()
    w.k_pool[:] = key
    o, lse = oracle.paged_attn(w.q, w.k_pool, w.v_pool, w.block_table, None, w.ctx_len, w.sm_scale, "f32")
    _, v = dense_rows(w, 0, 0, 0, L)
    for j in range(2):
        s = w.sm_scale * float(w.q[0, j].astype(np.float64) @ key.astype(np.float64))
        assert np.max(np.abs(o[0, j] - v.mean(axis=0))) < 1e-13
        assert abs(lse[0, j] - (s + math.log(L))) < 1e-12


def test_single_token_context_returns_its_value():
    w = _one_seq(1)
    o, lse = oracle.paged_attn(w.q, w.k_pool, w.v_pool, w.block_table, None, w.ctx_len, w.sm_scale, "f32")
    k, v = dense_rows(w, 0, 0, 0, 1)
    assert np.array_equal(o[0, 0], v[0]) and np.array_equal(o[0, 1], v[0])
    assert abs(lse[0, 0] - w.sm_scale * float(w.q[0, 0].astype(np.float64) @ k[0])) < 1e-14
    # a one-token range in the middle of a longer context, off the page start
    w = _one_seq(40)
    o, _ = oracle.paged_attn(w.q, w.k_pool, w.v_pool, w.block_table, [21], [22], w.sm_scale, "f32")
    _, v = dense_rows(w, 0, 0, 21, 22)
    assert np.array_equal(o[0, 0], v[0])


def test_zero_query_gives_uniform_weights():
    L = 50
    w = _one_seq(L)
    w.q[:] = 0
    o, lse = oracle.paged_attn(w.q, w.k_pool, w.v_pool, w.block_table, None, w.ctx_len, w.sm_scale, "f32")
    _, v = dense_rows(w, 0, 0, 0, L)
    assert np.max(np.abs(o[0, 0] - v.mean(axis=0))) < 1e-13
    assert abs(lse[0, 0] - math.log(L)) < 1e-13


def test_dominant_key_and_overflow_safety():
    L, t_star = 45, 29
    w = _one_seq(L, d=16)
    page, slot = w.block_table[0, t_star // 16], t_star % 16
    w.q[0, 0] = 0
    w.q[0, 0, 0] = 1.0
    w.k_pool[:, :, :, 0] = 0
    w.k_pool[page, 0, slot, 0] = 4000.0                    # logit 1000 at scale 1/4: exp overflows if unshifted
    o, lse = oracle.paged_attn(w.q, w.k_pool, w.v_pool, w.block_table, None, w.ctx_len, w.sm_scale, "f32")
    assert np.all(np.isfinite(o)) and np.all(np.isfinite(lse))
    assert np.max(np.abs(o[0, 0] - w.v_pool[page, 0, slot].astype(np.float64))) < 1e-300 + 1e-12
    assert abs(lse[0, 0] - 1000.0) < 1e-9


def test_logit_shift_moves_lse_only():
    L, c = 60, 3.25
    w = _one_seq(L, d=16)
    w.k_pool[..., 15] = 1.0
    w.q[..., 15] = 0.0
    a = oracle.paged_attn(w.q, w.k_pool, w.v_pool, w.block_table, None, w.ctx_len, w.sm_scale, "f32")
    w.q[..., 15] = np.float32(c / w.sm_scale)              # 13.0, exact in fp32
    b = oracle.paged_attn(w.q, w.k_pool, w.v_pool, w.block_table, None, w.ctx_len, w.sm_scale, "f32")
    assert np.max(np.abs(a[0] - b[0])) < 1e-13
    assert np.max(np.abs(b[1] - a[1] - c)) < 1e-12


def test_physical_placement_and_token_order_do_not_matter():
    L = 90
    w = wl.make_generic(8, [L], 4, 2, 32, dtype="f32", pool_factor=3.0)
    a = oracle.paged_attn(w.q, w.k_pool, w.v_pool, w.block_table, None, w.ctx_len, w.sm_scale, "f32")
    rng = np.random.default_rng(1)
    perm = rng.permutation(w.num_blocks)                   # new physical home of every page
    k2, v2 = np.empty_like(w.k_pool), np.empty_like(w.v_pool)
    k2[perm], v2[perm] = w.k_pool, w.v_pool
    bt2 = np.where(w.block_table >= 0, perm[np.maximum(w.block_table, 0)], -1).astype(np.int32)
    b = oracle.paged_attn(w.q, k2, v2, bt2, None, w.ctx_len, w.sm_scale, "f32")
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    # permute whole pages of the logical order (tokens move, set of (k, v) pairs unchanged)
    n_full = L // 16
    order = np.concatenate([rng.permutation(n_full), np.arange(n_full, w.block_table.shape[1])])
    bt3 = w.block_table[:, order]
    c = oracle.paged_attn(w.q, w.k_pool, w.v_pool, bt3, None, w.ctx_len, w.sm_scale, "f32")
    assert np.max(np.abs(a[0] - c[0])) < 1e-13 and np.max(np.abs(a[1] - c[1])) < 1e-13


def test_index_revealing_checksum():
    """q = 0 and V rows holding the logical token id: L * O is the exact sum of
    the ids that were read, so any wrong page or slot changes an integer."""
    lengths = [1, 15, 16, 17, 47, 128]
    w = wl.make_generic(2, lengths, 2, 2, 4, dtype="f32", pool_factor=2.5)
    w.q[:] = 0
    w.v_pool[:] = -1e6
    for i, L in enumerate(lengths):
        for t in range(L):
            w.v_pool[w.block_table[i, t // 16], :, t % 16, :] = t + 1000 * i
    for i, L in enumerate(lengths):
        for (b, e) in [(0, L), (L // 3, L), (0, max(1, L - 5))]:
            o, _ = oracle.paged_attn(w.q, w.k_pool, w.v_pool, w.block_table, np.full(len(lengths), b),
                                     np.full(len(lengths), e), 1.0, "f32", seqs=[i])
            want = sum(t + 1000 * i for t in range(b, e))
            assert abs(o[0, 0, 0] * (e - b) - want) < 1e-6 * max(1, want)


def test_gather_matches_fancy_indexing():
    w = wl.make_generic(4, [5, 64, 99], 4, 2, 8, dtype="bf16", pool_factor=2.0)
    for i, L in enumerate(w.ctx_len):
        for (b, e) in [(0, int(L)), (3, int(L)), (int(L) - 1, int(L)), (2, 2)]:
            k, v = oracle.gather_kv(w.k_pool, w.v_pool, w.block_table, i, b, e)
            t = np.arange(b, e)
            pages, slots = w.block_table[i, t // 16], t % 16
            assert np.array_equal(k, w.k_pool[pages][np.arange(len(t)), :, slots])
            assert np.array_equal(v, w.v_pool[pages][np.arange(len(t)), :, slots])


# ---------------------------------------------------------------------------
# merge
# ---------------------------------------------------------------------------
def _partials(w, cuts, seq=0):
    """Partials of sequence ``seq`` over consecutive ranges given by ``cuts``."""
    os_, ls_ = [], []
    for b, e in zip(cuts[:-1], cuts[1:]):
        begin = np.zeros(w.batch, dtype=np.int32) + b
        end = np.zeros(w.batch, dtype=np.int32) + e
        o, l = oracle.paged_attn(w.q, w.k_pool, w.v_pool, w.block_table, begin, end, w.sm_scale, w.dtype,
                                 seqs=[seq])
        os_.append(o[0])
        ls_.append(l[0])
    return np.stack(os_), np.stack(ls_)          # [P, Hq, D], [P, Hq]


@pytest.mark.parametrize("cuts", [[0, 16, 100], [0, 7, 7, 33, 100], [0, 1, 2, 3, 99, 100],
                                  list(range(0, 101, 4)), [0, 100], [0, 0, 100, 100]])
def test_split_equals_unsplit(cuts):
    w = wl.make_generic(6, [100], 4, 2, 32, dtype="bf16", pool_factor=1.3)
    full_o, full_l = oracle.paged_attn(w.q, w.k_pool, w.v_pool, w.block_table, None, w.ctx_len, w.sm_scale,
                                       w.dtype)
    po, pl = _partials(w, cuts)
    P = po.shape[0]
    for j in range(w.num_q_heads):
        mo, ml = oracle.merge(po[:, j], pl[:, j], [0, P])
        assert np.max(np.abs(mo[0] - full_o[0, j])) < 1e-12 and abs(ml[0] - full_l[0, j]) < 1e-12
        # against the library: dense softmax over the whole range
        bo, bl = brute(w, 0, j, 0, 100)
        assert np.max(np.abs(mo[0] - bo)) < 1e-12 and abs(ml[0] - bl) < 1e-12


def test_merge_is_associative_and_commutative():
    w = wl.make_generic(9, [200], 2, 1, 16, dtype="f32")
    po, pl = _partials(w, [0, 30, 64, 65, 150, 200])
    po, pl = po[:, 0], pl[:, 0]
    all_o, all_l = oracle.merge(po, pl, [0, 5])
    ab_o, ab_l = oracle.merge(po[:2], pl[:2], [0, 2])
    cde_o, cde_l = oracle.merge(po[2:], pl[2:], [0, 3])
    n_o, n_l = oracle.merge(np.stack([ab_o[0], cde_o[0]]), [ab_l[0], cde_l[0]], [0, 2])
    assert np.max(np.abs(n_o - all_o)) < 1e-13 and abs(n_l[0] - all_l[0]) < 1e-13
    order = [3, 0, 4, 2, 1]
    p_o, p_l = oracle.merge(po[order], pl[order], [0, 5])
    assert np.max(np.abs(p_o - all_o)) < 1e-13 and abs(p_l[0] - all_l[0]) < 1e-13


def test_merge_identities():
    rng = np.random.default_rng(0)
    a, b = rng.standard_normal(8), rng.standard_normal(8)
    ninf = -np.inf
    o, l = oracle.merge([a], [1.5], [0, 1])                           # one partial: identity
    assert np.array_equal(o[0], a) and l[0] == 1.5
    o, l = oracle.merge([a, b * 0 + 7], [1.5, ninf], [0, 2])          # empty partial: no-op
    assert np.array_equal(o[0], a) and l[0] == 1.5
    o, l = oracle.merge([a, b], [0.25, 0.25], [0, 2])                 # equal weights: mean, + ln 2
    assert np.max(np.abs(o[0] - (a + b) / 2)) < 1e-15 and abs(l[0] - (0.25 + math.log(2))) < 1e-15
    o, l = oracle.merge([a, b], [ninf, ninf], [0, 2])                 # nothing at all
    assert np.array_equal(o[0], np.zeros(8)) and l[0] == ninf
    o, l = oracle.merge(np.zeros((0, 8)), [], [0, 0])                 # zero partials
    assert np.array_equal(o[0], np.zeros(8)) and l[0] == ninf
    # closed form with weights 1:3
    o, l = oracle.merge([a, b], [0.0, math.log(3.0)], [0, 2])
    assert np.max(np.abs(o[0] - (a + 3 * b) / 4)) < 1e-15 and abs(l[0] - math.log(4.0)) < 1e-15
    # CSR with several rows, one of them empty
    o, l = oracle.merge([a, b, a], [0.0, 0.0, 2.0], [0, 2, 2, 3])
    assert np.max(np.abs(o[0] - (a + b) / 2)) < 1e-15 and l[1] == ninf and np.array_equal(o[2], a)


def test_empty_range_convention():
    w = _one_seq(20)
    o, l = oracle.paged_attn(w.q, w.k_pool, w.v_pool, w.block_table, [5], [5], w.sm_scale, "f32")
    assert np.array_equal(o, np.zeros_like(o)) and np.all(l == -np.inf)
    o, l = oracle.paged_attn(w.q, w.k_pool, w.v_pool, w.block_table, [9], [4], w.sm_scale, "f32")
    assert np.array_equal(o, np.zeros_like(o)) and np.all(l == -np.inf)
