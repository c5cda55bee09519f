"""Host-side checks of the persistent form's work-list logic (sort keys, tickets) through the library's
test aids, which run the very functions the kernels use.  No GPU call."""
import ctypes

import numpy as np
import pytest

from paper_2603_12831_amd import binding

SHORT = 256          # ranges up to this many tokens may be dealt out four to a ticket
WAVES = 4


@pytest.fixture(scope="module", autouse=True)
def _lib():
    binding.load_library()


def expected_tickets(n_entries, n_long, hkv, n_wg):
    """The rule, written out: items in list order; the short ones (behind the first n_long entries) go four to
    a ticket if there are at least four per workgroup, otherwise everything is one item per ticket."""
    n_items = n_entries * hkv
    first_short = min(n_long, n_entries) * hkv
    if n_items - first_short < WAVES * n_wg:
        first_short = n_items
    rows, grouped = [], []
    for i in range(first_short):
        rows.append([i] * WAVES)
        grouped.append(False)
    for i in range(first_short, n_items, WAVES):
        rows.append([i + w if i + w < n_items else -1 for w in range(WAVES)])
        grouped.append(True)
    return np.array(rows, dtype=np.int32).reshape(-1, WAVES), np.array(grouped, dtype=bool)


@pytest.mark.parametrize("hkv", [1, 2, 3, 4, 5, 8, 32])
@pytest.mark.parametrize("n_wg", [1, 7, 256])
def test_every_item_is_served_exactly_once(hkv, n_wg):
    rng = np.random.default_rng([80, hkv, n_wg])
    cases = [(0, 0), (1, 0), (1, 1), (5, 9)] + [(int(n), int(rng.integers(0, n + 3))) for n in rng.integers(1, 3000, size=40)]
    cases += [(WAVES * n_wg // hkv + d, 0) for d in (-1, 0, 1) if WAVES * n_wg // hkv + d >= 0]   # around the threshold
    for n_entries, n_long in cases:
        items, grouped = binding.omni_debug_ticket_map(n_entries, n_long, hkv, n_wg)
        exp_items, exp_grouped = expected_tickets(n_entries, n_long, hkv, n_wg)
        assert items.shape == exp_items.shape, (n_entries, n_long)
        assert np.array_equal(items, exp_items) and np.array_equal(grouped, exp_grouped), (n_entries, n_long)
        # stated independently of the model above: a partition of the items
        served = np.concatenate([items[~grouped][:, 0], items[grouped].ravel()])
        served = served[served >= 0]
        assert np.array_equal(np.sort(served), np.arange(n_entries * hkv))
        # one-item tickets first, every wave of such a ticket on the same item
        assert not np.any(grouped[:-1] & ~grouped[1:])
        assert np.all(items[~grouped] == items[~grouped][:, :1])


def test_grouping_needs_four_short_items_per_workgroup():
    for n_wg in (1, 16, 256):
        need = WAVES * n_wg
        _, g = binding.omni_debug_ticket_map(10 + need - 1, 10, 1, n_wg)
        assert not g.any()
        items, g = binding.omni_debug_ticket_map(10 + need, 10, 1, n_wg)
        assert g.sum() == n_wg and not g[:10].any()
        assert items[10].tolist() == [10, 11, 12, 13]


def test_ticket_map_argument_errors():
    lib = binding.load_library()
    n = ctypes.c_uint32(0)
    buf = (ctypes.c_int32 * 64)()
    assert lib.omni_debug_ticket_map(4, 0, 1, 1, None, 64, ctypes.byref(n)) == binding.OMNI_ERR_NULL
    assert lib.omni_debug_ticket_map(4, 0, 1, 1, buf, 64, None) == binding.OMNI_ERR_NULL
    assert lib.omni_debug_ticket_map(4, 0, 0, 1, buf, 64, ctypes.byref(n)) == binding.OMNI_ERR_SHAPE
    assert lib.omni_debug_ticket_map(4, 0, 1, 0, buf, 64, ctypes.byref(n)) == binding.OMNI_ERR_SHAPE
    assert lib.omni_debug_ticket_map(1 << 30, 0, 8, 1, buf, 64, ctypes.byref(n)) == binding.OMNI_ERR_SHAPE
    # a buffer that is too small is not overrun: pairs beyond the capacity stay unwritten
    for i in range(64):
        buf[i] = -7
    assert lib.omni_debug_ticket_map(100, 100, 1, 1, buf, 16, ctypes.byref(n)) == binding.OMNI_OK
    assert n.value == 100 and list(buf[16:]) == [-7] * 48 and buf[0] == 0 and buf[8] == 1


@pytest.mark.parametrize("chunk", [0, 64, 256, 512, 1024, 4096, 65536])
def test_sort_key_orders_ranges_longest_first_and_keeps_short_ones_apart(chunk):
    top = chunk if chunk else 20000
    tokens = np.unique(np.concatenate([np.arange(1, min(top, 700) + 1), np.linspace(1, top, 300).astype(int), [top]]))
    bins = np.array([binding.omni_debug_sort_bin(int(t), chunk) for t in tokens])
    assert bins.min() >= 0 and bins.max() <= 255
    assert np.all(np.diff(bins) <= 0)                                  # more tokens never sort later
    short = tokens <= SHORT
    assert np.array_equal(bins[short], 256 - (tokens[short] + 15) // 16)   # one key per page count
    assert np.all(bins[~short] < 256 - SHORT // 16)                    # every longer range sorts before them
    if chunk > SHORT:
        assert binding.omni_debug_sort_bin(chunk, chunk) == 0          # full chunks come first
    assert binding.omni_debug_sort_bin(0, chunk) == 256 and binding.omni_debug_sort_bin(-5, chunk) == 256
