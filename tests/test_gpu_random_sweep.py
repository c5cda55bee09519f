"""GPU parity on seeded random batches: head layouts of both head dims, ragged and empty ranges with and
without an offset, chunkings, hybrid batches with zero to six rows per sequence from elsewhere - each through
every kernel form (grid, persistent, planned list, vector kernel) and every route to the final rows (partials
+ merge, final rows + masked merge, fused), against the CPU fp64 oracle."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2603_12831_amd import binding, workloads as wl
from paper_2603_12831_amd.runner import DeviceWorkload
from test_gpu_parity import TOL, expected_full, ext_partials_from_oracle

pytestmark = pytest.mark.gpu

SHAPES = {128: [(8, 8), (8, 4), (6, 2), (16, 4), (16, 2), (32, 2), (32, 8), (12, 4), (5, 1), (14, 2), (28, 4)],
          64: [(8, 8), (4, 2), (6, 2), (16, 4), (12, 4), (8, 1), (16, 2)]}
FORMS = [(binding.OMNI_KERNEL_AUTO, False), (binding.OMNI_KERNEL_AUTO, True), (binding.OMNI_KERNEL_AUTO, 2),
         (binding.OMNI_KERNEL_VECTOR, False), (binding.OMNI_KERNEL_VECTOR, True)]


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("these tests need a GPU (run with -m gpu on an MI355X box)")
    binding.load_library()


def random_case(rng):
    d = int(rng.choice([128, 128, 64]))
    hq, hkv = SHAPES[d][int(rng.integers(0, len(SHAPES[d])))]
    dtype = "bf16" if rng.random() < 0.8 else "f32"
    batch = int(rng.integers(1, 40))
    lengths = rng.integers(1, [60, 700, 3000][int(rng.integers(0, 3))], size=batch)
    w = wl.make_generic(int(rng.integers(1, 1 << 30)), lengths, hq, hkv, d, dtype=dtype, pool_factor=1.2 + rng.random())
    begin = np.zeros(batch, dtype=np.int32)
    if rng.random() < 0.6:
        begin = (rng.random(batch) * lengths * rng.choice([0.0, 0.5, 0.95])).astype(np.int32)
    end = lengths.astype(np.int32).copy()
    if rng.random() < 0.3:                                 # an empty or a shortened range somewhere
        end[rng.integers(0, batch)] = begin[rng.integers(0, batch)]
        end = np.minimum(np.maximum(end, begin), lengths).astype(np.int32)
    chunk = int(rng.choice([0, 16, 32, 64, 256, 1024]))
    span = int(np.maximum(end - begin, 0).max())
    w.calls = [wl.DecodeCall(begin.copy(), end.copy(), chunk, 1 if chunk == 0 else max(1, (span + chunk - 1) // chunk))]
    ext, exp_begin = (None, None, None), begin
    if rng.random() < 0.4:                                 # hybrid: the tokens in front of `begin` come as rows from elsewhere
        pieces = np.where(begin > 0, rng.integers(0, 7, size=batch), 0)
        if pieces.sum() > 0:
            w.ext_ranges = [[((int(begin[i]) * j) // k, (int(begin[i]) * (j + 1)) // k) for j in range(k)]
                            for i, k in enumerate(int(x) for x in pieces)]
            ext = ext_partials_from_oracle(w)
            exp_begin = np.where(pieces > 0, 0, begin).astype(np.int32)
    return w, ext, expected_full(w, begin=exp_begin, end=end), d, dtype


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_batches_every_form_and_route(seed):
    rng = np.random.default_rng([2603, seed])
    worst = 0.0
    for case in range(60):
        w, ext, exp, d, dtype = random_case(rng)
        fin = np.isfinite(exp[1])
        for kernel in FORMS:
            for mode in ("merge", "final", "fused"):
                if mode == "fused" and not (kernel[1] and d == 128 and dtype == "bf16" and kernel[0] == binding.OMNI_KERNEL_AUTO):
                    continue
                dw = DeviceWorkload(w, out_dtype="f32", ext_o=ext[0], ext_lse=ext[1], ext_offsets=ext[2],
                                    workspace=kernel[1], mode=mode)
                for _ in range(2):
                    dw.poison_outputs()
                    dw.run(kernel=kernel[0])
                o, l = dw.results()
                what = "seed %d case %d: d %d, %d q / %d kv heads, %s, chunk %d, form %s, route %s" % (
                    seed, case, d, w.num_q_heads, w.num_kv_heads, dtype, w.calls[0].chunk_tokens, kernel, mode)
                assert np.array_equal(np.isfinite(l), fin) and np.all(np.isfinite(o)), what
                eo = float(np.max(np.abs(o - exp[0]))) if o.size else 0.0
                el = float(np.max(np.abs(l[fin] - exp[1][fin]))) if fin.any() else 0.0
                assert eo <= TOL[dtype] and el <= TOL[dtype], "%s: max abs err O %.3g LSE %.3g" % (what, eo, el)
                if kernel[1]:
                    assert dw.abandoned_waves() == 0, what
                worst = max(worst, eo / TOL[dtype], el / TOL[dtype])
                del dw
    print("seed %d: worst error / tolerance %.3f" % (seed, worst))
