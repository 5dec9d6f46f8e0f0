"""The query procedure on the library's static scratch array (``rii_query_noalloc``): called
through the C ABI, compared with ``rii_query`` -- the entry point it is a variant of -- to the bar
of the parity tests (identifiers bit-exact, distances bit-identical: the same kernels run), on
two calls in a row of which the second has the smaller input, so that what the first call left
in the array must not show in the second.  Collected last on purpose."""
import numpy as np
import pytest
import torch

import synth
from helpers import t2n

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rii():
    import paper_1808_03969_amd as r
    r.load_library()
    assert torch.cuda.is_available(), "these tests need the GPU"
    return r


def build(rii, N, M, K, seed):
    x = t2n(synth.mixture(1000 + seed, 0, N, 96))
    cb = rii.rii_train_codebooks(x[:4000], M, iters=3, seed=seed)
    codes = rii.rii_encode(cb, x)
    index = rii.Index(cb)
    index.add(codes)
    index.reconfigure(K, iters=1, seed=seed)
    return index


def same(a, b):
    return np.array_equal(t2n(a[0]), t2n(b[0])) and np.array_equal(t2n(a[1]), t2n(b[1]))


@pytest.mark.parametrize("M", [32, 16])
def test_query_noalloc_equals_query_twice_in_a_row(M, rii):
    N, K, R = 120_001, 64, 100
    index = build(rii, N, M, K, seed=40 + M)
    q_big = synth.mixture(2040, 0, 37, 96).cuda()
    q_small = synth.mixture(2041, 0, 3, 96).cuda()
    tid_big, off_big = synth.subset_batch(95, N, [30_000 if i % 2 else 900 for i in range(37)], "cuda")
    tid_small, off_small = synth.subset_batch(96, N, [700, 20_000, 5], "cuda")
    index.set_threshold(5_000)  # both branches of the switch occur in each batch
    L = 4 * (N // K)
    # first call: the larger batch, whole database and target sets
    for args_big, args_small in (
        ((q_big, R), (q_small, 7)),
        ((q_big, R, tid_big, off_big, 30_000), (q_small, 7, tid_small, off_small, 20_000)),
    ):
        ref_big = rii.rii_query(index, *args_big, L=L)
        ref_small = rii.rii_query(index, *args_small, L=L)
        got_big = rii.rii_query_noalloc(index, *args_big, L=L)
        got_small = rii.rii_query_noalloc(index, *args_small, L=L)   # smaller input right behind the larger one
        again_big = rii.rii_query_noalloc(index, *args_big, L=L)
        torch.cuda.synchronize()
        assert same(got_big, ref_big), "first call differs from rii_query"
        assert same(got_small, ref_small), "second, smaller call differs from rii_query"
        assert same(again_big, ref_big)
    # a linear-scan-only handle (no posting lists) and a one-query batch
    plain = rii.Index(np.ascontiguousarray(np.random.default_rng(1).normal(size=(M, 256, 96 // M)).astype(np.float32)))
    plain.add(np.random.default_rng(2).integers(0, 256, size=(50_000, M), dtype=np.uint8))
    a = rii.rii_query_noalloc(plain, q_big, R)
    b = rii.rii_query_noalloc(plain, q_small[:1].contiguous(), 1)
    torch.cuda.synchronize()
    assert same(a, rii.rii_query(plain, q_big, R)) and same(b, rii.rii_query(plain, q_small[:1].contiguous(), 1))


def test_query_noalloc_rejects_what_does_not_fit(rii):
    index = build(rii, 20_000, 32, 16, seed=7)
    Q = 4000  # 4000 tables of 32 KB alone exceed the 64 MB array
    q = synth.mixture(2042, 0, Q, 96).cuda()
    with pytest.raises(rii.RiiError) as e:
        rii.rii_query_noalloc(index, q, 10)
    assert e.value.status == -7
    held = index.info()["device_bytes"]
    ok = rii.rii_query_noalloc(index, q[:100].contiguous(), 10)
    torch.cuda.synchronize()
    assert index.info()["device_bytes"] == held, "the handle's own scratch must not be touched"
    assert same(ok, rii.rii_query(index, q[:100].contiguous(), 10))
