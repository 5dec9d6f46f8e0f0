"""The input generators: deterministic, sliceable, right shape and range."""
import numpy as np
import torch

import synth


def test_slices_agree_with_whole():
    a = synth.gaussian(3, 0, 100, 16)
    b = synth.gaussian(3, 40, 60, 16)
    assert torch.equal(a[40:60], b)
    assert not torch.equal(synth.gaussian(4, 0, 100, 16), a)
    m = synth.mixture(5, 0, 64, 96, n_comp=10)
    assert torch.equal(m[10:20], synth.mixture(5, 10, 20, 96, n_comp=10))


def test_distributions():
    g = synth.gaussian(1, 0, 4000, 32)
    assert abs(float(g.mean())) < 0.02 and abs(float(g.std()) - 1) < 0.02
    s = synth.sift_like(2, 0, 2000, 128)
    assert float(s.min()) >= 0 and float(s.max()) <= 255 and torch.equal(s, torch.round(s))
    assert 25 < float(s.mean()) < 40
    m = synth.mixture(3, 0, 2000, 96)
    np.testing.assert_allclose(torch.linalg.vector_norm(m, dim=1).numpy(), 1.0, rtol=1e-5)
    shifted = synth.mixture(3, 0, 2000, 96, shift=0.5)
    assert float((m - shifted).abs().mean()) > 0.01


def test_sorted_subset():
    for N, S in ((1000, 0), (1000, 1), (1000, 17), (1000, 499), (1000, 800), (1000, 1000), (10**6, 10**4)):
        s = synth.sorted_subset(9, 2, N, S)
        assert s.dtype == torch.int32 and s.numel() == S
        if S:
            assert int(s.min()) >= 0 and int(s.max()) < N
            assert bool((s[1:] > s[:-1]).all())
    assert not torch.equal(synth.sorted_subset(9, 2, 1000, 17), synth.sorted_subset(9, 3, 1000, 17))
    ids, off = synth.subset_batch(1, 500, [3, 0, 500, 20])
    assert off.tolist() == [0, 3, 3, 503, 523] and ids.numel() == 523
    # roughly uniform: mean of a large subset is near N/2
    big = synth.sorted_subset(4, 0, 10**6, 10**5).double()
    assert abs(float(big.mean()) / 1e6 - 0.5) < 0.01


def test_sample_rows_distinct():
    r = synth.sample_rows(1, 5000, 256)
    assert r.numel() == 256 and len(set(r.tolist())) == 256
