"""Helpers shared by the tests: tiny index construction on the host and result comparison.

None of this is product code.  The index pieces made here (random code books, random coarse
codes) are *data* for the search path; they do not need to be good quantisers.
"""
from __future__ import annotations

import numpy as np
import torch

import synth

RTOL = 1e-5  # bar on fp32 distances (relative)


def codebooks_from_rows(x: np.ndarray, M: int, Z: int = 256, seed: int = 7) -> np.ndarray:
    """Code books made of Z distinct data rows per sub-space: cb [M][Z][Ds]."""
    n, D = x.shape
    Ds = D // M
    rows = synth.sample_rows(seed, n, Z).numpy()
    return np.ascontiguousarray(x[rows].reshape(Z, M, Ds).transpose(1, 0, 2)).astype(np.float32)


def decode_np(cb: np.ndarray, codes: np.ndarray) -> np.ndarray:
    """Concatenate the selected code words (float64), written with numpy fancy indexing."""
    M = cb.shape[0]
    return np.concatenate([cb[m][codes[:, m]] for m in range(M)], axis=1).astype(np.float64)


def brute_force_sqdist(q: np.ndarray, xhat: np.ndarray) -> np.ndarray:
    """||q - xhat_n||^2 in float64 for every row."""
    diff = xhat - q.astype(np.float64)[None, :]
    return np.einsum("nd,nd->n", diff, diff)


def check_topk(ids, dist, ref_ids, ref_dist, dist_of_id=None, rtol=RTOL, exact_ids=True):
    """Compare a top-R result with a reference one.

    Distances must agree within ``rtol`` position by position.  Identifiers must be identical,
    except that where neighbouring reference distances tie within ``rtol`` any order (and, at
    the R-th boundary, any member of the tie) is accepted when ``exact_ids`` is False; then
    every returned id must be distinct and, if ``dist_of_id`` is given, carry its own distance.
    """
    ids, dist, ref_ids, ref_dist = map(np.asarray, (ids, dist, ref_ids, ref_dist))
    assert ids.shape == ref_ids.shape and dist.shape == ref_dist.shape
    fin = np.isfinite(ref_dist)
    assert np.array_equal(np.isfinite(dist), fin), "padding differs"
    assert np.all(ids[~fin] == -1) and np.all(ref_ids[~fin] == -1)
    np.testing.assert_allclose(dist[fin], ref_dist[fin], rtol=rtol, atol=0)
    assert np.all(np.diff(dist[fin]) >= 0), "not sorted by distance"
    if exact_ids:
        assert np.array_equal(ids, ref_ids), f"ids differ: {ids[:8]} vs {ref_ids[:8]}"
        return
    assert len(set(ids[fin].tolist())) == int(fin.sum()), "duplicate ids"
    if dist_of_id is not None:
        np.testing.assert_allclose(dist[fin], dist_of_id(ids[fin]), rtol=rtol, atol=0)
    bad = np.nonzero(ids != ref_ids)[0]
    for i in bad:
        # a mismatch is allowed only inside a run of (near-)equal reference distances
        lo = ref_dist[i] * (1 - 2 * rtol)
        hi = ref_dist[i] * (1 + 2 * rtol)
        tied = (ref_dist >= lo) & (ref_dist <= hi)
        assert tied.sum() > 1 or i == len(ref_ids) - 1, f"id mismatch at rank {i} without a tie"


def lex_topk(d: np.ndarray, ids: np.ndarray, R: int):
    """R smallest by (distance, id) with numpy's lexsort; padded with -1 / inf."""
    order = np.lexsort((ids, d))[:R]
    out_i = np.full(R, -1, dtype=np.int32)
    out_d = np.full(R, np.inf, dtype=d.dtype)
    out_i[: len(order)] = ids[order]
    out_d[: len(order)] = d[order]
    return out_i, out_d


def t2n(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy()
