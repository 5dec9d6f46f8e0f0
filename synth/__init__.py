"""Seeded synthetic input generators shared by the tests, the benchmark and the smoke check.

This module produces *inputs only* (database vectors, queries, training samples, target
identifier subsets).  It contains none of the search method's arithmetic: no quantiser, no
distance table, no scan, no selection.  Both the CPU oracle and the HIP library receive the
arrays made here; neither of them is imported here.

Everything is a pure function of (seed, element index): a counter-based generator built from a
64-bit integer mixing function, so any row range of a data set can be produced without
materialising the rest, on the CPU or on the GPU.  The integer stage is bit-identical on every
device; the floating-point stage (logarithm, cosine, normalisation) may differ in the last ulp
between devices, which is why a consumer that needs the same array on the host and on the GPU
generates it once and copies it.

The data sets stand in for the public benchmarks the paper measures on (Sec. 5.1: SIFT1M,
Deep1B), which are not available here; only their shape, value range and cluster structure are
imitated:

* ``gaussian``      i.i.d. N(0,1) vectors.
* ``sift_like``     non-negative integer-valued floats min(255, round(|N(0, 40^2)|)), D = 128.
* ``mixture``       1000-component Gaussian mixture, means N(0, I), sigma 0.3, L2-normalised,
                    D = 96; ``shift > 0`` moves every mean by N(0, shift^2 I) (vectors that arrive
                    after the index was built, Sec. 5.4).
* ``sorted_subset`` strictly increasing uniform random identifier subsets (the task of Sec. 5.3).
"""
from __future__ import annotations

import math

import torch

_M1 = -4658895280553007687  # 0xbf58476d1ce4e5b9 as a signed 64-bit value
_M2 = -7723592293110705685  # 0x94d049bb133111eb
_GOLD = -7046029254386353131  # 0x9e3779b97f4a7c15


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift of an int64 tensor."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix64(x: torch.Tensor) -> torch.Tensor:
    x = (x ^ _lsr(x, 30)) * _M1
    x = (x ^ _lsr(x, 27)) * _M2
    return x ^ _lsr(x, 31)


def _seed_key(seed: int, stream: int) -> int:
    """Scalar key for (seed, stream), computed with Python integers (mod 2^64)."""
    mask = (1 << 64) - 1
    z = (seed * 0x9E3779B97F4A7C15 + stream * 0xD1B54A32D192ED03 + 0x2545F4914F6CDD1D) & mask
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & mask
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & mask
    z ^= z >> 31
    return z - (1 << 64) if z >= (1 << 63) else z


def hash64(seed: int, stream: int, idx: torch.Tensor) -> torch.Tensor:
    """64 pseudo-random bits (as int64) for every element index in ``idx``."""
    return _mix64(_mix64(idx * _GOLD + _seed_key(seed, stream)))


def _uniform24(bits: torch.Tensor) -> torch.Tensor:
    """24-bit integer -> float32 in (0, 1), exact."""
    return (bits.to(torch.float32) + 0.5) * (1.0 / 16777216.0)


def normal_from_index(seed: int, stream: int, idx: torch.Tensor) -> torch.Tensor:
    """Standard normal float32 per element index (Box-Muller on two 24-bit uniforms)."""
    h = hash64(seed, stream, idx)
    u1 = _uniform24(_lsr(h, 40))
    u2 = _uniform24(_lsr(h, 16) & 0xFFFFFF)
    return torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)


def _elem_index(r0: int, r1: int, D: int, device) -> torch.Tensor:
    return torch.arange(r0 * D, r1 * D, dtype=torch.int64, device=device).view(r1 - r0, D)


def gaussian(seed: int, r0: int, r1: int, D: int, device="cpu") -> torch.Tensor:
    """Rows r0..r1-1 of an i.i.d. N(0,1) matrix with D columns (float32)."""
    return normal_from_index(seed, 0, _elem_index(r0, r1, D, device))


def sift_like(seed: int, r0: int, r1: int, D: int = 128, device="cpu") -> torch.Tensor:
    """Rows of a SIFT-shaped matrix: min(255, round(|N(0, 40^2)|)) stored as float32."""
    z = normal_from_index(seed, 0, _elem_index(r0, r1, D, device))
    return torch.clamp(torch.round(torch.abs(z) * 40.0), max=255.0)


def mixture_means(seed: int, n_comp: int, D: int, shift: float = 0.0, device="cpu") -> torch.Tensor:
    """Component means N(0, I); with ``shift`` every mean is moved by N(0, shift^2 I)."""
    mu = normal_from_index(seed, 1, _elem_index(0, n_comp, D, device))
    if shift > 0.0:
        mu = mu + shift * normal_from_index(seed, 3, _elem_index(0, n_comp, D, device))
    return mu


def mixture(seed: int, r0: int, r1: int, D: int = 96, n_comp: int = 1000, sigma: float = 0.3,
            shift: float = 0.0, means_seed: int | None = None, device="cpu") -> torch.Tensor:
    """Rows of a Deep-shaped matrix: Gaussian mixture with uniform weights, L2-normalised.

    ``means_seed`` fixes the component means independently of ``seed`` so that database rows,
    queries and later additions share one mixture."""
    mu = mixture_means(seed if means_seed is None else means_seed, n_comp, D, shift, device)
    rows = torch.arange(r0, r1, dtype=torch.int64, device=device)
    comp = _lsr(hash64(seed, 2, rows), 1) % n_comp
    x = mu[comp] + sigma * normal_from_index(seed, 0, _elem_index(r0, r1, D, device))
    return x / torch.linalg.vector_norm(x, dim=1, keepdim=True)


def sample_rows(seed: int, N: int, n: int, device="cpu") -> torch.Tensor:
    """``n`` distinct row numbers out of N (int64, in a seeded pseudo-random order).

    The first ``n`` positions of the permutation that sorts N hashed keys."""
    if n > N:
        raise ValueError("sample larger than population")
    keys = hash64(seed, 4, torch.arange(N, dtype=torch.int64, device=device))
    return torch.argsort(keys, stable=True)[:n].contiguous()


def sorted_subset(seed: int, query: int, N: int, S: int, device="cpu") -> torch.Tensor:
    """A uniform random S-subset of {0..N-1}, strictly increasing, int32.

    Draw a few more than S identifiers with replacement, drop duplicates (a uniform random set
    of U >= S distinct identifiers), then drop the U-S members whose value hashes smallest:
    a uniformly chosen sub-subset of a uniform set is uniform."""
    if S < 0 or S > N:
        raise ValueError("subset size out of range")
    if S == N:
        return torch.arange(N, dtype=torch.int32, device=device)
    if 2 * S > N:  # sample the complement instead
        comp = sorted_subset(seed, query, N, N - S, device).to(torch.int64)
        keep = torch.ones(N, dtype=torch.bool, device=device)
        keep[comp] = False
        return torch.nonzero(keep).view(-1).to(torch.int32)
    stream = 16 + 2 * query
    extra = 0
    while True:
        expected_dup = S * S / (2.0 * N)
        n_draw = S + int(2 * expected_dup + 8 * math.sqrt(expected_dup + 1) + 16) + extra
        draws = _lsr(hash64(seed, stream, torch.arange(n_draw, dtype=torch.int64, device=device)), 1) % N
        uniq = torch.unique(draws)  # sorted
        U = uniq.numel()
        if U >= S:
            break
        extra += n_draw  # practically never reached
    if U > S:
        drop_key = _lsr(hash64(seed, stream + 1, uniq), 1)  # unsigned order of the hash
        drop = torch.topk(drop_key, U - S, largest=False).indices
        keep = torch.ones(U, dtype=torch.bool, device=device)
        keep[drop] = False
        uniq = uniq[keep]
    return uniq.to(torch.int32)


def _draw_count(N: int, S: int) -> int:
    expected_dup = S * S / (2.0 * N)
    return S + int(2 * expected_dup + 8 * math.sqrt(expected_dup + 1) + 16)


def _sorted_subsets_equal_size(seed: int, q0: int, B: int, N: int, S: int, device) -> torch.Tensor | None:
    """``sorted_subset`` for queries q0..q0+B-1 at once ([B][S] int32), or None if a row came up short."""
    n_draw = _draw_count(N, S)
    idx = torch.arange(n_draw, dtype=torch.int64, device=device)
    key1 = torch.tensor([_seed_key(seed, 16 + 2 * (q0 + b)) for b in range(B)], dtype=torch.int64, device=device)
    key2 = torch.tensor([_seed_key(seed, 17 + 2 * (q0 + b)) for b in range(B)], dtype=torch.int64, device=device)
    draws = _lsr(_mix64(_mix64(idx[None, :] * _GOLD + key1[:, None])), 1) % N
    # one flat sort per step (row number in the high bits) instead of one sort per row
    row = torch.arange(B, dtype=torch.int64, device=device)[:, None]
    vals = (torch.sort(((row << 32) | draws).view(-1)).values & 0xFFFFFFFF).view(B, n_draw)
    dup = torch.zeros_like(vals, dtype=torch.bool)
    dup[:, 1:] = vals[:, 1:] == vals[:, :-1]
    U = (~dup).sum(dim=1)
    if int(U.min()) < S:
        return None
    # the U-S members with the smallest hash are dropped; the comparison uses the top 36 bits
    # of the hash, which selects the same members unless two of them tie exactly at the cut
    # (then the row count check below fails and the caller falls back to sorted_subset)
    big = (1 << 36) - 1
    drop_key = _lsr(_mix64(_mix64(vals * _GOLD + key2[:, None])), 28)
    drop_key = torch.where(dup, torch.full_like(drop_key, big), drop_key)
    ordered = (torch.sort(((row << 36) | drop_key).view(-1)).values & big).view(B, n_draw)
    n_drop = U - S                                  # members to drop per row: the n_drop smallest keys
    thr = torch.where(n_drop > 0, ordered.gather(1, (n_drop - 1).clamp(min=0)[:, None]).squeeze(1),
                      torch.full_like(n_drop, -1))
    keep = (~dup) & (drop_key > thr[:, None])
    if not bool((keep.sum(dim=1) == S).all()):
        return None
    return vals[keep].view(B, S).to(torch.int32)


def subset_batch(seed: int, N: int, sizes, device="cpu", batch: int = 64):
    """Target identifiers for a batch of queries in CSR form.

    ``sizes[i]`` is |S| of query i.  Returns (target_ids int32 [sum sizes], offsets int64 [Q+1]).
    Query i gets ``sorted_subset(seed, i, N, sizes[i])``; equal sizes are produced many queries
    at a time with the same arithmetic."""
    sizes = [int(s) for s in sizes]
    off = torch.zeros(len(sizes) + 1, dtype=torch.int64)
    off[1:] = torch.cumsum(torch.tensor(sizes, dtype=torch.int64), 0)
    ids = torch.empty(int(off[-1]), dtype=torch.int32, device=device)
    Q = len(sizes)
    S = sizes[0] if sizes else 0
    if Q > 1 and all(s == S for s in sizes) and 0 < S < N and 2 * S <= N:
        while batch > 1 and batch * _draw_count(N, S) > (1 << 27):
            batch //= 2
        for q0 in range(0, Q, batch):
            B = min(batch, Q - q0)
            rows = _sorted_subsets_equal_size(seed, q0, B, N, S, device)
            if rows is None:
                rows = torch.stack([sorted_subset(seed, q0 + b, N, S, device) for b in range(B)])
            ids[q0 * S:(q0 + B) * S] = rows.reshape(-1)
        return ids, off.to(device)
    for i, s in enumerate(sizes):
        if s:
            ids[int(off[i]):int(off[i + 1])] = sorted_subset(seed, i, N, s, device)
    return ids, off.to(device)
